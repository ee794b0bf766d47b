// Two layers in one launch, the first layer's output never leaving the chip (Section 6.4: the
// pooling results of a thread block can feed the next convolution layer out of shared memory when one
// block computes them all; procedure step 4 of Section 5.1 then needs no trip through global memory).
//
// One workgroup per image.  The image, both filter tensors (transposed to [column][filter], so that
// lanes = filters read consecutive words) and the intermediate map live in LDS; that bounds the shapes
// this applies to (LeNet-sized pairs: conv 5x5 1->20 on 28x28 + pooling, then conv 5x5 20->50 + pooling).
// Both layers run the same window loop: a wavefront takes one output position (one pooling window when
// the layer pools) and 64 filters; it compacts the window's columns 64 at a time with ballot(x != 0), in
// the scan order of Algorithm 1 (channel, kernel row, kernel column), and multiplies only the nonzero
// ones with the 64 filters' values of their column (Algorithm 2's row product).
// ReLU, the optional bias and the optional max over the pooling window follow in registers
// (Algorithm 4's reduction); the first layer stores to LDS, the second to global memory.
#include "sconv_internal.h"

namespace sconv {

namespace {

constexpr int kPairThreads = 1024;
constexpr int kPairWaves = kPairThreads / 64;

struct PairCfg {
    int Kp1, Kp2;             // filters padded to whole wavefronts
    int MH, MW;               // the intermediate map (first layer's stored output)
    int off_w1, off_mid, off_w2;   // LDS offsets in floats (the image starts at 0)
};

// w[K][L] (global) -> wt[L][Kp] (LDS), zero for filters past K
__device__ __forceinline__ void stage_filters(const float* __restrict__ w, int K, int L, int Kp, float* wt, int tid)
{
    for (int i = tid; i < Kp * L; i += kPairThreads) {
        const int k = i / L, col = i - k * L;      // consecutive threads: consecutive words of one filter
        wt[col * Kp + k] = k < K ? w[(size_t)k * L + col] : 0.0f;
    }
}

// One layer out of LDS: in[C][H][W], wt[L][Kp].  Output [K][PH or OH][PW or OW] to out_lds and / or out_glob.
//
// The window's L = C*R*S columns are taken 64 at a time, one per lane, in the scan order of Algorithm 1:
// every lane fetches the element its column has in this window (zero for a tap in the padding or a column
// past L), ballot(x != 0) is the compaction - the set bits, in ascending order, are the (value, column)
// pairs the scan would have appended - and the wavefront then walks only those: value broadcast from its
// lane, the 64 filters' values of that column from LDS, one multiply-add per lane.  Four pairs are fetched
// before their products are issued, so the LDS reads overlap.
__device__ __forceinline__ void layer_from_lds(const Problem& p, bool pooled, const float* in, const float* wt, int Kp,
                                               float* out_lds, float* __restrict__ out_glob, float* __restrict__ copy_glob,
                                               int wave, int lane)
{
    const int OHs = pooled ? p.PH : p.OH, OWs = pooled ? p.PW : p.OW;
    const int npos = OHs * OWs, kblocks = Kp / 64;
    const int wh = pooled ? p.ph : 1, ww = pooled ? p.pw : 1, ws = pooled ? p.ps : 1;
    const int RS = p.R * p.S;
    for (int item = wave; item < npos * kblocks; item += kPairWaves) {
        const int kb = item / npos, pos = item - kb * npos;
        const int oy = pos / OWs, ox = pos - oy * OWs;
        const int k = kb * 64 + lane;
        const float* wk = wt + k;
        float m = -INFINITY;
        for (int py = 0; py < wh; ++py)
            for (int px = 0; px < ww; ++px) {
                const int ih0 = (oy * ws + py) * p.stride - p.pad, iw0 = (ox * ws + px) * p.stride - p.pad;
                float acc = 0.0f;
                for (int cb = 0; cb < p.L; cb += 64) {
                    const int col = cb + lane;
                    const int c = col / RS, rem = col - c * RS;
                    const int r = rem / p.S, sx = rem - r * p.S;
                    const int ih = ih0 + r, iw = iw0 + sx;
                    const bool ok = col < p.L && ih >= 0 && ih < p.H && iw >= 0 && iw < p.W;
                    const float xv = ok ? in[(c * p.H + ih) * p.W + iw] : 0.0f;
                    unsigned long long mask = __ballot(xv != 0.0f);
                    while (mask) {
                        // up to four nonzeros of the window; a missing one repeats the first with value 0
                        int bit[4];
                        float v[4], wv[4];
                        bit[0] = __builtin_ctzll(mask);
                        mask &= mask - 1;
#pragma unroll
                        for (int j = 1; j < 4; ++j) {
                            const bool have = mask != 0;
                            bit[j] = have ? __builtin_ctzll(mask) : -1;
                            if (have) mask &= mask - 1;
                        }
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const int bj = bit[j] < 0 ? bit[0] : bit[j];
                            const float t = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(xv), bj));
                            v[j] = bit[j] < 0 ? 0.0f : t;
                            wv[j] = wk[(cb + bj) * Kp];
                        }
#pragma unroll
                        for (int j = 0; j < 4; ++j) acc = fmaf(v[j], wv[j], acc);
                    }
                }
                m = fmaxf(m, acc);
            }
        if (k < p.K) {
            float v = m + bias_of(p, (size_t)k);
            if (p.relu) v = fmaxf(v, 0.0f);
            if (out_lds) out_lds[(size_t)k * npos + pos] = v;
            if (out_glob) out_glob[(size_t)k * npos + pos] = v;
            if (copy_glob) copy_glob[(size_t)k * npos + pos] = v;
        }
    }
}

__global__ __launch_bounds__(kPairThreads) void pair_kernel(Problem p1, int pooled1, Problem p2, int pooled2, PairCfg cfg,
                                                            const float* __restrict__ x, const float* __restrict__ w1,
                                                            const float* __restrict__ w2, float* __restrict__ mid_out,
                                                            float* __restrict__ y)
{
    extern __shared__ __align__(16) float lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = blockIdx.x;
    float* img = lds;
    float* wt1 = lds + cfg.off_w1;
    float* mid = lds + cfg.off_mid;
    float* wt2 = lds + cfg.off_w2;

    const int in_elems = p1.C * p1.H * p1.W;
    const float* xn = x + (size_t)n * in_elems;
    for (int i = tid; i < in_elems; i += kPairThreads) img[i] = xn[i];
    stage_filters(w1, p1.K, p1.L, cfg.Kp1, wt1, tid);
    stage_filters(w2, p2.K, p2.L, cfg.Kp2, wt2, tid);
    __syncthreads();

    const int mid_elems = p1.K * cfg.MH * cfg.MW;
    layer_from_lds(p1, pooled1 != 0, img, wt1, cfg.Kp1, mid, nullptr,
                   mid_out ? mid_out + (size_t)n * mid_elems : nullptr, wave, lane);
    __syncthreads();

    const int out_elems = p2.K * (pooled2 ? p2.PH * p2.PW : p2.OH * p2.OW);
    layer_from_lds(p2, pooled2 != 0, mid, wt2, cfg.Kp2, nullptr, y + (size_t)n * out_elems, nullptr, wave, lane);
}

}  // namespace

int launch_pair(const Problem& p1, bool pooled1, const Problem& p2, bool pooled2, const float* x, const float* w1,
                const float* w2, float* mid_out, float* y, hipStream_t stream)
{
    if (p1.G != 1 || p2.G != 1) return SCONV_EUNSUPPORTED;
    PairCfg cfg;
    cfg.Kp1 = (p1.K + 63) / 64 * 64;
    cfg.Kp2 = (p2.K + 63) / 64 * 64;
    cfg.MH = pooled1 ? p1.PH : p1.OH;
    cfg.MW = pooled1 ? p1.PW : p1.OW;
    if (p2.N != p1.N || p2.C != p1.K || p2.H != cfg.MH || p2.W != cfg.MW) return SCONV_EINVAL;
    const long long img = (long long)p1.C * p1.H * p1.W, w1f = (long long)p1.L * cfg.Kp1,
                    midf = (long long)p1.K * cfg.MH * cfg.MW, w2f = (long long)p2.L * cfg.Kp2;
    const long long total = img + w1f + midf + w2f;
    if (total * 4 > 160 * 1024) return SCONV_EUNSUPPORTED;    // the pair does not fit one workgroup's LDS
    cfg.off_w1 = (int)img;
    cfg.off_mid = (int)(img + w1f);
    cfg.off_w2 = (int)(img + w1f + midf);
    const size_t lds_bytes = (size_t)total * 4;
    static size_t opted = 48 * 1024;   // under the dispatcher's lock
    if (lds_bytes > opted) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(pair_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds_bytes) != hipSuccess)
            return SCONV_ELAUNCH;
        opted = lds_bytes;
    }
    hipLaunchKernelGGL(pair_kernel, dim3((unsigned)p1.N), dim3(kPairThreads), lds_bytes, stream, p1, pooled1 ? 1 : 0, p2,
                       pooled2 ? 1 : 0, cfg, x, w1, w2, mid_out, y);
    return launch_status();
}

}  // namespace sconv

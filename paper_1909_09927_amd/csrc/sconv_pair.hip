// Two layers in one launch, the first layer's output never leaving the chip (Section 6.4: the
// pooling results of a thread block can feed the next convolution layer out of shared memory when one
// block computes them all; procedure step 4 of Section 5.1 then needs no trip through global memory).
//
// One workgroup per image.  The image, both filter tensors (transposed to [column][filter], so that
// lanes = filters read consecutive words) and the intermediate map live in LDS; that bounds the shapes
// this applies to (LeNet-sized pairs: conv 5x5 1->20 on 28x28 + pooling, then conv 5x5 20->50 + pooling).
// Both layers run the same window loop: a wavefront takes one output position (one pooling window when
// the layer pools) and 64 filters; it walks the window's columns in the scan order of Algorithm 1
// (channel, kernel row, kernel column), reads each element once for all lanes - a broadcast LDS read, so
// the test `x != 0` is the same for the whole wavefront and a zero costs one scalar branch - and
// multiplies the nonzero ones with the 64 filters' values of that column (Algorithm 2's row product).
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
__device__ __forceinline__ void layer_from_lds(const Problem& p, bool pooled, const float* in, const float* wt, int Kp,
                                               float* out_lds, float* __restrict__ out_glob, float* __restrict__ copy_glob,
                                               int wave, int lane)
{
    const int OHs = pooled ? p.PH : p.OH, OWs = pooled ? p.PW : p.OW;
    const int npos = OHs * OWs, kblocks = Kp / 64;
    const int wh = pooled ? p.ph : 1, ww = pooled ? p.pw : 1, ws = pooled ? p.ps : 1;
    for (int item = wave; item < npos * kblocks; item += kPairWaves) {
        const int kb = item / npos, pos = item - kb * npos;
        const int oy = pos / OWs, ox = pos - oy * OWs;
        const int k = kb * 64 + lane;
        float m = -INFINITY;
        for (int py = 0; py < wh; ++py)
            for (int px = 0; px < ww; ++px) {
                const int oh = oy * ws + py, ow = ox * ws + px;
                float acc = 0.0f;
                for (int c = 0; c < p.C; ++c)
                    for (int r = 0; r < p.R; ++r) {
                        const int ih = oh * p.stride - p.pad + r;
                        if (ih < 0 || ih >= p.H) continue;          // padding rows hold no nonzero
                        for (int s = 0; s < p.S; ++s) {
                            const int iw = ow * p.stride - p.pad + s;
                            if (iw < 0 || iw >= p.W) continue;
                            // the same word for every lane: one broadcast read, a uniform test
                            const float v = __int_as_float(__builtin_amdgcn_readfirstlane(
                                __float_as_int(in[(c * p.H + ih) * p.W + iw])));
                            if (v != 0.0f) acc = fmaf(v, wt[((c * p.R + r) * p.S + s) * Kp + k], acc);
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

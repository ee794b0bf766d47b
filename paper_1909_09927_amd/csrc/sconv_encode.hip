// Materialising format conversion: Algorithm 1 (ECR) / Algorithm 3 (PECR) with the channel loop
// of Section 7 outside.  One wavefront owns one window row.  The 64 lanes take 64 consecutive
// columns (c, r, s ascending, the paper's scan order), so the rank of a lane among the lanes
// that hold a nonzero (ballot + population count of the lower lanes) is exactly the slot the
// sequential scan would have used; the running count carries over to the next 64 columns.
#include "sconv_internal.h"

namespace sconv {

namespace {

constexpr int kEncodeBlock = 256;  // 4 wavefronts = 4 rows per workgroup

__device__ __forceinline__ unsigned lanes_below(unsigned long long mask, int lane)
{
    return __popcll(mask & ((1ull << lane) - 1ull));
}

__global__ __launch_bounds__(kEncodeBlock) void encode_kernel(Problem p, int pecr, long long rows,
                                                              const float* __restrict__ x,
                                                              float* __restrict__ values,
                                                              int32_t* __restrict__ index,
                                                              int32_t* __restrict__ count)
{
    const int lane = threadIdx.x & 63;
    const long long row = (long long)blockIdx.x * (kEncodeBlock / 64) + (threadIdx.x >> 6);
    if (row >= rows) return;  // whole wavefront leaves together

    // row -> (n, g, oh, ow)
    int oh, ow;
    long long ng;
    if (!pecr) {
        long long q = row;
        ow = (int)(q % p.OW); q /= p.OW;
        oh = (int)(q % p.OH); q /= p.OH;
        ng = q;
    } else {
        long long q = row;
        int px = (int)(q % p.pw); q /= p.pw;
        int py = (int)(q % p.ph); q /= p.ph;
        int pwi = (int)(q % p.PW); q /= p.PW;
        int phi = (int)(q % p.PH); q /= p.PH;
        ng = q;
        oh = phi * p.ps + py;
        ow = pwi * p.ps + px;
    }
    const int g = (int)(ng % p.G);
    const int n = (int)(ng / p.G);
    const int ih0 = oh * p.stride - p.pad;
    const int iw0 = ow * p.stride - p.pad;
    const float* xg = x + ((long long)n * p.C + (long long)g * p.Cg) * p.H * p.W;

    // this lane's first column, split into (c, r, s); then steps of 64 columns with carries
    const int RS = p.R * p.S;
    int c = lane / RS;
    int rs = lane - c * RS;
    int r = rs / p.S;
    int s = rs - r * p.S;
    const int dc = 64 / RS;
    const int drs = 64 - dc * RS;
    const int dr = drs / p.S;
    const int ds = drs - dr * p.S;

    float* vrow = values + row * p.L;
    int32_t* irow = index + row * p.L;

    // The compacted (value, column) pairs pass through a 128-slot ring in LDS (one per wavefront)
    // and leave it 64 at a time, so every store to HBM is one whole run of 64 consecutive slots
    // of the row instead of a ragged piece per 64 columns.
    __shared__ float ring_v[kEncodeBlock / 64][128];
    __shared__ int32_t ring_i[kEncodeBlock / 64][128];
    float* rv = ring_v[threadIdx.x >> 6];
    int32_t* ri = ring_i[threadIdx.x >> 6];

    int cnt = 0;       // nonzeros found so far (wavefront-uniform)
    int flushed = 0;   // slots of the row already stored (a multiple of 64)
    constexpr int UN = 4;   // column groups loaded together before any of them is ranked
    for (int col0 = 0; col0 < p.L; col0 += 64 * UN) {
        float v[UN];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int col = col0 + 64 * u + lane;
            v[u] = 0.0f;
            if (col < p.L) {
                const int ih = ih0 + r, iw = iw0 + s;
                if (ih >= 0 && ih < p.H && iw >= 0 && iw < p.W)
                    v[u] = xg[((long long)c * p.H + ih) * p.W + iw];
            }
            s += ds;
            if (s >= p.S) { s -= p.S; r += 1; }
            r += dr;
            if (r >= p.R) { r -= p.R; c += 1; }
            c += dc;
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const bool nz = v[u] != 0.0f;  // +0, -0 dropped; denormals, negatives kept
            const unsigned long long mask = __ballot(nz);
            if (nz) {
                const int slot = (cnt + lanes_below(mask, lane)) & 127;
                rv[slot] = v[u];
                ri[slot] = col0 + 64 * u + lane;
            }
            cnt += __popcll(mask);
            __builtin_amdgcn_wave_barrier();
            if (cnt - flushed >= 64) {   // at most 127 pairs are pending: one run leaves
                const int slot = (flushed + lane) & 127;
                vrow[flushed + lane] = rv[slot];
                irow[flushed + lane] = ri[slot];
                flushed += 64;
                __builtin_amdgcn_wave_barrier();
            }
        }
    }
    // what is left in the ring, then zeros up to the end of the row
    for (int slot = flushed + lane; slot < p.L; slot += 64) {
        const bool live = slot < cnt;
        vrow[slot] = live ? rv[slot & 127] : 0.0f;
        irow[slot] = live ? ri[slot & 127] : 0;
    }
    if (lane == 0) count[row] = (!pecr && cnt == 0) ? -1 : cnt;
}

}  // namespace

int launch_encode(const Problem& p, int fmt, const float* x, float* values, int32_t* index,
                  int32_t* count, hipStream_t stream)
{
    long long rows = (long long)p.N * p.G;
    rows *= fmt == SCONV_FMT_ECR ? (long long)p.OH * p.OW : (long long)p.PH * p.PW * p.ph * p.pw;
    if (rows == 0) return SCONV_OK;
    const long long blocks = (rows + kEncodeBlock / 64 - 1) / (kEncodeBlock / 64);
    if (blocks >= (1ll << 31)) return SCONV_EUNSUPPORTED;
    hipLaunchKernelGGL(encode_kernel, dim3((unsigned)blocks), dim3(kEncodeBlock), 0, stream, p,
                       fmt == SCONV_FMT_PECR ? 1 : 0, rows, x, values, index, count);
    return launch_status();
}

}  // namespace sconv

// Materialising format conversion: Algorithm 1 (ECR) / Algorithm 3 (PECR) with the channel loop
// of Section 7 outside.  One wavefront owns one window row.  The 64 lanes take 64 consecutive
// columns (c, r, s ascending, the paper's scan order), so the rank of a lane among the lanes
// that hold a nonzero (ballot + population count of the lower lanes) is exactly the slot the
// sequential scan would have used; the running count carries over to the next 64 columns.
#include <stdlib.h>
#include <string.h>

#include <algorithm>

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


// Tiled form of the same conversion.  A workgroup takes TR consecutive rows of one (image, group):
// their windows overlap (neighbouring outputs share all but one column of taps) and lie in a small
// box of the map, so the box is read once per workgroup - contiguous runs along the width, staged
// in LDS a chunk of channels at a time - instead of once per window in pieces of S elements (a
// 3x3 window row touches 21 cache lines per 64 columns; a 1x1 row 64).  Each wavefront then scans
// its row out of LDS exactly as above; the row's ring and counts persist across the channel chunks.
constexpr int kTileBlock = 1024;       // 16 wavefronts: TR / 16 rows each
constexpr int STAGE = 4096;            // staged input elements per chunk (16 KB)
constexpr int PER_THREAD = STAGE / kTileBlock;

// TR rows per workgroup: 16 (one per wavefront), or 32 for 1x1 layers, whose rows are short (256-512
// columns): the set-up of a tile and its three barriers then serve twice the output, and a channel's box is
// a run of 32 positions (a whole 128-byte line) instead of 16.
template <int TR>
__global__ __launch_bounds__(kTileBlock) void encode_tile_kernel(Problem p, int pecr, int rows_per_ng,
                                                                   int tiles_per_ng, const float* __restrict__ x,
                                                                   float* __restrict__ values,
                                                                   int32_t* __restrict__ index,
                                                                   int32_t* __restrict__ count)
{
    __shared__ float stage[STAGE];          // [channel of the chunk][box row][box column]
    __shared__ int32_t box_off[STAGE];      // box element -> offset in a channel plane, -1 outside the map
    __shared__ float ring_v[TR][128];
    __shared__ int32_t ring_i[TR][128];
    __shared__ int s_ih0[TR], s_iw0[TR];
    constexpr int RPW = TR / (kTileBlock / 64);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ng = blockIdx.x / tiles_per_ng;
    const int tile = blockIdx.x - ng * tiles_per_ng;
    const int g = ng % p.G, n = ng / p.G;
    const int rl0 = tile * TR;                              // first row of the tile inside (n, g)
    const int nrows = min(TR, rows_per_ng - rl0);
    const int HWp = p.H * p.W;

    // window origins of the tile's rows
    if (tid < TR) {
        int oh = 0, ow = 0;
        const int q0 = rl0 + min(tid, nrows - 1);           // rows past the end repeat the last one
        if (!pecr) {
            oh = q0 / p.OW;
            ow = q0 - oh * p.OW;
        } else {
            int q = q0;
            const int px = q % p.pw; q /= p.pw;
            const int py = q % p.ph; q /= p.ph;
            const int pwi = q % p.PW;
            const int phi = q / p.PW;
            oh = phi * p.ps + py;
            ow = pwi * p.ps + px;
        }
        s_ih0[tid] = oh * p.stride - p.pad;
        s_iw0[tid] = ow * p.stride - p.pad;
    }
    __syncthreads();
    int ih_min = s_ih0[0], ih_max = s_ih0[0], iw_min = s_iw0[0], iw_max = s_iw0[0];
    for (int i = 1; i < nrows; ++i) {
        ih_min = min(ih_min, s_ih0[i]); ih_max = max(ih_max, s_ih0[i]);
        iw_min = min(iw_min, s_iw0[i]); iw_max = max(iw_max, s_iw0[i]);
    }
    const int BH = ih_max - ih_min + p.R, BW = iw_max - iw_min + p.S;
    const int plane = BH * BW;                               // the host made sure it fits STAGE
    for (int pe = tid; pe < plane; pe += kTileBlock) {
        const int bh = pe / BW, bw = pe - bh * BW;
        const int ih = ih_min + bh, iw = iw_min + bw;
        box_off[pe] = (ih >= 0 && ih < p.H && iw >= 0 && iw < p.W) ? ih * p.W + iw : -1;
    }
    const int CC = min(p.Cg, STAGE / plane);                 // channels per chunk
    const unsigned magic = plane > 1 ? (unsigned)((1ull << 32) / (unsigned)plane) + 1u : 0u;
    const float* xg = x + ((long long)n * p.C + (long long)g * p.Cg) * HWp;
    __syncthreads();

    // this lane's first column of a chunk, split into (c, r, s); then steps of 64 columns
    const int RS = p.R * p.S;
    const int c_first = lane / RS;
    const int rs_first = lane - c_first * RS;
    const int r_first = rs_first / p.S;
    const int s_first = rs_first - r_first * p.S;
    const int dc = 64 / RS;
    const int drs = 64 - dc * RS;
    const int dr = drs / p.S;
    const int ds = drs - dr * p.S;

    int cnt[RPW], flushed[RPW];
#pragma unroll
    for (int j = 0; j < RPW; ++j) cnt[j] = flushed[j] = 0;

    // loads of one chunk: element e of the staged block is channel e / plane, box element e % plane
    float pre[PER_THREAD];
    auto fetch = [&](int c0) {
        const int lim = min(CC, p.Cg - c0) * plane;
#pragma unroll
        for (int k = 0; k < PER_THREAD; ++k) {
            const int e = k * kTileBlock + tid;
            pre[k] = 0.0f;
            if (e < lim) {
                const int c = magic ? (int)__umulhi((unsigned)e, magic) : e;
                const int off = box_off[e - c * plane];
                if (off >= 0) pre[k] = xg[(long long)(c0 + c) * HWp + off];
            }
        }
    };
    fetch(0);
    for (int c0 = 0; c0 < p.Cg; c0 += CC) {
        const int ccur = min(CC, p.Cg - c0);
#pragma unroll
        for (int k = 0; k < PER_THREAD; ++k) stage[k * kTileBlock + tid] = pre[k];
        __syncthreads();
        if (c0 + CC < p.Cg) fetch(c0 + CC);
        const int ncols = ccur * RS;                         // columns of this chunk
#pragma unroll
        for (int j = 0; j < RPW; ++j) {
            const int rr = wave * RPW + j;
            if (rr >= nrows) continue;
            const int boff = (s_ih0[rr] - ih_min) * BW + (s_iw0[rr] - iw_min);
            float* rv = ring_v[rr];
            int32_t* ri = ring_i[rr];
            float* vrow = values + ((long long)ng * rows_per_ng + rl0 + rr) * p.L;
            int32_t* irow = index + ((long long)ng * rows_per_ng + rl0 + rr) * p.L;
            int c = c_first, r = r_first, s = s_first;
            for (int lc0 = 0; lc0 < ncols; lc0 += 64) {
                const int lc = lc0 + lane;
                const float v = lc < ncols ? stage[c * plane + boff + r * BW + s] : 0.0f;
                const bool nz = v != 0.0f;  // +0, -0 dropped; denormals, negatives kept
                const unsigned long long mask = __ballot(nz);
                if (nz) {
                    const int slot = (cnt[j] + lanes_below(mask, lane)) & 127;
                    rv[slot] = v;
                    ri[slot] = c0 * RS + lc;
                }
                cnt[j] += __popcll(mask);
                __builtin_amdgcn_wave_barrier();
                if (cnt[j] - flushed[j] >= 64) {
                    const int slot = (flushed[j] + lane) & 127;
                    vrow[flushed[j] + lane] = rv[slot];
                    irow[flushed[j] + lane] = ri[slot];
                    flushed[j] += 64;
                    __builtin_amdgcn_wave_barrier();
                }
                s += ds;
                if (s >= p.S) { s -= p.S; r += 1; }
                r += dr;
                if (r >= p.R) { r -= p.R; c += 1; }
                c += dc;
            }
        }
        __syncthreads();   // the staged chunk is free again
    }
#pragma unroll
    for (int j = 0; j < RPW; ++j) {
        const int rr = wave * RPW + j;
        if (rr >= nrows) continue;
        const long long row = (long long)ng * rows_per_ng + rl0 + rr;
        float* vrow = values + row * p.L;
        int32_t* irow = index + row * p.L;
        for (int slot = flushed[j] + lane; slot < p.L; slot += 64) {
            const bool live = slot < cnt[j];
            vrow[slot] = live ? ring_v[rr][slot & 127] : 0.0f;
            irow[slot] = live ? ring_i[rr][slot & 127] : 0;
        }
        if (lane == 0) count[row] = (!pecr && cnt[j] == 0) ? -1 : cnt[j];
    }
}

}  // namespace

int launch_encode(const Problem& p, int fmt, const float* x, float* values, int32_t* index,
                  int32_t* count, hipStream_t stream)
{
    const bool pecr = fmt == SCONV_FMT_PECR;
    const long long rows_per_ng = pecr ? (long long)p.PH * p.PW * p.ph * p.pw : (long long)p.OH * p.OW;
    const long long rows = (long long)p.N * p.G * rows_per_ng;
    if (rows == 0) return SCONV_OK;
    // Measured: staging pays on large maps (56x56: 1.2-1.45x; the window-per-wavefront kernel's
    // pieces of S elements then miss the caches) and on 1x1 layers with long channel loops; on maps
    // of 28x28 and below the plain kernel's gathers hit the caches and its lack of barriers wins
    // (1.05-1.4x).
    const bool large_map = (long long)p.H * p.W >= 2048;
    const bool long_1x1 = p.R == 1 && p.S == 1 && (long long)p.H * p.W >= 196 && p.Cg >= 384;
    bool tiled = large_map || long_1x1;
    if (const char* pin = env_value("SCONV_ENCODE"))   // tuning aid and tests: "tile" or "rows"
        tiled = !strcmp(pin, "tile");
    // The tiled kernel needs the box of a tile's windows to fit its staging buffer.  The rows of a
    // tile are consecutive: in ECR order they span at most (TR-1)/OW + 2 output rows, in PECR order
    // (TR-1)/(ph*pw*PW) + 2 rows of pooling windows; the box is never wider than the padded map.
    auto try_tiled = [&](int TR, auto kernel) -> int {
        const long long span_oh = pecr ? (long long)((TR - 1) / ((long long)p.ph * p.pw * p.PW) + 1) * p.ps + p.ph - 1
                                       : (long long)(TR - 1) / p.OW + 1;
        const long long bh_max = std::min<long long>(span_oh, p.OH - 1) * p.stride + p.R;
        const long long bw_max = std::min<long long>((long long)(p.OW - 1) * p.stride + p.S, p.W + 2LL * p.pad);
        const long long tiles_per_ng = (rows_per_ng + TR - 1) / TR;
        const long long tiles = tiles_per_ng * p.N * p.G;
        if (bh_max * bw_max > STAGE || tiles >= (1ll << 31) || rows_per_ng >= (1ll << 31)) return SCONV_EUNSUPPORTED;
        hipLaunchKernelGGL(kernel, dim3((unsigned)tiles), dim3(kTileBlock), 0, stream, p, pecr ? 1 : 0,
                           (int)rows_per_ng, (int)tiles_per_ng, x, values, index, count);
        return launch_status();
    };
    if (tiled) {
        int rc = SCONV_EUNSUPPORTED;
        if (p.R == 1 && p.S == 1 && !env_value("SCONV_ENCODE_TR16")) rc = try_tiled(32, encode_tile_kernel<32>);
        if (rc == SCONV_EUNSUPPORTED) rc = try_tiled(16, encode_tile_kernel<16>);
        if (rc != SCONV_EUNSUPPORTED) return rc;
    }
    const long long blocks = (rows + kEncodeBlock / 64 - 1) / (kEncodeBlock / 64);
    if (blocks >= (1ll << 31)) return SCONV_EUNSUPPORTED;
    hipLaunchKernelGGL(encode_kernel, dim3((unsigned)blocks), dim3(kEncodeBlock), 0, stream, p, pecr ? 1 : 0, rows, x,
                       values, index, count);
    return launch_status();
}

}  // namespace sconv

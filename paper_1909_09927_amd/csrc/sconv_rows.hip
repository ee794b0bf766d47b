// General window-row kernel: the structure of Sections 5 and 6 carried to many channels,
// filters and images, for any kernel size, stride, padding, grouping and pooling window.
//
// A workgroup (4 wavefronts) owns WA window rows of one (image, group) and KT = 64*KPL filters
// of that group; every wavefront owns a quarter of the window rows and all KT filters (a lane
// holds KPL filters, 64 apart).  The L = Cg*R*S columns of the rows are walked in chunks of CK
// columns, software-pipelined: while a chunk is multiplied, the next chunk's filters and
// activations are already on their way from HBM/L2 into registers.  Per chunk:
//   1. the filter tile w[k][chunk] is written to LDS transposed to [column][k], so that the 64
//      lanes of a wavefront (64 consecutive filters) read one column without bank conflicts;
//   2. the dense chunk of the window rows is loaded with lanes across windows: for one column
//      (c, r, s) consecutive windows read consecutive addresses of the NCHW map (Section 5.3,
//      Fig. 5), zero padding reads as zero;
//   3. every wavefront converts its own window rows on chip: it scans the chunk's columns 64 at
//      a time (ascending c, r, s), and ballot + population count of the lower lanes give each
//      nonzero its slot in the row's compacted list in LDS (value, column) - Algorithm 1 /
//      Algorithm 3 at wavefront level; zeros are never emitted;
//   4. the sparse product of Algorithm 2: for every stored nonzero of a row (the same for all
//      lanes) each lane multiplies by its own filters' values at that column and accumulates in
//      registers; zeros cost nothing.
// The epilogue transposes the accumulators through LDS so that stores run along the output
// width: plain (optionally ReLU) for ECR order, or ReLU + max over the p_h*p_w adjacent rows of
// each pooling window for PECR order (Algorithm 4's reduction), storing only the pooled tensor.
#include "sconv_internal.h"

namespace sconv {

namespace {

constexpr int kBlock = 256;
constexpr int kWaves = kBlock / 64;
constexpr int kMaxLds = 44 * 1024;  // per workgroup: three workgroups share a CU's 160 KiB
constexpr int kMaxCK = 64;          // columns per chunk; bounds the staging registers

struct RowsCfg {
    int WT;       // window rows per workgroup (multiple of the pooling window size when pooling)
    int WA;       // rows of the register/LDS tile, 32 or 64, >= WT; rows WT..WA-1 stay empty
    int CK;       // columns per chunk (multiple of 16, at most kMaxCK)
    int PP;       // p_h*p_w when pooling, else 1
    int wpg;      // window rows per (image, group) in tile order
    int wtiles;   // tiles per (image, group)
};

__device__ __forceinline__ unsigned lanes_below(unsigned long long mask, int lane)
{
    return __popcll(mask & ((1ull << lane) - 1ull));
}

// LDS carve-up (dynamic); the same arithmetic runs on the host in rows_lds_bytes().
struct RowsLds {
    float* wt;        // [CK][KT+1]   filter tile, transposed; reused as out[KT][WA+1] at the end
    uint2* nz;        // [WA][CK]     compacted (value bits, byte offset of the column in wt)
    float* xt;        // [WA][CK+1]   dense chunk of the window rows
    int* origin;      // [WA][2]      ih0, iw0 of each window row (far out of range when unused)
    int* coloff;      // [2][CK]      offset of a chunk column from the window origin
    int* colrs;       // [2][CK]      (r << 16) | s
};

__host__ __device__ inline size_t rows_wt_words(int CK, int KT, int WA)
{
    size_t wt_words = (size_t)CK * (KT + 1);
    size_t out_words = (size_t)KT * (WA + 1);
    size_t a = wt_words > out_words ? wt_words : out_words;
    return (a + 3) & ~(size_t)3;  // keeps the uint2 array 16-byte aligned
}

size_t rows_lds_bytes(const RowsCfg& c, int KT)
{
    return rows_wt_words(c.CK, KT, c.WA) * 4 + (size_t)c.WA * c.CK * 8 + (size_t)c.WA * (c.CK + 1) * 4 +
           (size_t)c.WA * 8 + (size_t)c.CK * 16;
}

template <int KPL, int NWW, bool POOL>
__global__ __launch_bounds__(kBlock) void rows_kernel(Problem p, RowsCfg cfg,
                                                      const float* __restrict__ x,
                                                      const float* __restrict__ w,
                                                      float* __restrict__ y)
{
    constexpr int KT = 64 * KPL;
    constexpr int KTP = KT + 1;
    constexpr int WA = NWW * kWaves;
    constexpr int WTP = WA + 1;
    constexpr int XJS = kBlock / WA;               // column step of the activation loader (8 or 4)
    constexpr int XPT = kMaxCK / XJS;              // activation loads per thread and chunk (8 or 16)
    constexpr int WPT = KT * kMaxCK / kBlock;      // filter loads per thread and chunk (16 or 32)
    extern __shared__ __align__(16) unsigned char smem[];
    const int CKP = cfg.CK + 1;
    RowsLds lds;
    lds.wt = reinterpret_cast<float*>(smem);
    lds.nz = reinterpret_cast<uint2*>(lds.wt + rows_wt_words(cfg.CK, KT, WA));
    lds.xt = reinterpret_cast<float*>(lds.nz + (size_t)WA * cfg.CK);
    lds.origin = reinterpret_cast<int*>(lds.xt + (size_t)WA * CKP);
    lds.coloff = lds.origin + 2 * WA;
    lds.colrs = lds.coloff + 2 * cfg.CK;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int n = blockIdx.z / p.G;
    const int g = blockIdx.z - n * p.G;
    const int k0 = blockIdx.y * KT;                 // first filter of the tile inside the group
    const int q0 = blockIdx.x * cfg.WT;             // first window row of the tile
    const int RS = p.R * p.S;
    const int HW = p.H * p.W;

    auto fill_table = [&](int slot, int c0) {       // column table of the chunk starting at c0
        if (tid < cfg.CK) {
            const int col = min(c0 + tid, p.L - 1);
            const int c = col / RS;
            const int rs = col - c * RS;
            const int r = rs / p.S;
            const int s = rs - r * p.S;
            lds.coloff[slot * cfg.CK + tid] = c * HW + r * p.W + s;
            lds.colrs[slot * cfg.CK + tid] = (r << 16) | s;
        }
    };

    // window origins of the tile (ECR order: q = oh*OW + ow; PECR order: ((ph*PW+pw)*PP + py*p_w+px))
    if (tid < WA) {
        const int q = q0 + tid;
        int ih0 = -(1 << 20), iw0 = 0;  // every tap of an unused row is out of range
        if (tid < cfg.WT && q < cfg.wpg) {
            int oh, ow;
            if (POOL) {
                const int pp = q % cfg.PP, po = q / cfg.PP;
                const int py = pp / p.pw, px = pp - py * p.pw;
                const int phi = po / p.PW, pwi = po - phi * p.PW;
                oh = phi * p.ps + py;
                ow = pwi * p.ps + px;
            } else {
                oh = q / p.OW;
                ow = q - oh * p.OW;
            }
            ih0 = oh * p.stride - p.pad;
            iw0 = ow * p.stride - p.pad;
        }
        lds.origin[2 * tid] = ih0;
        lds.origin[2 * tid + 1] = iw0;
    }
    fill_table(0, 0);
    __syncthreads();

    float acc[KPL][NWW];
#pragma unroll
    for (int i = 0; i < KPL; ++i)
#pragma unroll
        for (int a = 0; a < NWW; ++a) acc[i][a] = 0.0f;

    const float* xg = x + ((size_t)n * p.C + (size_t)g * p.Cg) * HW;
    const float* wg = w + ((size_t)g * p.Kg + k0) * p.L;
    const int kvalid = min(KT, p.Kg - k0);

    // loader mappings.  Filters: lanes along the columns of one filter (contiguous in memory),
    // wavefront w takes filters w, w+4, ...; a filter past the group's last one re-reads the
    // last valid one (its lanes' results are never stored).  Activations: thread = (window,
    // column phase), a half or whole wavefront covers consecutive windows.
    const int xw = tid % WA;
    const int xj0 = tid / WA;
    const int xih0 = lds.origin[2 * xw], xiw0 = lds.origin[2 * xw + 1];
    const int xbase = xih0 <= -(1 << 20) ? 0 : xih0 * p.W + xiw0;

    float wstage[WPT];
    float xstage[XPT];
    auto prefetch = [&](int slot, int c0) {
        const int ck = min(cfg.CK, p.L - c0);
        // filters: element (k, j): j = lane (+64 never needed: CK <= 64), k = wave + 4*u
        const int j = min(lane, ck - 1);
#pragma unroll
        for (int u = 0; u < WPT; ++u) {
            const int k = wave + u * kWaves;
            wstage[u] = wg[(size_t)min(k, kvalid - 1) * p.L + c0 + j];
        }
        const int* coloff = lds.coloff + slot * cfg.CK;
        const int* colrs = lds.colrs + slot * cfg.CK;
#pragma unroll
        for (int u = 0; u < XPT; ++u) {
            const int jj = xj0 + u * XJS;
            float v = 0.0f;
            if (jj < ck) {
                const int rs = colrs[jj];
                const int ih = xih0 + (rs >> 16), iw = xiw0 + (rs & 0xffff);
                if (ih >= 0 && ih < p.H && iw >= 0 && iw < p.W) v = xg[xbase + coloff[jj]];
            }
            xstage[u] = v;
        }
    };
    auto commit = [&](int ck) {   // staged registers -> LDS
        if (lane < ck) {
#pragma unroll
            for (int u = 0; u < WPT; ++u) lds.wt[lane * KTP + wave + u * kWaves] = wstage[u];
        }
#pragma unroll
        for (int u = 0; u < XPT; ++u) {
            const int jj = xj0 + u * XJS;
            if (jj < ck) lds.xt[xw * CKP + jj] = xstage[u];
        }
    };

    prefetch(0, 0);
    int slot = 0;
    for (int c0 = 0; c0 < p.L; c0 += cfg.CK) {
        const int ck = min(cfg.CK, p.L - c0);
        __syncthreads();                 // every wavefront is done with the previous chunk's tiles
        commit(ck);
        const bool more = c0 + cfg.CK < p.L;
        if (more) fill_table(slot ^ 1, c0 + cfg.CK);
        __syncthreads();
        if (more) prefetch(slot ^ 1, c0 + cfg.CK);   // in flight during steps 3 and 4
        slot ^= 1;

        // 3. conversion of this wavefront's own window rows
        int cnts[NWW];
#pragma unroll
        for (int i = 0; i < NWW; ++i) {
            const int wi = wave * NWW + i;
            uint2* dst = lds.nz + (size_t)wi * cfg.CK;
            const float v = lane < ck ? lds.xt[wi * CKP + lane] : 0.0f;
            const bool nzv = v != 0.0f;
            const unsigned long long mask = __ballot(nzv);
            if (nzv) dst[lanes_below(mask, lane)] = make_uint2(__float_as_uint(v), (unsigned)(lane * KTP * 4));
            cnts[i] = __popcll(mask);
        }

        // 4. sparse product: lanes across filters, the nonzero list is uniform over the wavefront;
        //    four nonzeros in flight per step.  (LDS operations of one wavefront complete in
        //    order, so the lists written above are visible to the reads below.)
        const char* wt_lane = reinterpret_cast<const char*>(lds.wt + lane);
#pragma unroll
        for (int i = 0; i < NWW; ++i) {
            const int wi = wave * NWW + i;
            const int cnt = cnts[i];
            const uint2* src = lds.nz + (size_t)wi * cfg.CK;
            int e = 0;
            for (; e + 4 <= cnt; e += 4) {
                const uint4 t01 = *reinterpret_cast<const uint4*>(src + e);
                const uint4 t23 = *reinterpret_cast<const uint4*>(src + e + 2);
                float w0[KPL], w1[KPL], w2[KPL], w3[KPL];
#pragma unroll
                for (int q = 0; q < KPL; ++q) {
                    w0[q] = *reinterpret_cast<const float*>(wt_lane + t01.y + 256 * q);
                    w1[q] = *reinterpret_cast<const float*>(wt_lane + t01.w + 256 * q);
                    w2[q] = *reinterpret_cast<const float*>(wt_lane + t23.y + 256 * q);
                    w3[q] = *reinterpret_cast<const float*>(wt_lane + t23.w + 256 * q);
                }
#pragma unroll
                for (int q = 0; q < KPL; ++q) {
                    float a = acc[q][i];
                    a = fmaf(__uint_as_float(t01.x), w0[q], a);
                    a = fmaf(__uint_as_float(t01.z), w1[q], a);
                    a = fmaf(__uint_as_float(t23.x), w2[q], a);
                    a = fmaf(__uint_as_float(t23.z), w3[q], a);
                    acc[q][i] = a;
                }
            }
            for (; e < cnt; ++e) {
                const uint2 t = src[e];
#pragma unroll
                for (int q = 0; q < KPL; ++q)
                    acc[q][i] = fmaf(__uint_as_float(t.x),
                                     *reinterpret_cast<const float*>(wt_lane + t.y + 256 * q), acc[q][i]);
            }
        }
    }

    // epilogue: out[k][window] through LDS (aliases the filter tile)
    __syncthreads();
    float* out = lds.wt;
#pragma unroll
    for (int q = 0; q < KPL; ++q)
#pragma unroll
        for (int i = 0; i < NWW; ++i) out[(lane + 64 * q) * WTP + wave * NWW + i] = acc[q][i];
    __syncthreads();

    if (!POOL) {
        const int plane = p.OH * p.OW;
        const int nw = min(cfg.WT, cfg.wpg - q0);
        float* yg = y + ((size_t)n * p.K + (size_t)g * p.Kg + k0) * plane + q0;
        for (int idx = tid; idx < KT * WA; idx += kBlock) {
            const int k = idx / WA, i = idx - k * WA;
            if (k < kvalid && i < nw) {
                float v = out[k * WTP + i] + bias_of(p, (size_t)g * p.Kg + k0 + k);
                if (p.relu) v = fmaxf(v, 0.0f);
                yg[(size_t)k * plane + i] = v;
            }
        }
    } else {
        const int plane = p.PH * p.PW;
        const int TP = cfg.WT / cfg.PP;             // pooled outputs per tile
        const int po0 = q0 / cfg.PP;
        const int np = min(TP, plane - po0);
        float* yg = y + ((size_t)n * p.K + (size_t)g * p.Kg + k0) * plane + po0;
        for (int idx = tid; idx < KT * TP; idx += kBlock) {
            const int k = idx / TP, i = idx - k * TP;
            if (k < kvalid && i < np) {
                float m = out[k * WTP + i * cfg.PP];
                for (int t = 1; t < cfg.PP; ++t) m = fmaxf(m, out[k * WTP + i * cfg.PP + t]);
                yg[(size_t)k * plane + i] = fmaxf(m + bias_of(p, (size_t)g * p.Kg + k0 + k), 0.0f);   // bias, ReLU
            }
        }
    }
}

template <int KPL, int NWW, bool POOL>
int launch_one(const Problem& p, const RowsCfg& cfg, dim3 grid, size_t lds, const float* x,
               const float* w, float* y, hipStream_t stream)
{
    hipLaunchKernelGGL((rows_kernel<KPL, NWW, POOL>), grid, dim3(kBlock), lds, stream, p, cfg, x, w, y);
    return launch_status();
}

template <int KPL, bool POOL>
int launch_wa(const Problem& p, const RowsCfg& cfg, dim3 grid, size_t lds, const float* x,
              const float* w, float* y, hipStream_t stream)
{
    return cfg.WA == 32 ? launch_one<KPL, 8, POOL>(p, cfg, grid, lds, x, w, y, stream)
                        : launch_one<KPL, 16, POOL>(p, cfg, grid, lds, x, w, y, stream);
}

}  // namespace

int launch_rows(const Problem& p, bool pooled, const float* x, const float* w, float* y,
                hipStream_t stream)
{
    RowsCfg cfg;
    cfg.PP = pooled ? p.ph * p.pw : 1;
    if (cfg.PP > 64 || p.R > 32767 || p.S > 32767) return SCONV_EUNSUPPORTED;
    cfg.wpg = pooled ? p.PH * p.PW * cfg.PP : p.OH * p.OW;

    // Window rows per tile: 32 (64 when one pooling window alone needs more), then the largest
    // whole number of pooling windows that fits; rows past WT are marked unused.
    cfg.WA = cfg.PP > 32 ? 64 : 32;
    cfg.WT = (cfg.WA / cfg.PP) * cfg.PP;
    cfg.wtiles = (cfg.wpg + cfg.WT - 1) / cfg.WT;

    // Filters per tile: 128 (two per lane) when the group has more than 64 and the launch still
    // has plenty of workgroups, else 64.
    int kpl = p.Kg > 64 ? 2 : 1;
    if (kpl == 2) {
        const long long wgs = (long long)cfg.wtiles * ((p.Kg + 127) / 128) * p.N * p.G;
        if (wgs < 1536) kpl = 1;
    }
    const int kt = 64 * kpl;

    // Columns per chunk: the largest multiple of 16 (at most kMaxCK, at most L rounded up) that fits.
    int ck = kMaxCK;
    if (ck > p.L) ck = (p.L + 15) / 16 * 16;
    cfg.CK = ck;
    while (rows_lds_bytes(cfg, kt) > (size_t)kMaxLds && cfg.CK > 16) cfg.CK -= 16;
    const size_t lds = rows_lds_bytes(cfg, kt);
    if (lds > (size_t)kMaxLds) return SCONV_EUNSUPPORTED;

    const unsigned gz = (unsigned)(p.N * p.G);
    const unsigned gy = (unsigned)((p.Kg + kt - 1) / kt);
    if (gz > 65535u || gy > 65535u) return SCONV_EUNSUPPORTED;
    dim3 grid((unsigned)cfg.wtiles, gy, gz);
    if (kpl == 2)
        return pooled ? launch_wa<2, true>(p, cfg, grid, lds, x, w, y, stream)
                      : launch_wa<2, false>(p, cfg, grid, lds, x, w, y, stream);
    return pooled ? launch_wa<1, true>(p, cfg, grid, lds, x, w, y, stream)
                  : launch_wa<1, false>(p, cfg, grid, lds, x, w, y, stream);
}

}  // namespace sconv

// General window-row kernel: the structure of Sections 5 and 6 carried to many channels,
// filters and images, for any kernel size, stride, padding, grouping and pooling window.
//
// A workgroup (4 wavefronts) owns WT window rows of one (image, group) and KT filters of that
// group.  The L = Cg*R*S columns of the rows are walked in chunks of CK columns.  Per chunk:
//   1. the filter tile w[k][chunk] is staged into LDS transposed to [column][k], so that the 64
//      lanes of a wavefront (64 consecutive filters) read one column without bank conflicts;
//   2. every window row of the tile is converted on chip: a wavefront scans the chunk's columns
//      64 at a time (ascending c, r, s), and ballot + population count of the lower lanes give
//      each nonzero its slot in the row's compacted list in LDS (value, column) - Algorithm 1 /
//      Algorithm 3 at wavefront level; zero padding reads as zeros and is never emitted;
//   3. the sparse product of Algorithm 2: for every stored nonzero of a row (the same for all
//      lanes) each lane multiplies by its own filter's value at that column and accumulates in
//      a register; zeros cost nothing.
// The epilogue transposes the accumulators through LDS so that stores run along the output
// width: plain (optionally ReLU) for ECR order, or ReLU + max over the p_h*p_w adjacent rows of
// each pooling window for PECR order (Algorithm 4's reduction), storing only the pooled tensor.
#include "sconv_internal.h"

namespace sconv {

namespace {

constexpr int kBlock = 256;
constexpr int kWaves = kBlock / 64;
constexpr int kMaxLds = 64 * 1024;  // per workgroup; two workgroups then share a CU's 160 KiB

struct RowsCfg {
    int WT;       // window rows per workgroup (multiple of the pooling window size when pooling)
    int WA;       // rows of the register/LDS tile, 32 or 64, >= WT; rows WT..WA-1 stay empty
    int KT;       // filters per workgroup (multiple of 64)
    int KW;       // wavefronts across filters (1, 2 or 4); the other 4/KW split the windows
    int CK;       // columns per chunk
    int PP;       // p_h*p_w when pooling, else 1
    int wpg;      // window rows per (image, group) in tile order
    int wtiles;   // tiles per (image, group)
};

__device__ __forceinline__ unsigned lanes_below(unsigned long long mask, int lane)
{
    return __popcll(mask & ((1ull << lane) - 1ull));
}

// LDS carve-up (dynamic): see rows_lds_bytes() for the same arithmetic on the host.
struct RowsLds {
    float* wt;        // [CK][KT+1]   filter tile, transposed; reused as out[KT][WA+1] at the end
    uint2* nz;        // [WA][CK]     compacted (value bits, byte offset of the column in wt)
    int* cnt;         // [WA]
    int* origin;      // [WA][2]      ih0, iw0 of each window row (far out of range when unused)
    int* coloff;      // [CK]         offset of a chunk column from the window origin
    int* colrs;       // [CK]         (r << 16) | s
};

template <int NWW, bool POOL>
__global__ __launch_bounds__(kBlock) void rows_kernel(Problem p, RowsCfg cfg,
                                                      const float* __restrict__ x,
                                                      const float* __restrict__ w,
                                                      float* __restrict__ y)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int KTP = cfg.KT + 1;
    const int WTP = cfg.WA + 1;
    RowsLds lds;
    {
        size_t wt_words = (size_t)cfg.CK * KTP;
        size_t out_words = (size_t)cfg.KT * WTP;  // WTP = WA + 1
        size_t a = wt_words > out_words ? wt_words : out_words;
        a = (a + 1) & ~(size_t)1;  // keep the uint2 array 8-byte aligned
        lds.wt = reinterpret_cast<float*>(smem);
        lds.nz = reinterpret_cast<uint2*>(lds.wt + a);
        lds.cnt = reinterpret_cast<int*>(lds.nz + (size_t)cfg.WA * cfg.CK);
        lds.origin = lds.cnt + cfg.WA;
        lds.coloff = lds.origin + 2 * cfg.WA;
        lds.colrs = lds.coloff + cfg.CK;
    }

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int n = blockIdx.z / p.G;
    const int g = blockIdx.z - n * p.G;
    const int k0 = blockIdx.y * cfg.KT;             // first filter of the tile inside the group
    const int q0 = blockIdx.x * cfg.WT;             // first window row of the tile
    const int kw = wave % cfg.KW;                   // which 64 filters this wavefront owns
    const int ww = wave / cfg.KW;                   // which NWW window rows it owns
    const int kl = kw * 64 + lane;                  // filter index inside the tile
    const int RS = p.R * p.S;
    const int HW = p.H * p.W;

    // window origins of the tile (ECR order: q = oh*OW + ow; PECR order: ((ph*PW+pw)*PP + py*p_w+px))
    if (tid < cfg.WA) {
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

    float acc[NWW];
#pragma unroll
    for (int i = 0; i < NWW; ++i) acc[i] = 0.0f;

    const float* xg = x + ((size_t)n * p.C + (size_t)g * p.Cg) * HW;
    const float* wg = w + ((size_t)g * p.Kg + k0) * p.L;
    const int kvalid = min(cfg.KT, p.Kg - k0);

    for (int c0 = 0; c0 < p.L; c0 += cfg.CK) {
        const int ck = min(cfg.CK, p.L - c0);
        __syncthreads();  // previous chunk fully consumed (and origins visible on the first pass)

        // column table of this chunk
        if (tid < ck) {
            const int col = c0 + tid;
            const int c = col / RS;
            const int rs = col - c * RS;
            const int r = rs / p.S;
            const int s = rs - r * p.S;
            lds.coloff[tid] = c * HW + r * p.W + s;
            lds.colrs[tid] = (r << 16) | s;
        }
        // 1. filter tile, transposed: consecutive lanes read consecutive columns of one filter
        for (int k = wave; k < cfg.KT; k += kWaves) {
            const float* src = wg + (size_t)k * p.L + c0;
            for (int j = lane; j < ck; j += 64)
                lds.wt[j * KTP + k] = k < kvalid ? src[j] : 0.0f;
        }
        __syncthreads();

        // 2. conversion of the tile's window rows, one wavefront per row at a time
        for (int wi = wave; wi < cfg.WA; wi += kWaves) {
            const int ih0 = lds.origin[2 * wi], iw0 = lds.origin[2 * wi + 1];
            const int base = ih0 <= -(1 << 20) ? 0 : ih0 * p.W + iw0;
            uint2* dst = lds.nz + (size_t)wi * cfg.CK;
            int cnt = 0;
            for (int j0 = 0; j0 < ck; j0 += 64) {
                const int j = j0 + lane;
                float v = 0.0f;
                if (j < ck) {
                    const int rs = lds.colrs[j];
                    const int ih = ih0 + (rs >> 16), iw = iw0 + (rs & 0xffff);
                    if (ih >= 0 && ih < p.H && iw >= 0 && iw < p.W) v = xg[base + lds.coloff[j]];
                }
                const bool nzv = v != 0.0f;
                const unsigned long long mask = __ballot(nzv);
                if (nzv) {
                    const int slot = cnt + lanes_below(mask, lane);
                    dst[slot] = make_uint2(__float_as_uint(v), (unsigned)(j * KTP * 4));
                }
                cnt += __popcll(mask);
            }
            if (lane == 0) lds.cnt[wi] = cnt;
        }
        __syncthreads();

        // 3. sparse product: lanes across filters, the nonzero list is uniform over the wavefront
        const char* wt_lane = reinterpret_cast<const char*>(lds.wt + kl);
#pragma unroll
        for (int i = 0; i < NWW; ++i) {
            const int wi = ww * NWW + i;
            const int cnt = lds.cnt[wi];
            const uint2* src = lds.nz + (size_t)wi * cfg.CK;
            float a = acc[i];
            for (int e = 0; e < cnt; ++e) {
                const uint2 t = src[e];
                a = fmaf(__uint_as_float(t.x), *reinterpret_cast<const float*>(wt_lane + t.y), a);
            }
            acc[i] = a;
        }
    }

    // epilogue: out[k][window] through LDS (aliases the filter tile)
    __syncthreads();
    float* out = lds.wt;
#pragma unroll
    for (int i = 0; i < NWW; ++i) out[kl * WTP + ww * NWW + i] = acc[i];
    __syncthreads();

    if (!POOL) {
        const int plane = p.OH * p.OW;
        const int nw = min(cfg.WT, cfg.wpg - q0);
        float* yg = y + ((size_t)n * p.K + (size_t)g * p.Kg + k0) * plane + q0;
        for (int idx = tid; idx < cfg.KT * cfg.WT; idx += kBlock) {
            const int k = idx / cfg.WT, i = idx - k * cfg.WT;
            if (k < kvalid && i < nw) {
                float v = out[k * WTP + i];
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
        for (int idx = tid; idx < cfg.KT * TP; idx += kBlock) {
            const int k = idx / TP, i = idx - k * TP;
            if (k < kvalid && i < np) {
                float m = 0.0f;  // ReLU folded into the start value
                for (int t = 0; t < cfg.PP; ++t) m = fmaxf(m, out[k * WTP + i * cfg.PP + t]);
                yg[(size_t)k * plane + i] = m;
            }
        }
    }
}

size_t rows_lds_bytes(const RowsCfg& c)
{
    size_t wt_words = (size_t)c.CK * (c.KT + 1);
    size_t out_words = (size_t)c.KT * (c.WA + 1);
    size_t a = wt_words > out_words ? wt_words : out_words;
    a = (a + 1) & ~(size_t)1;
    return a * 4 + (size_t)c.WA * c.CK * 8 + (size_t)c.WA * 4 * 3 + (size_t)c.CK * 8;
}

template <int NWW, bool POOL>
int launch_one(const Problem& p, const RowsCfg& cfg, dim3 grid, size_t lds, const float* x,
               const float* w, float* y, hipStream_t stream)
{
    auto kern = rows_kernel<NWW, POOL>;
    static size_t allowed = 48 * 1024;  // dynamic LDS above 48 KiB is opted into once
    if (lds > allowed) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds) != hipSuccess)
            return SCONV_ELAUNCH;
        allowed = kMaxLds;
    }
    hipLaunchKernelGGL(kern, grid, dim3(kBlock), lds, stream, p, cfg, x, w, y);
    return launch_status();
}

template <bool POOL>
int launch_nww(int nww, const Problem& p, const RowsCfg& cfg, dim3 grid, size_t lds, const float* x,
               const float* w, float* y, hipStream_t stream)
{
    switch (nww) {
    case 8: return launch_one<8, POOL>(p, cfg, grid, lds, x, w, y, stream);
    case 16: return launch_one<16, POOL>(p, cfg, grid, lds, x, w, y, stream);
    case 32: return launch_one<32, POOL>(p, cfg, grid, lds, x, w, y, stream);
    case 64: return launch_one<64, POOL>(p, cfg, grid, lds, x, w, y, stream);
    default: return SCONV_EUNSUPPORTED;
    }
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
    // whole number of pooling windows that fits.  The register tile NWW*WW covers WA rows; rows
    // past WT are marked unused.
    cfg.WA = cfg.PP > 32 ? 64 : 32;
    const int wt_alloc = cfg.WA;
    cfg.WT = (wt_alloc / cfg.PP) * cfg.PP;
    cfg.wtiles = (cfg.wpg + cfg.WT - 1) / cfg.WT;

    // Filters per tile: up to 256 (one wavefront per 64); fewer when the launch would be small.
    int kt = (p.Kg + 63) / 64 * 64;
    if (kt > 256) kt = 256;
    if (kt == 192) kt = 256;
    long long wgs = (long long)cfg.wtiles * ((p.Kg + kt - 1) / kt) * p.N * p.G;
    while (kt > 64 && wgs < 1024) {
        kt /= 2;
        wgs = (long long)cfg.wtiles * ((p.Kg + kt - 1) / kt) * p.N * p.G;
    }
    cfg.KT = kt;
    cfg.KW = kt / 64;
    const int WW = kWaves / cfg.KW;
    const int nww = wt_alloc / WW;

    // Columns per chunk: the largest multiple of 16 (at most 128, at most L rounded up) that fits.
    int ck = 128;
    if (ck > p.L) ck = (p.L + 15) / 16 * 16;
    cfg.CK = ck;
    while (rows_lds_bytes(cfg) > (size_t)kMaxLds && cfg.CK > 16) cfg.CK -= 16;
    const size_t lds = rows_lds_bytes(cfg);
    if (lds > (size_t)kMaxLds) return SCONV_EUNSUPPORTED;

    const unsigned gz = (unsigned)(p.N * p.G);
    const unsigned gy = (unsigned)((p.Kg + kt - 1) / kt);
    if (gz > 65535u || gy > 65535u) return SCONV_EUNSUPPORTED;
    dim3 grid((unsigned)cfg.wtiles, gy, gz);
    return pooled ? launch_nww<true>(nww, p, cfg, grid, lds, x, w, y, stream)
                  : launch_nww<false>(nww, p, cfg, grid, lds, x, w, y, stream);
}

}  // namespace sconv

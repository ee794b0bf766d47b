// Element-stationary 3x3 kernel without shared staging: the arithmetic and the position code of
// sconv_tap.hip (Section 5.4: only nonzero elements are multiplied; lanes hold filters, the
// accumulators of an output tile live in registers), but every wavefront fetches the filter values of
// its own channels itself, straight into registers, one channel ahead.
//
// Why: in the staged kernel a workgroup meets at a barrier for every chunk of 16 channels, and a
// wavefront's wait for its next elements also waits for the chunk's filter fetch (vector loads return
// in order); measured on the 512-channel layers, wavefronts spend half of their time waiting and the
// vector pipe is busy half of the time although eight wavefronts are resident per SIMD.  Here
// nothing is shared during the channel loop, so there is no barrier and no wait other than a
// wavefront's own prefetch, which one channel's products cover.
//
// The price: filters must be readable 64 lanes = 64 consecutive filters at a time, which the
// [K][C/G][3][3] layout is not (consecutive filters lie 36*C/G bytes apart).  The kernel reads a
// transposed copy, [group][block of 64 filters][channel][tap][64], zero-filled past the group's last
// filter.  A caller whose filters stay the same from call to call writes it once (sconv_filter_prep) and
// passes it with every call; otherwise a first small kernel writes it into the caller's workspace before
// every launch (9.4 MB for 512 x 512 filters, about 10 us); with neither the plans of this file do not
// apply and the staged kernel runs.
#include <stdio.h>
#include <string.h>

#include <map>
#include <utility>

#include "sconv_internal.h"
#include "sconv_tapt.h"

namespace sconv {

namespace {

#include "sconv_tap_common.h"

// w[K][Cg][9] -> wt[(g * kblocks + kb) * Cg * 9 + ct][64] with ct = c * 9 + tap, through a 64 x 64 LDS
// tile so that both sides are accessed in runs of 64 consecutive words.
__global__ __launch_bounds__(1024) void transpose_filters_kernel(Problem p, int kblocks,
                                                                const float* __restrict__ w, float* __restrict__ wt)
{
    constexpr int KB = 64;
    __shared__ float tile[64][65];
    const int ct0 = blockIdx.x * 64;          // first (channel, tap) entry of the tile
    const int kk0 = blockIdx.y * 64;          // first filter of the tile inside the group's padded range
    const int g = blockIdx.z;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int kpad = kblocks * KB;            // filters per group, rounded up to whole blocks
#pragma unroll
    for (int i = 0; i < 4; ++i) {             // row r: filter kk0 + r, 64 consecutive entries
        const int r = ty + 16 * i;
        const int kk = kk0 + r, ct = ct0 + tx;
        float v = 0.0f;
        if (kk < p.Kg && ct < p.L) v = w[((size_t)g * p.Kg + kk) * p.L + ct];
        tile[r][tx] = v;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {             // row r: entry ct0 + r, 64 consecutive filters
        const int r = ty + 16 * i;
        const int ct = ct0 + r, kk = kk0 + tx;
        if (ct < p.L && kk < kpad) {
            const int kb = kk / KB, ki = kk - kb * KB;
            wt[(((size_t)g * kblocks + kb) * p.L + ct) * KB + ki] = tile[tx][r];
        }
    }
}

template <class G, int NWV>
__global__ __launch_bounds__(NWV * 64) void tapt_kernel(Problem p, TapCfg cfg, const float* __restrict__ x,
                                                    const float* __restrict__ wt, float* __restrict__ y)
{
    extern __shared__ __align__(16) float lds[];  // slice reduction only

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ts = wave % cfg.NT;                  // spatial tile slot
    const int cs = wave / cfg.NT;                  // channel slice
    // Workgroups are handed to the eight XCDs in turn, in launch order.  They are renumbered so that an XCD
    // works on few filter blocks AND few images: the eight XCDs form xcd_remap groups along the filter blocks
    // times 8 / xcd_remap groups along grid z (images), so that an XCD's L2 has to hold 1 / xcd_remap of the
    // transposed filters and xcd_remap / 8 of the input instead of everything being fetched into all eight.
    int bx = blockIdx.x, by = blockIdx.y, bz = blockIdx.z;
    if (cfg.xcd_remap) {
        const unsigned a = (unsigned)cfg.xcd_remap, bgroups = 8u / a;
        const unsigned kper = gridDim.y / a;                 // filter blocks per XCD
        const unsigned lin = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
        const unsigned xcd = lin & 7u, idx = lin >> 3;
        const unsigned xa = xcd % a, xb = xcd / a;
        bx = (int)(idx % gridDim.x);
        const unsigned t = idx / gridDim.x;
        by = (int)(xa * kper + t % kper);
        bz = (int)((t / kper) * bgroups + xb);
    }
    const int ss = bz % cfg.NSS;                   // channel range of the workgroup
    const int ng = bz / cfg.NSS;
    const int n = ng / p.G;
    const int g = ng - n * p.G;
    const int kb0 = by * G::KB;
    const int tile = bx * cfg.NT + ts;
    const bool tile_ok = tile < cfg.ntiles;
    const int ty = tile / cfg.tiles_x, tx = tile - ty * cfg.tiles_x;
    const int oh0 = ty * G::TH, ow0 = tx * G::TW;
    const int HWp = p.H * p.W;
    const int kvalid = min(G::KB, p.Kg - kb0);

    unsigned xoff[G::NX];
    bool xok[G::NX];
#pragma unroll
    for (int q = 0; q < G::NX; ++q) {
        const int P = q * 64 + lane;
        const int ih = P / G::IW, iw = P - ih * G::IW;
        const int xr = oh0 * G::STRIDE - G::HH + ih, xc = ow0 * G::STRIDE - G::HW + iw;
        xok[q] = tile_ok && P < G::NPOS && xr >= 0 && xr < p.H && xc >= 0 && xc < p.W;
        xoff[q] = xok[q] ? (unsigned)(xr * p.W + xc) : 0u;
    }
    const float* xg = x + ((size_t)n * p.C + (size_t)g * p.Cg) * HWp;
    // the block's transposed filters: entry (c, tap) of filter lane + 64*i at wl[(c*9 + tap)*KB + 64*i]
    // (filter register i of the lane: block by * KPL + i, cfg.wt_blocks blocks per group)
    const float* wl = wt + ((size_t)g * cfg.wt_blocks + (size_t)by * G::KPL) * p.L * 64 + lane;
    const size_t wblock = (size_t)p.L * 64;

    float acc[G::KPL][G::ACC];
#pragma unroll
    for (int i = 0; i < G::KPL; ++i)
#pragma unroll
        for (int a = 0; a < G::ACC; ++a) acc[i][a] = 0.0f;

    // this wavefront's channels: slice cs of the workgroup's range, itself part ss of the group's
    const int per = p.Cg / (cfg.NSS * cfg.NCS);
    const int c_lo = (ss * cfg.NCS + cs) * per, c_hi = c_lo + per;

    auto load_x = [&](int c, float (&dst)[G::NX]) {
        const float* base = xg + (size_t)c * HWp;
#pragma unroll
        for (int q = 0; q < G::NX; ++q) {
            const float t = base[xoff[q]];
            dst[q] = xok[q] ? t : 0.0f;
        }
    };
    auto load_w = [&](int c, float (&dst)[G::KPL][9]) {
#pragma unroll
        for (int i = 0; i < G::KPL; ++i) {
            const float* base = wl + i * wblock + (size_t)c * 9 * 64;
#pragma unroll
            for (int j = 0; j < 9; ++j) dst[i][j] = base[j * 64];
        }
    };

    float xn[G::NX], wn[G::KPL][9];
    load_x(c_lo, xn);
    load_w(c_lo, wn);
    for (int c = c_lo; c < c_hi; ++c) {
        float xv[G::NX], wr[G::KPL][9];
        unsigned mask[2 * G::NX];
        unsigned any = 0;
#pragma unroll
        for (int q = 0; q < G::NX; ++q) {
            xv[q] = xn[q];
            const unsigned long long m = __ballot(xv[q] != 0.0f);
            mask[2 * q] = (unsigned)m;
            mask[2 * q + 1] = (unsigned)(m >> 32);
            any |= mask[2 * q] | mask[2 * q + 1];
        }
#pragma unroll
        for (int j = 0; j < 9; ++j)
#pragma unroll
            for (int i = 0; i < G::KPL; ++i) wr[i][j] = wn[i][j];
        // the next channel's operands (the last channel is read again past the end of the range)
        const int cn = min(c + 1, c_hi - 1);
        load_x(cn, xn);
        load_w(cn, wn);
        if (any) all_positions<G>(std::make_integer_sequence<int, (G::NPOS + 3) / 4>{}, mask, xv, acc, wr);
    }

    reduce_slices<G>(cfg, lds, acc, ts, cs, lane);
    if (cs != 0 || !tile_ok) return;
    store_tile<G>(p, acc, y, ss, n, g, kb0, kvalid, oh0, ow0, lane);
}

template <class G, int NWV>
int launch_nwv(const Problem& p, const TapCfg& cfg, dim3 grid, size_t lds_bytes, const float* x, const float* wt,
               float* y, hipStream_t stream)
{
    auto kern = tapt_kernel<G, NWV>;
    static size_t opted = 48 * 1024;
    if (lds_bytes > opted) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds_bytes) != hipSuccess)
            return SCONV_ELAUNCH;
        opted = lds_bytes;
    }
    hipLaunchKernelGGL(kern, grid, dim3(NWV * 64), lds_bytes, stream, p, cfg, x, wt, y);
    return launch_status();
}

int prep_blocks(const Problem& p) { return (p.Kg + 127) / 128 * 2; }

// bytes of the workspace a launch keeps for the transposed filters: none when the caller brought them
size_t wt_bytes(const Problem& p) { return p.wprep ? 0 : filter_prep_bytes(p); }

}  // namespace

size_t filter_prep_bytes(const Problem& p)
{
    return ((size_t)p.G * prep_blocks(p) * p.L * 64 * sizeof(float) + 255) / 256 * 256;
}

int launch_filter_prep(const Problem& p, const float* w, float* wt, hipStream_t stream)
{
    const int kblocks = prep_blocks(p);
    const dim3 tgrid((unsigned)((p.L + 63) / 64), (unsigned)kblocks, (unsigned)p.G);
    if (tgrid.y > 65535 || tgrid.z > 65535) return SCONV_EUNSUPPORTED;
    hipLaunchKernelGGL(transpose_filters_kernel, tgrid, dim3(1024), 0, stream, p, kblocks, w, wt);
    return launch_status();
}

// Decomposition of one launch of the transposed-filter kernel: wavefronts per workgroup nwv = NT tiles
// x NCS channel slices (slices only add up through LDS at the end), NSS workgroups per tile along the
// channels.  split: 0 = not allowed, 1 = allowed, 2 = required (a plain tile serving a pooled call).
// Pinned decompositions are taken as they are; otherwise the rule inside.
template <class G>
Plan plan_tapt(const Problem& p, int split)
{
    Plan best;
    // the transposed filters come with the call, or are written into the workspace first
    if (!p.wprep && (!split_scratch_possible(nullptr) || split_scratch_bytes() < wt_bytes(p))) return best;
    TapCfg cfg;
    cfg.tiles_y = (p.OH + G::TH - 1) / G::TH;
    cfg.tiles_x = (p.OW + G::TW - 1) / G::TW;
    cfg.ntiles = cfg.tiles_x * cfg.tiles_y;
    const int kblocks = (p.Kg + G::KB - 1) / G::KB;
    const size_t red_per_tile = (size_t)G::KPL * G::ACC * 64 * sizeof(float);
    const size_t part_bytes = (size_t)p.N * p.K * p.OH * p.OW * sizeof(float);
    int pin_nwv = 0, pin_ncs = 0, pin_nss = 0;
    pinned_split("SCONV_TAP_SPLIT", &pin_nwv, &pin_ncs, &pin_nss);
    const long long tile_waves = (long long)cfg.ntiles * kblocks * p.N * p.G;
    int nwv = pin_nwv, ncs = pin_ncs, nss = pin_nss ? pin_nss : 1;
    if (!pin_nwv) {
        // Measured (sconv_tune's picks on 128- to 512-channel layers): eight channel slices whenever a slice
        // keeps 16 channels - many short wavefronts even out the last round -, one tile per workgroup,
        // two from 512 channels up (plain tiles only); pooled tiles of 14-wide maps, few per image, sixteen slices.
        ncs = 1;
        // (a whole-map tile is the only tile of its image: all wavefronts of its workgroup are slices of it)
        const int want = ((G::POOL && G::HW == 0) || (cfg.ntiles == 1 && p.Cg >= 512 && G::MAXW == 16)) ? 16 : 8;
        while (ncs < want && p.Cg / (ncs * 2) >= 16 && p.Cg % (ncs * 2) == 0) ncs *= 2;
        nwv = ((p.Cg >= 512 && !G::POOL) || ncs == 16) && G::MAXW == 16 ? 16 : 8;
        if (ncs > nwv) ncs = nwv;
        if (cfg.ntiles == 1 && ncs >= 8) nwv = ncs;
        if (split == 2) nss = 2;
        // (small launches: the channels of a tile over several workgroups as well, until 3072 to 4096 wavefronts -
        // about half of what the chip holds - share the work; a wavefront keeps 16 channels, or 4 when the launch has
        // fewer than 1024 wavefronts to begin with - sconv_tune's picks with prepared filters: 512 @28x28 at batch 1
        // 8 slices x 4 workgroups, 512 @14x14 and 256 @14x14 x 8, 512 @7x7 x 16, 2048 in 16 groups @7x7 x 4;
        // 192 -> 384 @7x7 at batch 32, 24 channels per wavefront, unsplit)
        // (the smallest stop at 3072: 512 @14x14 at batch 1 runs 20.5 us 8 ways and 23.5 us 16 ways)
        const int keep = tile_waves * ncs < 1024 ? 4 : 16;
        const long long fill = tile_waves * ncs < 1024 ? 3072 : 4096;
        while (split >= 1 && split_scratch_possible(nullptr) && nss < 16 && tile_waves * ncs * nss < fill &&
               p.Cg / (ncs * nss * 2) >= keep && p.Cg % (ncs * nss * 2) == 0)
            nss *= 2;
        // (and then one tile per workgroup: with two, half of the workgroups)
        if (nss > 1 && nwv > ncs && ncs >= 8) nwv = ncs;
    }
    if (nwv != 8 && !(nwv == 16 && G::MAXW == 16)) return best;
    // (16 wavefronts leave 128 registers: two filters per lane on a 5x7 tile do not fit without spilling)
    if (nwv == 16 && G::KPL * G::ACC > 60) return best;
    if (ncs < 1 || ncs > nwv || (ncs & (ncs - 1)) || nss < 1 || p.Cg % (ncs * nss)) return best;
    if (nss > 1 && (split == 0 || G::POOL || !split_scratch_possible(nullptr) || wt_bytes(p) + nss * part_bytes > split_scratch_bytes() ||
                    (long long)p.N * p.G * nss > 65535))
        return best;
    if (nss == 1 && split == 2) return best;
    const int nt = nwv / ncs;
    size_t lds_bytes = ncs > 1 ? nt * red_per_tile : 0;
    // room for half of the slices side by side makes the reduction a tree
    if (ncs > 2 && lds_bytes * (ncs / 2) <= 64 * 1024) lds_bytes *= ncs / 2;
    if (lds_bytes > 160 * 1024) return best;
    best.cfg = cfg;
    best.cfg.NT = nt;
    best.cfg.NCS = ncs;
    best.cfg.CPW = 0;
    best.cfg.NSS = nss;
    best.cfg.RW = ncs > 1 ? (int)(lds_bytes / (nt * red_per_tile)) : 1;
    best.nwv = nwv;
    best.kblocks = kblocks;
    best.lds_bytes = lds_bytes;
    best.nss = nss;
    best.wgs1 = (long long)((cfg.ntiles + nt - 1) / nt) * kblocks * p.N * p.G;
    // priced like the staged kernel's channel time without its per-chunk waits
    const double nnz = 0.3 * G::NPOS;
    const double t_channel = 60.0 + 6.0 * G::NPOS + nnz * (14.0 + 4.5 * 9.0 * G::ACC * G::KPL / G::NPOS);
    const double waves = (double)best.wgs1 * nwv * nss;
    const double rounds = waves > 8.0 * 1024 ? waves / (8.0 * 1024) : 1.0;
    best.cost = rounds * (double)p.Cg / (ncs * nss) * t_channel * 4.0 + 12000.0 + (nss > 1 ? 9000.0 : 0.0);
    return best;
}

template <class G>
int launch_tapt(const Plan& pl, const Problem& p, bool pooled, const float* x, const float* w, float* y,
                hipStream_t stream)
{
    const long long gx = (pl.cfg.ntiles + pl.cfg.NT - 1) / pl.cfg.NT;
    const long long gz = (long long)p.N * p.G * pl.nss;
    if (gz > 65535 || pl.kblocks > 65535 || gx >= (1LL << 31)) return SCONV_EUNSUPPORTED;
    float* ws = split_scratch(stream);
    const size_t wtb = wt_bytes(p);
    if (!p.wprep && (!ws || split_scratch_bytes() < wtb)) return SCONV_EUNSUPPORTED;
    const float* wt = p.wprep ? p.wprep : ws;
    float* part = ws ? ws + wtb / sizeof(float) : nullptr;
    Problem q = p;
    float* out = y;
    if (pl.nss > 1) {
        if (G::POOL || !part || wtb + (size_t)pl.nss * p.N * p.K * p.OH * p.OW * sizeof(float) > split_scratch_bytes())
            return SCONV_EUNSUPPORTED;
        out = part;
        q.relu = 0;
        q.bias = nullptr;
    } else if (pooled != G::POOL) {
        return SCONV_EUNSUPPORTED;
    }
    if (p.Cg % (pl.cfg.NCS * pl.nss)) return SCONV_EUNSUPPORTED;
    if (!p.wprep) {
        if (const int trc = launch_filter_prep(p, w, ws, stream)) return trc;
    }
    const dim3 grid((unsigned)gx, (unsigned)pl.kblocks, (unsigned)gz);
    TapCfg cfg = pl.cfg;
    cfg.wt_blocks = prep_blocks(p);
    // XCD groups along the filter blocks (a) and along grid z (8 / a): the split that makes an XCD fetch the
    // least - filters / a + input * a / 8 - among those that divide the grid evenly and leave an XCD at most
    // 2.5 MB of filters, so that they stay in its 4 MB L2 while the input streams through
    cfg.xcd_remap = 0;
    if (!env_value("SCONV_NO_XCD_REMAP") && gx * pl.kblocks * gz < (1LL << 32)) {
        const double wbytes = (double)p.K * p.L * 4.0, xbytes = (double)p.N * p.C * p.H * p.W * 4.0;
        double best = 0.0;
        for (int a = 1; a <= 8; a *= 2) {
            if (pl.kblocks % a || gz % (8 / a)) continue;
            const double fetched = wbytes / a + xbytes * a / 8.0 + (wbytes / a > 2.5e6 ? 1e12 / a : 0.0);
            if (!cfg.xcd_remap || fetched < best) {
                cfg.xcd_remap = a;
                best = fetched;
            }
        }
    }
    int rc;
    if (G::MAXW == 16 && pl.nwv == 16)
        rc = launch_nwv<G, G::MAXW>(q, cfg, grid, pl.lds_bytes, x, wt, out, stream);
    else
        rc = launch_nwv<G, 8>(q, cfg, grid, pl.lds_bytes, x, wt, out, stream);
    if (rc != SCONV_OK || pl.nss == 1) return rc;
    return launch_split_reduce(p, pooled, out, pl.nss, y, stream);
}

// The tile geometries this kernel is built for (the names carry a trailing t in the candidate table of
// sconv_tap.hip, which owns the dispatch).
#define SCONV_TAPT_INSTANCE(NAME, ...)                                                                         \
    TaptPlan tapt_plan_##NAME(const Problem& p, int split)                                                     \
    {                                                                                                          \
        const Plan pl = plan_tapt<Geom<__VA_ARGS__>>(p, split);                                                \
        TaptPlan t;                                                                                            \
        t.cost = pl.cost; t.nwv = pl.nwv; t.ncs = pl.cfg.NCS; t.nt = pl.cfg.NT; t.nss = pl.nss;                \
        return t;                                                                                              \
    }                                                                                                          \
    int tapt_launch_##NAME(const Problem& p, bool pooled, int split, const float* x, const float* w, float* y, \
                           hipStream_t stream)                                                                 \
    {                                                                                                          \
        const Plan pl = plan_tapt<Geom<__VA_ARGS__>>(p, split);                                                \
        if (pl.cost < 0.0) return SCONV_EUNSUPPORTED;                                                          \
        return launch_tapt<Geom<__VA_ARGS__>>(pl, p, pooled, x, w, y, stream);                                 \
    }

SCONV_TAPT_INSTANCE(5x7k1, 1, 5, 7, 1, 1, false)
SCONV_TAPT_INSTANCE(5x7k1n, 1, 5, 7, 1, 1, false, 1, false)
SCONV_TAPT_INSTANCE(5x7k2, 2, 5, 7, 1, 1, false)
SCONV_TAPT_INSTANCE(7x7k1, 1, 7, 7, 0, 0, false)
SCONV_TAPT_INSTANCE(7x7k2, 2, 7, 7, 0, 0, false)
SCONV_TAPT_INSTANCE(p4x14k1, 1, 4, 14, 1, 0, true)
SCONV_TAPT_INSTANCE(p4x6k1, 1, 4, 6, 1, 1, true)
SCONV_TAPT_INSTANCE(p4x6k2, 2, 4, 6, 1, 1, true)
SCONV_TAPT_INSTANCE(p2x14k2, 2, 2, 14, 1, 0, true)
SCONV_TAPT_INSTANCE(p2x14k1, 1, 2, 14, 1, 0, true)
SCONV_TAPT_INSTANCE(p2x14hk1, 1, 2, 14, 1, 1, true)
SCONV_TAPT_INSTANCE(p2x14hk2, 2, 2, 14, 1, 1, true)
SCONV_TAPT_INSTANCE(s2_3x4k1, 1, 3, 4, 1, 1, false, 2)
SCONV_TAPT_INSTANCE(s2_3x4k2, 2, 3, 4, 1, 1, false, 2)

}  // namespace sconv

// General matrix-core kernel: any kernel size up to 15x15, any stride, padding and grouping, any
// channel count; optional max-pooling epilogue (2x2 / stride 2 in registers, any other window of up
// to 64 results through a copy of the tile in LDS).
//
// Same arithmetic as the wide 3x3 kernel - 64 window rows per wavefront in format order (ECR
// (n, oh, ow), or PECR (n, ph, pw, py, px) for the fused call, Section 6.2), one
// v_mfma_f32_16x16x1 per 16-row block and column, a block skipped when its 16 elements under
// that column are all zero - but the columns col = c*R*S + r*S + s of the window rows
// (Algorithm 1's scan order with the channel loop of Section 7 outside) are walked as one linear
// sequence in chunks of 64, so nothing depends on the kernel's shape at compile time:
//   * the filter chunk w[k][col0 .. col0+63] is staged to LDS as [column][filter] (coalesced
//     256-byte reads of a filter row, one padding word per LDS row against bank conflicts);
//   * what a column (c, r, s) needs from a lane is the same for every window row: one wavefront
//     computes, per chunk, each column's byte offset and the two mask bits of its kernel row and
//     column into a small LDS table; a lane's element under the column is one buffer load at lane
//     offset + column offset.  Whether the tap lies inside the map is one AND + compare of those
//     bits against two per-lane bit masks (valid rows r, valid columns s of the lane's window); a tap outside the map, a column past L or a lane
//     past the last window row loads from an offset beyond the buffer's size, which the
//     hardware answers with zero without touching memory;
//   * elements are loaded one group of 8 columns ahead of the group being multiplied.
// Channel slices split every chunk's columns between the wavefronts of a tile; the reduction and
// the epilogue are the wide kernel's.
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "sconv_wide_common.h"

namespace sconv {

namespace {

using namespace wide;

constexpr int CW = 64;   // columns per staged chunk
constexpr int U = 8;     // columns per prefetch group

struct GenCfg {
    unsigned magicT, magicS;   // floor(2^32 / d) + 1 for d = R*S and d = S (exact quotients for our
                               // ranges); 0 stands for d = 1
    int nchunks;               // ceil(L / CW)
    int nss;                   // workgroups splitting the chunks of a tile; above 1 the results are
                               // raw partial sums, stored into slice blockIdx.z % nss of y
};

// POOL: 0 plain; 1 fused 2x2 / stride 2 pooling (four window rows of a pooling window = the four
// accumulator elements a lane holds for one filter); 2 any pooling window of up to 64 results:
// a tile is 64 / (p_h*p_w) whole pooling windows in PECR order, the window rows of a pooling
// window are consecutive lanes, and the maximum is taken over a copy of the tile in LDS.
template <int KPL, int POOL, int NWV, bool DENSE>
__global__ __launch_bounds__(NWV * 64) void gen_kernel(Problem p, WideCfg cfg, GenCfg gc,
                                                       const float* __restrict__ x,
                                                       const float* __restrict__ w, float* __restrict__ y)
{
    extern __shared__ __align__(16) float lds[];  // two filter buffers; reused for the reduction

    constexpr int KB = 64 * KPL;       // filters per workgroup
    constexpr int KBP = KB + 1;        // LDS row stride (floats)
    constexpr int BUF = CW * KBP;      // floats per buffer
    constexpr int FPT = KB / NWV;      // filters a thread stages per chunk (its column = its lane)
    static_assert(FPT * NWV == KB, "staging must divide evenly");

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ts = wave % cfg.NT;                  // tile slot
    const int cs = wave / cfg.NT;                  // column slice
    const int g = blockIdx.z / gc.nss;
    const int ss = blockIdx.z - g * gc.nss;
    const int ch0 = ss * gc.nchunks / gc.nss, ch1 = (ss + 1) * gc.nchunks / gc.nss;   // this workgroup's chunks
    const int kb0 = blockIdx.y * KB;
    const int tile = blockIdx.x * cfg.NT + ts;
    const bool tile_ok = tile < cfg.ntiles;
    const int HWp = p.H * p.W;
    const int plane = POOL ? p.PH * p.PW : p.OH * p.OW;
    const unsigned T = (unsigned)(p.R * p.S);

    // this lane's window row
    const int P = tile * 64 + lane;
    bool pos_ok = tile_ok && P < cfg.npos;
    int n = 0, oh = 0, ow = 0;
    const int WR = POOL == 2 ? p.ph * p.pw : 4;    // window rows per pooling window
    const int wpt = 64 / WR;                       // pooling windows per tile
    if (POOL == 2) {
        const int wl = lane / WR, e = lane - wl * WR;
        const int widx = tile * wpt + wl;          // pooling window number in the batch
        pos_ok = tile_ok && wl < wpt && widx < cfg.npos;
        if (pos_ok) {
            n = widx / plane;
            const int rem = widx - n * plane;
            const int phi = rem / p.PW, pwi = rem - phi * p.PW;
            const int py = e / p.pw, px = e - py * p.pw;
            oh = phi * p.ps + py;
            ow = pwi * p.ps + px;
        }
    } else if (pos_ok) {
        if (!POOL) {
            n = P / plane;
            const int rem = P - n * plane;
            oh = rem / p.OW;
            ow = rem - oh * p.OW;
        } else {
            const int pp = P >> 2, e = P & 3;      // pooling window, result inside it (py, px)
            n = pp / plane;
            const int rem = pp - n * plane;
            const int ph = rem / p.PW, pw = rem - ph * p.PW;
            oh = 2 * ph + (e >> 1);
            ow = 2 * pw + (e & 1);
        }
    }
    const int ih0 = oh * p.stride - p.pad, iw0 = ow * p.stride - p.pad;
    // bit r: row ih0 + r is inside the map; bit 16 + s: column iw0 + s is.  Bit 31 is never set.
    unsigned rcmask = 0;
    if (pos_ok) {
        for (int r = 0; r < p.R; ++r)
            if (ih0 + r >= 0 && ih0 + r < p.H) rcmask |= 1u << r;
        for (int s = 0; s < p.S; ++s)
            if (iw0 + s >= 0 && iw0 + s < p.W) rcmask |= 0x10000u << s;
    }
    // byte offset of the window's origin from the group's first channel; it wraps for windows that
    // start in the padding and is only ever used together with a tap that lies inside the map
    const unsigned boff0 = 4u * (unsigned)((n * p.C) * HWp + ih0 * p.W + iw0);

    const float* xg = x + (size_t)g * p.Cg * HWp;
    const unsigned xbytes = 4u * (unsigned)((p.N * p.C - g * p.Cg) * HWp);   // from xg to the tensor's end
    const __amdgpu_buffer_rsrc_t xres =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(xg), 0, (int)xbytes, 0x00020000);
    const float* wg = w + ((size_t)g * p.Kg + kb0) * p.L;
    const int kvalid = min(KB, p.Kg - kb0);

    v16f acc[KPL][4];
#pragma unroll
    for (int i = 0; i < KPL; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][q][v] = 0.0f;

    // Filter staging: wavefront wv moves filters wv, wv + NWV, ... of the block, lane l their column
    // col0 + l.  A filter past the group's last one re-reads the last valid filter (its results are
    // never stored); a column past L re-reads column L - 1 (its elements are loaded as zeros, so
    // its instructions are skipped).
    float stage[FPT];
    auto fetch_chunk = [&](int ch) {
        const int col = min(ch * CW + lane, p.L - 1);
#pragma unroll
        for (int i = 0; i < FPT; ++i) {
            const int k = min(wave + i * NWV, kvalid - 1);
            stage[i] = wg[(size_t)k * p.L + col];
        }
    };
    auto store_chunk = [&](float* buf) {
#pragma unroll
        for (int i = 0; i < FPT; ++i) buf[lane * KBP + wave + i * NWV] = stage[i];
    };

    // Column table.  What a column (c, r, s) needs from a lane - the two mask bits of its kernel row
    // and column, and its byte offset from the window's origin - is the same for every window row,
    // so one wavefront works it out per chunk (a lane per column, two multiply-high divisions) and
    // leaves it in LDS, one chunk ahead of the loads that use it; three table buffers rotate, so
    // the chunk being written is never one that a slower wavefront still reads.
    uint2* tab = reinterpret_cast<uint2*>(lds + 2 * BUF);   // [3][CW]: (needed mask bits, byte offset)
    auto write_table = [&](int lc) {   // lc: chunk number counted from the workgroup's first
        if (wave != 0) return;
        const unsigned col = (unsigned)((ch0 + lc) * CW + lane);
        const unsigned c = gc.magicT ? __umulhi(col, gc.magicT) : col;
        const unsigned t = col - c * T;
        const unsigned r = gc.magicS ? __umulhi(t, gc.magicS) : t;
        const unsigned s = t - r * (unsigned)p.S;
        uint2 e;
        e.x = col < (unsigned)p.L ? ((1u << r) | (0x10000u << s)) : 0x80000000u;   // bit 31: no lane has it
        e.y = 4u * (c * (unsigned)HWp + r * (unsigned)p.W + s);
        tab[(lc % 3) * CW + lane] = e;
    };

    // Loads the elements of the U columns starting at column `jb` of the wavefront's share of the
    // chunk whose table is buffer `tb`.  Per lane and column: AND, compare, add, select, load.
    auto issue = [&](int tb, int jb, float (&dst)[U]) {
        const uint2* te = tab + tb * CW + cs * cfg.CPW + jb;   // the same address in every lane
        uint2 e[U];
#pragma unroll
        for (int u = 0; u < U; ++u) e[u] = te[u];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool ok = (rcmask & e[u].x) == e[u].x;
            const unsigned vo = ok ? boff0 + e[u].y : 0x80000000u;
            dst[u] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(xres, (int)vo, 0, 0));
        }
    };

    // Multiplies U columns: elements in xc, filter values from the staged chunk.
    auto compute = [&](const float* buf, int jb, const float (&xc)[U]) {
        unsigned long long m[U];
        unsigned long long any = 0;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            m[u] = __ballot(xc[u] != 0.0f);
            any |= m[u];
        }
        if (!any) return;
        const float* wl = buf + (cs * cfg.CPW + jb) * KBP + lane;
        float wq[2][KPL];
#pragma unroll
        for (int i = 0; i < KPL; ++i) wq[0][i] = wl[64 * i];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (u + 1 < U) {
#pragma unroll
                for (int i = 0; i < KPL; ++i) wq[(u + 1) & 1][i] = wl[(u + 1) * KBP + 64 * i];
            }
            tap_blocks<KPL, DENSE>(xc[u], m[u], wq[u & 1], acc);
        }
    };

    // the wavefront's groups in the order it walks them: CPW / U per chunk
    int ptb = 0, pjb = 0;   // the next group to load: table buffer of its chunk, column in the slice
    auto advance = [&]() {
        pjb += U;
        if (pjb == cfg.CPW) {
            pjb = 0;
            ptb = ptb == 2 ? 0 : ptb + 1;
        }
    };

    fetch_chunk(ch0);
    write_table(0);
    __syncthreads();
    float xa[U], xb[U];
    issue(ptb, pjb, xa);
    advance();
    for (int lc = 0; lc < ch1 - ch0; ++lc) {
        float* buf = lds + (lc & 1) * BUF;
        store_chunk(buf);
        write_table(lc + 1);   // past the last chunk: columns >= L, whose loads read nothing, or the
                               // next workgroup's first columns, whose elements are loaded and dropped
        __syncthreads();
        if (lc + 1 < ch1 - ch0) fetch_chunk(ch0 + lc + 1);
        for (int jb = 0; jb < cfg.CPW; jb += 2 * U) {
            issue(ptb, pjb, xb);
            advance();
            compute(buf, jb, xa);
            issue(ptb, pjb, xa);
            advance();
            compute(buf, jb + U, xb);
        }
    }

    if constexpr (POOL == 2) {
        // the tile, summed over the slices, goes to LDS as [filter register][window row][filter];
        // then every wavefront of the tile takes pooling windows, a lane per filter
        reduce_slices<KPL>(cfg, lds, acc, lane, ts, cs);
        __syncthreads();                 // the reduction's buffers are read, the filter buffers free
        float* tl = lds + (size_t)ts * (KPL * 64 * 64);
        const int bps = 4 / cfg.NCS;
        const int kf = lane & 15, rg = lane >> 4;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (cs != q / bps) continue;
#pragma unroll
            for (int i = 0; i < KPL; ++i)
#pragma unroll
                for (int b = 0; b < 4; ++b)
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        tl[(i * 64 + 16 * q + 4 * rg + e) * 64 + 16 * b + kf] = acc[i][q][4 * b + e];
        }
        __syncthreads();
        if (!tile_ok) return;
        for (int wl = cs; wl < wpt; wl += cfg.NCS) {
            const int widx = tile * wpt + wl;      // uniform
            if (widx >= cfg.npos) break;
            const int nn = widx / plane, rem = widx - nn * plane;
#pragma unroll
            for (int i = 0; i < KPL; ++i) {
                const int k = 64 * i + lane;
                float m = tl[(i * 64 + wl * WR) * 64 + lane];
                for (int e = 1; e < WR; ++e) m = fmaxf(m, tl[(i * 64 + wl * WR + e) * 64 + lane]);
                if (k < kvalid) {                  // bias, then ReLU (both commute with the maximum)
                    const size_t kglob = (size_t)g * p.Kg + kb0 + k;
                    y[((size_t)nn * p.K + kglob) * plane + rem] = fmaxf(m + bias_of(p, kglob), 0.0f);
                }
            }
        }
    } else {
        // split: slice ss of the partial sums (plain layout; the host switched ReLU off)
        finish_tile<KPL, POOL == 1>(p, cfg, lds, acc, lane, ts, cs, tile, tile_ok, g, kb0, kvalid, plane,
                                    y + (size_t)ss * p.N * p.K * plane);
    }
}

struct Plan {
    double cost = -1.0;   // model clocks; negative = not applicable
    WideCfg cfg;
    int nwv = 0;
    int kblocks = 0;
    size_t lds_bytes = 0;
    int nss = 1;          // workgroups per tile along the columns (partial sums through scratch)
    long long wgs1 = 0;   // workgroups of the launch before that split
};

template <int KPL, int POOL, int NWV>
int occupancy(size_t lds_bytes)
{
    int nb = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, gen_kernel<KPL, POOL, NWV, false>, NWV * 64, lds_bytes) !=
            hipSuccess || nb < 1)
        nb = 1;
    return nb;
}

// Decomposition of one launch, with the wide kernel's model: the matrix time of the most loaded
// SIMD plus what does not overlap with it (slice reduction, half of the filter staging, a latency
// penalty when a SIMD holds a single wavefront).  A launch of fewer than 128 tile-workgroups also
// splits the chunks of a tile over NSS workgroups (split: 0 = not allowed, 1 = allowed, 2 =
// required - the plain kernel serving a pooled layer): the smallest power of two that gives every
// compute unit a workgroup and leaves each workgroup two chunks; a second, small kernel adds the
// partial sums.
template <int KPL, int POOL>
Plan plan_geom(const Problem& p, int split)
{
    constexpr int KB = 64 * KPL;
    Plan best;
    WideCfg cfg;
    if (POOL == 2) {
        // whole pooling windows per tile; npos counts pooling windows
        const int wpt = 64 / (p.ph * p.pw);
        cfg.npos = p.N * p.PH * p.PW;
        cfg.ntiles = (cfg.npos + wpt - 1) / wpt;
    } else {
        cfg.npos = POOL ? p.N * p.PH * p.PW * 4 : p.N * p.OH * p.OW;
        cfg.ntiles = (cfg.npos + 63) / 64;
    }
    cfg.vec4 = 0;
    const int kblocks = (p.Kg + KB - 1) / KB;
    const int nchunks = (p.L + CW - 1) / CW;
    const double t_column = 4.0 * KPL * 34.0 + 30.0;
    const double stage_clocks = (double)KB * nchunks * CW * 4.0 / 64.0;

    int pin_nwv = 0, pin_ncs = 0, pin_nss = 0;   // tuning aid: SCONV_GEN_SPLIT="nwv,ncs[,nss]"
    pinned_split("SCONV_GEN_SPLIT", &pin_nwv, &pin_ncs, &pin_nss);
    const bool small = (long long)cfg.ntiles * ((p.Kg + 63) / 64) * p.G < 128;
    const size_t part_bytes = (size_t)p.N * p.K * p.OH * p.OW * sizeof(float);
    auto split_fits = [&](int nss) {
        return !POOL && nss <= nchunks && nss * part_bytes <= split_scratch_bytes() && (long long)p.G * nss <= 65535;
    };
    // a pinned decomposition is priced as it is; the model ranks the unsplit decompositions and
    // splits the winner afterwards
    const int nss = pin_nss ? pin_nss : 1;
    if (nss > 1 && (split == 0 || !split_fits(nss))) return best;
    if (pin_nss == 1 && split == 2) return best;
    // A fused call that is not small keeps its one kernel, the convolution tensor on chip (Section 6.4),
    // also where the plain kernel split two ways with the pooling in the adding kernel measures faster
    // (overlapping 3x3 / stride 2 windows fill the 64-row tiles poorly: 384->256 3x3 in 2 groups @13x13 + that
    // pooling at batch 32, 105 us fused against 92 split); only a pinned decomposition asks for that.
    if (!pin_nss && split == 2 && !small) return best;
    for (int nwv = 4; nwv <= 8; nwv *= 2) {
        if (KPL == 2 && nwv == 4) continue;      // 32 staging registers per thread: not built
        for (int ncs = 1; ncs <= 4; ncs *= 2) {
            const int nt = nwv / ncs;
            if (pin_nwv && (pin_nwv != nwv || pin_ncs != ncs)) continue;
            if (!pin_nwv && nt > 1 && nt / 2 >= cfg.ntiles) continue;   // half of the tile slots empty
            size_t lds_bytes = 2 * (size_t)CW * (KB + 1) * sizeof(float) + 3 * CW * sizeof(uint2);
            const size_t red_bytes = (size_t)nt * 4 * (ncs - 1) * KPL * 16 * 64 * sizeof(float);
            if (red_bytes > lds_bytes) lds_bytes = red_bytes;
            // general pooling windows: a copy of every tile of the workgroup in LDS
            if (POOL == 2 && (size_t)nt * KPL * 64 * 64 * sizeof(float) > lds_bytes)
                lds_bytes = (size_t)nt * KPL * 64 * 64 * sizeof(float);
            if (lds_bytes > 160 * 1024) continue;
            const int occ = nwv == 4 ? occupancy<KPL, POOL, (KPL == 2 ? 8 : 4)>(lds_bytes)
                                     : occupancy<KPL, POOL, 8>(lds_bytes);
            const long long wgs1 = (long long)((cfg.ntiles + nt - 1) / nt) * kblocks * p.G;
            if (nss > 1 && wgs1 >= 512 && current_pin()) continue;   // sconv_tune: not worth a trial
            const long long wgs = wgs1 * nss;
            const long long per_cu = (wgs + 255) / 256;
            const double per_simd = (double)per_cu * nwv / 4.0;
            const double resident = (double)(per_cu < occ ? per_cu : occ) * nwv / 4.0;
            const double wave = (double)nchunks / nss * (CW / ncs) * t_column +
                                (ncs > 1 ? 64.0 * KPL * 20.0 + 800.0 : 0.0);
            double cost = per_simd * wave * (resident < 2.0 ? 1.25 : 1.0) + per_cu * stage_clocks / nss * 0.5 +
                          (nss > 1 ? 9000.0 : 0.0);                            // second kernel
            if (best.cost < 0.0 || cost < best.cost) {
                best.cost = cost;
                best.cfg = cfg;
                best.cfg.NT = nt;
                best.cfg.NCS = ncs;
                best.cfg.CPW = CW / ncs;
                best.nwv = nwv;
                best.kblocks = kblocks;
                best.lds_bytes = lds_bytes;
                best.nss = nss;
                best.wgs1 = wgs1;
            }
        }
    }
    if (!pin_nss && split && small && best.cost >= 0.0) {
        int want = split == 2 ? 2 : 1;
        // down to one chunk per workgroup (measured on 1x1 832->256 @7x7: 8 ways 14.4 us, 4 ways
        // 17.0); two chunks when the adding kernel also pools (it reads every part of a window:
        // 512->256 @28x28 + pool 15.6 against 19.7 us)
        // (kernels of 3x3 and more: two chunks, sconv_tune's pick on four batch-1 layers - 3x3 128 stride 2
        // @56x56 17.1 against 19.7 us, 160->320 @14x14 16.2 against 18.9)
        const int keep = (split == 2 || p.R * p.S >= 9) ? 4 : 2;
        while (want < 16 && best.wgs1 * want < 256 && want * keep <= nchunks) want *= 2;
        if (want > 1 && !split_fits(want)) want = 1;
        if (want == 1 && split == 2) return Plan();
        best.nss = want;
        if (want > 1) best.cost = best.cost / want + 9000.0;
    }
    return best;
}

template <int KPL, int POOL, int NWV, bool DENSE>
int launch_nwv(const Problem& p, const WideCfg& cfg, const GenCfg& gc, dim3 grid, size_t lds_bytes,
               const float* x, const float* w, float* y, hipStream_t stream)
{
    auto kern = gen_kernel<KPL, POOL, NWV, DENSE>;
    static size_t opted = 0;  // dynamic LDS above 48 KiB is opted into (largest request so far)
    if (lds_bytes > opted) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) != hipSuccess)
            return SCONV_ELAUNCH;
        opted = lds_bytes;
    }
    hipLaunchKernelGGL(kern, grid, dim3(NWV * 64), lds_bytes, stream, p, cfg, gc, x, w, y);
    return launch_status();
}

template <int KPL, int POOL, bool DENSE>
int launch_plan(const Plan& pl, const Problem& p, bool pooled, const float* x, const float* w, float* y,
                hipStream_t stream)
{
    const long long gx = (pl.cfg.ntiles + pl.cfg.NT - 1) / pl.cfg.NT;
    const long long gz = (long long)p.G * pl.nss;
    if (gz > 65535 || pl.kblocks > 65535 || gx >= (1LL << 31)) return SCONV_EUNSUPPORTED;
    const dim3 grid((unsigned)gx, (unsigned)pl.kblocks, (unsigned)gz);
    GenCfg gc;
    gc.magicT = p.R * p.S > 1 ? (unsigned)((1ULL << 32) / (unsigned)(p.R * p.S)) + 1u : 0u;
    gc.magicS = p.S > 1 ? (unsigned)((1ULL << 32) / (unsigned)p.S) + 1u : 0u;
    gc.nchunks = (p.L + CW - 1) / CW;
    gc.nss = pl.nss;
    Problem q = p;
    float* out = y;
    if (pl.nss > 1) {
        // raw partial sums of every chunk range into the scratch slices; the second kernel below
        // adds them and applies the epilogue
        if (POOL || pl.nss > gc.nchunks ||
            (size_t)pl.nss * p.N * p.K * p.OH * p.OW * sizeof(float) > split_scratch_bytes())
            return SCONV_EUNSUPPORTED;
        out = split_scratch(stream);
        if (!out) return SCONV_EUNSUPPORTED;
        q.relu = 0;
        q.bias = nullptr;
    } else if (pooled != (POOL != 0)) {
        return SCONV_EUNSUPPORTED;
    }
    WideCfg cfg = pl.cfg;
    const int plane = p.OH * p.OW;
    cfg.vec4 = (!POOL && plane % 4 == 0 && (reinterpret_cast<uintptr_t>(out) & 15) == 0) ? 1 : 0;
    int rc;
    if (KPL == 1 && pl.nwv == 4)
        rc = launch_nwv<KPL, POOL, (KPL == 1 ? 4 : 8), DENSE>(q, cfg, gc, grid, pl.lds_bytes, x, w, out, stream);
    else
        rc = launch_nwv<KPL, POOL, 8, DENSE>(q, cfg, gc, grid, pl.lds_bytes, x, w, out, stream);
    if (rc != SCONV_OK || pl.nss == 1) return rc;
    return launch_split_reduce(p, pooled, out, pl.nss, y, stream);
}

bool shape_ok(const Problem& p, bool pooled)
{
    if (p.R > 15 || p.S > 15) return false;            // one mask bit per kernel row and column
    if (pooled && p.ph * p.pw > 64) return false;      // whole pooling windows in a 64-row tile
    // 32-bit byte offsets into the input with the top bit free, 32-bit window row numbers
    if ((long long)p.N * p.C * p.H * p.W >= (1LL << 29)) return false;
    const long long npos = pooled ? (long long)p.N * p.PH * p.PW * 64 : (long long)p.N * p.OH * p.OW;
    if (npos >= (1LL << 31) - 64) return false;
    // the multiply-high quotients col / (R*S) and t / S are exact while dividend * divisor < 2^32
    const long long T = (long long)p.R * p.S;
    if (((long long)p.L + 2 * CW) * T >= (1LL << 32)) return false;
    return true;
}

struct Candidate {
    const char* name;
    Plan (*plan)(const Problem&, int);
    int (*launch)(const Plan&, const Problem&, bool, const float*, const float*, float*, hipStream_t);
    bool pooled;
    int kpl;
    bool by_model;
    bool any_window = false;   // pooled: serves every pooling window (the others 2x2 / stride 2 only)
};

const Candidate kCandidates[] = {
    {"gk1", plan_geom<1, false>, launch_plan<1, false, false>, false, 1, true},
    {"gk2", plan_geom<2, false>, launch_plan<2, false, false>, false, 2, true},
    {"gpk1", plan_geom<1, true>, launch_plan<1, true, false>, true, 1, true},
    {"gpk2", plan_geom<2, true>, launch_plan<2, true, false>, true, 2, true},
    // the same without zero tests: only when named (sconv_tune's measurement, or a pin)
    {"gk1d", plan_geom<1, false>, launch_plan<1, false, true>, false, 1, false},
    {"gk2d", plan_geom<2, false>, launch_plan<2, false, true>, false, 2, false},
    {"gpk1d", plan_geom<1, true>, launch_plan<1, true, true>, true, 1, false},
    {"gpk2d", plan_geom<2, true>, launch_plan<2, true, true>, true, 2, false},
    // any pooling window of up to 64 results
    {"ggk1", plan_geom<1, 2>, launch_plan<1, 2, false>, true, 1, true, true},
    {"ggk2", plan_geom<2, 2>, launch_plan<2, 2, false>, true, 2, true, true},
};

}  // namespace

const char* const* gen_geoms()
{
    static const char* const names[] = {"gk1", "gk2", "gpk1", "gpk2", "gk1d", "gk2d", "gpk1d", "gpk2d", "ggk1", "ggk2", nullptr};
    return names;
}

bool gen_supported(const Problem& p, bool pooled) { return shape_ok(p, pooled); }

int launch_gen(const Problem& p, bool pooled, const float* x, const float* w, float* y,
               hipStream_t stream)
{
    if (!shape_ok(p, pooled)) return SCONV_EUNSUPPORTED;
    const char* pin = pinned_geom("SCONV_GEN_GEOM");   // tuning aid: candidate name
    const Candidate* best = nullptr;
    Plan best_plan;
    // a split of the chunks across workgroups needs a workspace lent for the stream
    const bool can_split = split_scratch_possible(stream);
    // A pooled layer: first the plain kernel with the split (the second kernel pools), which the
    // model offers for small launches only; the pooled kernel when that does not apply.
    for (int pass = pooled && can_split ? 0 : 1; pass < 2 && !best; ++pass) {
        for (const Candidate& c : kCandidates) {
            if (c.pooled != (pooled && pass == 1)) continue;
            if (c.pooled && c.any_window == (p.ph == 2 && p.pw == 2 && p.ps == 2)) continue;
            if (p.Kg <= 64 * (c.kpl - 1)) continue;
            if (pin ? strcmp(pin, c.name) != 0 : !c.by_model) continue;
            const Plan pl = c.plan(p, c.pooled != pooled ? 2 : (can_split && !c.pooled ? 1 : 0));
            if (pl.cost < 0.0) continue;
            if (!best || pl.cost < best_plan.cost) {
                best = &c;
                best_plan = pl;
            }
        }
    }
    if (!best) return SCONV_EUNSUPPORTED;
    if (env_value("SCONV_TRACE_PLAN"))
        fprintf(stderr, "sconv: gen %s nwv=%d ncs=%d nt=%d nss=%d cost=%.0f\n", best->name, best_plan.nwv,
                best_plan.cfg.NCS, best_plan.cfg.NT, best_plan.nss, best_plan.cost);
    return best->launch(best_plan, p, pooled, x, w, y, stream);
}

}  // namespace sconv

// Wide-granule matrix-core kernel: 3x3 convolutions of any stride and padding, optional
// 2x2 / stride 2 max-pooling epilogue.
//
// The window rows of the paper are taken 64 at a time in format order - ECR order (n, oh, ow) for
// the plain convolution, PECR order (n, ph, pw, py, px) for the fused one, so that the four
// results of a pooling window are neighbours (Section 6.2).  Lane l of a wavefront owns window
// row 64 * tile + l.  For one input channel and one tap (r, s) every lane loads the element its
// window has under that tap (zero outside the map), ballot(x != 0) is the compaction, and
// v_mfma_f32_16x16x1 multiplies 16 neighbouring rows' elements (one 16-lane block of that
// register, broadcast to all four blocks) with the tap's filter values of 64 filters (one per
// lane): 1024 multiply-adds per instruction.  A block whose 16 elements are all zero is skipped
// with one scalar test; scalar work overlaps the matrix pipe, vector work does not, which is why
// the per-channel vector work here is two instructions per tap (the padding select and the
// compare) against 4 * KPL matrix instructions.  The skip granule - 16 window rows under one tap
// of one channel - is coarse: with independent zeros it only pays above 85-90 % zeros, below that
// the kernel runs as a dense direct convolution at the matrix pipe's rate; clustered zeros (dead
// channels, flat regions) are skipped at any ratio.
//
// Accumulator layout of the instruction (checked on the device): element v of lane l belongs to
// filter 16 * (v / 4) + l % 16 and to row 4 * (l / 16) + v % 4 of the broadcast block - four
// consecutive window rows per lane, which is one pooling window in PECR order.
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "sconv_wide_common.h"

namespace sconv {

namespace {

using namespace wide;

template <int KPL_, int R_, int S_, bool POOL_>
struct WGeom {
    static constexpr int KPL = KPL_;            // filters per lane (64 * KPL filters per workgroup)
    static constexpr int R = R_, S = S_, T = R_ * S_;
    static constexpr bool POOL = POOL_;
    static constexpr int KB = 64 * KPL;
    static constexpr int KBP = KB;              // LDS row stride: rows stay 256-byte aligned, so the
                                                // filter reads need no address arithmetic
    static constexpr int CCH = (T == 1) ? 64 : 8;   // channels per staged chunk
    static constexpr int ROWS = CCH * T;        // LDS rows per buffer: (channel, tap)
    static constexpr int BUF = ROWS * KBP;      // floats per buffer
    static constexpr int NACC = 64 * KPL;       // accumulator floats per lane
};

template <class G, int NWV>
__global__ __launch_bounds__(NWV * 64) void wide_kernel(Problem p, WideCfg cfg, const float* __restrict__ x,
                                                   const float* __restrict__ w, float* __restrict__ y)
{
    extern __shared__ __align__(16) float lds[];  // two filter buffers; reused for the reduction

    constexpr int T = G::T;
    const int tid = threadIdx.x;
    constexpr int nthr = NWV * 64;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: scalar registers
    const int ts = wave % cfg.NT;                  // tile slot
    const int cs = wave / cfg.NT;                  // channel slice
    const int g = blockIdx.z;
    const int kb0 = blockIdx.y * G::KB;            // first filter of the block inside the group
    const int tile = blockIdx.x * cfg.NT + ts;
    const bool tile_ok = tile < cfg.ntiles;
    const int HWp = p.H * p.W;
    const int plane = G::POOL ? p.PH * p.PW : p.OH * p.OW;   // stored results per image and filter

    // this lane's window row and the byte offsets of its taps inside a channel plane set
    const int P = tile * 64 + lane;
    const bool pos_ok = tile_ok && P < cfg.npos;
    int n = 0, oh = 0, ow = 0;
    if (pos_ok) {
        if (!G::POOL) {
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
    unsigned boff[T];   // 0 (a valid address) where the tap lies outside the map
    bool ok[T];
#pragma unroll
    for (int t = 0; t < T; ++t) {
        const int ih = oh * p.stride - p.pad + t / G::S, iw = ow * p.stride - p.pad + t % G::S;
        ok[t] = pos_ok && ih >= 0 && ih < p.H && iw >= 0 && iw < p.W;
        boff[t] = ok[t] ? 4u * (unsigned)((n * p.C) * HWp + ih * p.W + iw) : 0u;
    }
    const float* xg = x + (size_t)g * p.Cg * HWp;
    const float* wg = w + ((size_t)g * p.Kg + kb0) * p.L;  // filter k of the block: wg + k*L
    const int kvalid = min(G::KB, p.Kg - kb0);

    v16f acc[G::KPL][4];
#pragma unroll
    for (int i = 0; i < G::KPL; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][q][v] = 0.0f;

    // Filter staging.  A chunk is KB filters x ROWS = CCH*T consecutive floats of each filter.
    // TPF threads share one filter, each moving EPT consecutive floats, so the global offset and
    // the LDS index are one per-thread base plus compile-time steps.  A filter past the group's
    // last one (ragged last block) re-reads the last valid filter: its lanes compute values that
    // are never stored, and no address leaves the tensor.
    constexpr int TPF = nthr / G::KB;
    constexpr int EPT = G::ROWS / TPF;
    constexpr int VW = (EPT % 4 == 0) ? 4 : (EPT % 2 == 0) ? 2 : 1;   // floats per staging load
    static_assert(TPF * G::KB == nthr && EPT * TPF == G::ROWS && EPT % VW == 0, "staging must divide evenly");
    typedef float vst __attribute__((ext_vector_type(VW)));
    vst stage[EPT / VW];
    const int sk = tid / TPF, ssub = tid - sk * TPF;
    const unsigned sgoff = (unsigned)(min(sk, kvalid - 1) * p.L + ssub * EPT);
    const int sloff = ssub * EPT * G::KBP + sk;
    auto fetch_chunk = [&](int c0) {
        const vst* base = reinterpret_cast<const vst*>(wg + c0 * T + sgoff);
#pragma unroll
        for (int i = 0; i < EPT / VW; ++i) stage[i] = base[i];
    };
    auto store_chunk = [&](float* buf) {
#pragma unroll
        for (int i = 0; i < EPT; ++i) buf[sloff + i * G::KBP] = stage[i / VW][i % VW];
    };
    auto load_x = [&](int c, float (&dst)[T]) {
        // uniform base; a prefetch past the last channel re-reads the last one
        const char* base = (const char*)(xg + (size_t)min(c, p.Cg - 1) * HWp);
#pragma unroll
        for (int t = 0; t < T; ++t) {
            // the offset is made opaque here so that its zero extension stays next to the load:
            // the load then takes the scalar base and the 32-bit lane offset as they are
            asm volatile("" : "+v"(boff[t]));
            dst[t] = *(const float*)(base + boff[t]);
        }
    };

    const int nchunks = p.Cg / G::CCH;
    // the wavefront's channels in the order it walks them: CPW (even) per chunk
    auto channel_at = [&](int k) { return (k / cfg.CPW) * G::CCH + cs * cfg.CPW + k % cfg.CPW; };
    auto load_w = [&](const float* buf, int cc, float (&dst)[T][G::KPL]) {
        const float* wl = buf + (cs * cfg.CPW + cc) * T * G::KBP + lane;
#pragma unroll
        for (int t = 0; t < T; ++t)
#pragma unroll
            for (int i = 0; i < G::KPL; ++i) dst[t][i] = wl[t * G::KBP + 64 * i];
    };
    // one channel: elements in xq (loaded two channels ago; refilled here with the channel two
    // ahead), filters in wr
    auto channel = [&](float (&xq)[T], int knext, const float (&wr)[T][G::KPL]) {
        float cur[T];
        unsigned long long m[T];
        unsigned long long any = 0;
#pragma unroll
        for (int t = 0; t < T; ++t) {
            cur[t] = ok[t] ? xq[t] : 0.0f;
            m[t] = __ballot(cur[t] != 0.0f);
            any |= m[t];
        }
        load_x(channel_at(knext), xq);
        if (any) {
#pragma unroll
            for (int t = 0; t < T; ++t) tap_blocks<G::KPL>(cur[t], m[t], wr[t], acc);
        }
    };

    fetch_chunk(0);
    float xa[T], xb[T];
    load_x(channel_at(0), xa);
    load_x(channel_at(1), xb);
    int k = 0;
    for (int ch = 0; ch < nchunks; ++ch) {
        float* buf = lds + (ch & 1) * G::BUF;
        store_chunk(buf);
        __syncthreads();
        if (ch + 1 < nchunks) fetch_chunk((ch + 1) * G::CCH);

        float wa[T][G::KPL], wb[T][G::KPL];
        load_w(buf, 0, wa);
        for (int cc = 0; cc < cfg.CPW; cc += 2, k += 2) {
            load_w(buf, cc + 1, wb);
            channel(xa, k + 2, wa);
            if (cc + 2 < cfg.CPW) load_w(buf, cc + 2, wa);
            channel(xb, k + 3, wb);
        }
    }

    finish_tile<G::KPL, G::POOL>(p, cfg, lds, acc, lane, ts, cs, tile, tile_ok, g, kb0, kvalid, plane, y);
}

template <class G, int NWV>
int occupancy(size_t lds_bytes)
{
    int nb = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, wide_kernel<G, NWV>, NWV * 64, lds_bytes) !=
            hipSuccess || nb < 1)
        nb = 1;
    return nb;
}

template <class G, int NWV>
int launch_nwv(const Problem& p, const WideCfg& cfg, dim3 grid, size_t lds_bytes, const float* x,
               const float* w, float* y, hipStream_t stream)
{
    auto kern = wide_kernel<G, NWV>;
    static size_t opted = 0;  // dynamic LDS above 48 KiB is opted into (largest request so far)
    if (lds_bytes > opted) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) != hipSuccess)
            return SCONV_ELAUNCH;
        opted = lds_bytes;
    }
    hipLaunchKernelGGL(kern, grid, dim3(NWV * 64), lds_bytes, stream, p, cfg, x, w, y);
    return launch_status();
}

struct Plan {
    double cost = -1.0;   // model clocks; negative = not applicable
    WideCfg cfg;
    int nwv = 0;
    int kblocks = 0;
    size_t lds_bytes = 0;
};

// Decomposition of one launch: ntiles x kblocks x groups tile-wavefronts, each walking Cg
// channels; NCS wavefronts split the channels of a tile, NT tiles share the staged filters of a
// workgroup.  The matrix pipe of a SIMD is saturated by one or two wavefronts, so the model is the
// matrix time of the most loaded SIMD plus what does not overlap with it: the slice reduction,
// filter staging (counted at half), and a latency penalty when a SIMD holds a single wavefront.
template <class G>
Plan plan_geom(const Problem& p)
{
    Plan best;
    WideCfg cfg;
    cfg.npos = G::POOL ? p.N * p.PH * p.PW * 4 : p.N * p.OH * p.OW;
    cfg.ntiles = (cfg.npos + 63) / 64;
    cfg.vec4 = 0;
    const int kblocks = (p.Kg + G::KB - 1) / G::KB;
    const double t_channel = G::T * (4.0 * G::KPL * 34.0 + 9.0) + 60.0;
    const double stage_clocks = (double)G::KB * p.Cg * G::T * 4.0 / 64.0;

    int pin_nwv = 0, pin_ncs = 0;   // tuning aid: SCONV_WIDE_SPLIT="nwv,ncs"
    pinned_split("SCONV_WIDE_SPLIT", &pin_nwv, &pin_ncs);
    for (int nwv = 4; nwv <= 8; nwv *= 2) {
        if (nwv * 64 < G::KB || G::ROWS % (nwv * 64 / G::KB)) continue;
        for (int ncs = 1; ncs <= 4 && 2 * ncs <= G::CCH; ncs *= 2) {   // an even number of channels per slice
            const int nt = nwv / ncs;
            if (pin_nwv && (pin_nwv != nwv || pin_ncs != ncs)) continue;
            if (!pin_nwv && nt > 1 && nt / 2 >= cfg.ntiles) continue;   // half of the tile slots empty
            size_t lds_bytes = 2 * (size_t)G::BUF * sizeof(float);
            const size_t red_bytes = (size_t)nt * 4 * (ncs - 1) * G::KPL * 16 * 64 * sizeof(float);
            if (red_bytes > lds_bytes) lds_bytes = red_bytes;
            if (lds_bytes > 160 * 1024) continue;
            const int occ = nwv == 4 ? occupancy<G, 4>(lds_bytes) : occupancy<G, 8>(lds_bytes);
            const long long wgs = (long long)((cfg.ntiles + nt - 1) / nt) * kblocks * p.G;
            const long long per_cu = (wgs + 255) / 256;                 // most loaded compute unit
            const double per_simd = (double)per_cu * nwv / 4.0;          // its wavefronts per SIMD
            const double resident = (double)(per_cu < occ ? per_cu : occ) * nwv / 4.0;
            const double wave = (double)p.Cg / ncs * t_channel + (ncs > 1 ? G::NACC * 20.0 + 800.0 : 0.0);
            double cost = per_simd * wave * (resident < 2.0 ? 1.25 : 1.0) + per_cu * stage_clocks * 0.5;
            if (best.cost < 0.0 || cost < best.cost) {
                best.cost = cost;
                best.cfg = cfg;
                best.cfg.NT = nt;
                best.cfg.NCS = ncs;
                best.cfg.CPW = G::CCH / ncs;
                best.nwv = nwv;
                best.kblocks = kblocks;
                best.lds_bytes = lds_bytes;
            }
        }
    }
    return best;
}

template <class G>
int launch_plan(const Plan& pl, const Problem& p, const float* x, const float* w, float* y,
                hipStream_t stream)
{
    const long long gx = (pl.cfg.ntiles + pl.cfg.NT - 1) / pl.cfg.NT;
    if (p.G > 65535 || pl.kblocks > 65535 || gx >= (1LL << 31)) return SCONV_EUNSUPPORTED;
    const dim3 grid((unsigned)gx, (unsigned)pl.kblocks, (unsigned)p.G);
    WideCfg cfg = pl.cfg;
    const int plane = p.OH * p.OW;
    cfg.vec4 = (!G::POOL && plane % 4 == 0 && (reinterpret_cast<uintptr_t>(y) & 15) == 0) ? 1 : 0;
    if constexpr (256 >= G::KB && G::ROWS % (256 / G::KB) == 0) {
        if (pl.nwv == 4) return launch_nwv<G, 4>(p, cfg, grid, pl.lds_bytes, x, w, y, stream);
    }
    return launch_nwv<G, 8>(p, cfg, grid, pl.lds_bytes, x, w, y, stream);
}

using W33_1 = WGeom<1, 3, 3, false>;
using W33_2 = WGeom<2, 3, 3, false>;
using WP33_1 = WGeom<1, 3, 3, true>;
using WP33_2 = WGeom<2, 3, 3, true>;

bool shape_ok(const Problem& p, bool pooled)
{
    if (p.R != 3 || p.S != 3) return false;
    if (p.Cg % 8) return false;                       // whole staged chunks of channels only
    if (pooled && (p.ph != 2 || p.pw != 2 || p.ps != 2)) return false;
    // 32-bit byte offsets into the input, 32-bit window row numbers
    if ((long long)p.N * p.C * p.H * p.W >= (1LL << 30)) return false;
    const long long npos = pooled ? (long long)p.N * p.PH * p.PW * 4 : (long long)p.N * p.OH * p.OW;
    if (npos >= (1LL << 31) - 64) return false;
    return true;
}

struct Candidate {
    const char* name;
    Plan (*plan)(const Problem&);
    int (*launch)(const Plan&, const Problem&, const float*, const float*, float*, hipStream_t);
    bool pooled;
    int kpl;              // filters per lane: needs more than 64*(kpl-1) filters in the group
};

const Candidate kCandidates[] = {
    {"w33k1", plan_geom<W33_1>, launch_plan<W33_1>, false, 1},
    {"w33k2", plan_geom<W33_2>, launch_plan<W33_2>, false, 2},
    {"wp33k1", plan_geom<WP33_1>, launch_plan<WP33_1>, true, 1},
    {"wp33k2", plan_geom<WP33_2>, launch_plan<WP33_2>, true, 2},
};

}  // namespace

const char* const* wide_geoms()
{
    static const char* const names[] = {"w33k1", "w33k2", "wp33k1", "wp33k2", nullptr};
    return names;
}

bool wide_supported(const Problem& p, bool pooled) { return shape_ok(p, pooled); }

int launch_wide(const Problem& p, bool pooled, const float* x, const float* w, float* y,
                hipStream_t stream)
{
    if (!shape_ok(p, pooled)) return SCONV_EUNSUPPORTED;
    if (reinterpret_cast<uintptr_t>(w) & 15) return SCONV_EUNSUPPORTED;   // filter staging loads 16 bytes
    const char* pin = pinned_geom("SCONV_WIDE_GEOM");   // tuning aid: candidate name
    const Candidate* best = nullptr;
    Plan best_plan;
    for (const Candidate& c : kCandidates) {
        if (c.pooled != pooled) continue;
        if (p.Kg <= 64 * (c.kpl - 1)) continue;
        if (pin && strcmp(pin, c.name) != 0) continue;
        Plan pl = c.plan(p);
        if (pl.cost < 0.0) continue;
        // measured on eight layer shapes: one filter per lane (twice the wavefronts, half the
        // registers) is 3-45 % faster than two in seven of them and 3 % slower in one; the model's
        // matrix and staging clocks alone price the two alike
        if (c.kpl == 2) pl.cost *= 1.25;
        if (!best || pl.cost < best_plan.cost) {
            best = &c;
            best_plan = pl;
        }
    }
    if (!best) return SCONV_EUNSUPPORTED;
    return best->launch(best_plan, p, x, w, y, stream);
}

}  // namespace sconv

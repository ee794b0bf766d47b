// Device code shared by the element-stationary 3x3 kernels (sconv_tap.hip: filters staged through LDS;
// sconv_tapt.hip: filters read from a transposed copy): tile geometry, the position-specialised
// product code, the tile epilogue and the slice reduction.  Included inside namespace sconv { namespace { .
#pragma once

#include <utility>

template <int KPL_, int TH_, int TW_, int HH_, int HW_, bool POOL_, int STRIDE_ = 1, bool GT_ = true>
struct Geom {
    static constexpr bool GT = GT_;             // test four positions at once before testing each
    static constexpr int KPL = KPL_;            // filters per lane
    static constexpr int TH = TH_, TW = TW_;    // output tile
    static constexpr int HH = HH_, HW = HW_;    // 1: tile carries a halo row/column on each side;
                                                // 0: tile spans the whole map in that direction
    static constexpr bool POOL = POOL_;
    static constexpr int STRIDE = STRIDE_;      // convolution stride (2 only with halo on both axes)
    // input rows oh0*STRIDE - HH .. (oh0+TH-1)*STRIDE + 1 (pad 1, 3 taps)
    static constexpr int IH = (TH - 1) * STRIDE + 1 + 2 * HH, IW = (TW - 1) * STRIDE + 1 + 2 * HW;
    static constexpr int NPOS = IH * IW;
    static constexpr int NX = (NPOS + 63) / 64;  // input registers per channel
    static constexpr int ACC = TH * TW;
    static constexpr int KB = 64 * KPL;          // filters per workgroup
    static constexpr int KBP = KB + 1;           // LDS row stride (odd: conflict-free transposed writes)
    static constexpr int CCH = 16 / KPL;         // channels per staged chunk
    static constexpr int ROWS = CCH * 9;         // LDS rows per buffer
    static constexpr int BUF = ROWS * KBP;       // floats per buffer
    // 16 wavefronts per workgroup leave 128 registers per lane; tiles whose accumulators and
    // filter registers do not fit run with 8 wavefronts (up to 256 registers) instead.
    static constexpr int MAXW = (KPL * ACC + 9 * KPL + 26 > 128) ? 8 : 16;
};

struct TapCfg {
    int NT, NCS;        // wavefronts per workgroup = NT spatial tiles x NCS channel slices
    int CPW;            // channels per wavefront per chunk = CCH / NCS
    int tiles_x, tiles_y, ntiles;
    int NSS;            // workgroups splitting the channels of a tile; above 1 the results are raw
                        // partial sums, stored into slice blockIdx.z % NSS of y
    int RW;             // slices whose sums fit into LDS side by side during the slice reduction
    int wt_blocks = 0;  // transposed-filter kernel: blocks of 64 filters per group in the transposed layout
    int xcd_remap = 0;  // transposed-filter kernel: XCD groups along the filter blocks (1, 2, 4, 8; 0 = as launched)
};

// One input position P of the tile: test its mask bit, broadcast the value, run its products.
template <class G, int P>
__device__ __forceinline__ void position(const unsigned (&mask)[2 * G::NX],
                                         const float (&xv)[G::NX], float (&acc)[G::KPL][G::ACC],
                                         const float (&wr)[G::KPL][9])
{
    constexpr int q = P / 64, l = P % 64;
    constexpr int ih = P / G::IW, iw = P % G::IW;
    if (mask[P / 32] & (1u << (P % 32))) {   // one scalar bit test per position
        const float v = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(xv[q]), l));
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            // x row xr = oh0*STRIDE - HH + ih feeds the output row oh with oh*STRIDE - 1 + r = xr
            const int nr = ih - G::HH + 1 - r;
            if (nr < 0 || nr % G::STRIDE != 0 || nr / G::STRIDE >= G::TH) continue;
            const int orow = nr / G::STRIDE;
#pragma unroll
            for (int s = 0; s < 3; ++s) {
                const int nc = iw - G::HW + 1 - s;
                if (nc < 0 || nc % G::STRIDE != 0 || nc / G::STRIDE >= G::TW) continue;
                const int ocol = nc / G::STRIDE;
#pragma unroll
                for (int i = 0; i < G::KPL; ++i)
                    acc[i][orow * G::TW + ocol] = fmaf(v, wr[i][r * 3 + s], acc[i][orow * G::TW + ocol]);
            }
        }
    }
}

// Four consecutive positions: one scalar test of their four mask bits first.  With 70 % zeros or
// more a quarter or more of the groups is empty and costs one test instead of four.
template <class G, int P4>
__device__ __forceinline__ void position_group(const unsigned (&mask)[2 * G::NX],
                                               const float (&xv)[G::NX], float (&acc)[G::KPL][G::ACC],
                                               const float (&wr)[G::KPL][9])
{
    constexpr int P0 = 4 * P4;
    constexpr int cnt = (P0 + 4 <= G::NPOS) ? 4 : G::NPOS - P0;
    constexpr unsigned bits = ((1u << cnt) - 1u) << (P0 % 32);   // P0 % 4 == 0: one mask word
    if (!G::GT || (mask[P0 / 32] & bits)) {
        position<G, P0>(mask, xv, acc, wr);
        if constexpr (cnt > 1) position<G, P0 + 1>(mask, xv, acc, wr);
        if constexpr (cnt > 2) position<G, P0 + 2>(mask, xv, acc, wr);
        if constexpr (cnt > 3) position<G, P0 + 3>(mask, xv, acc, wr);
    }
}

template <class G, int... P4s>
__device__ __forceinline__ void all_positions(std::integer_sequence<int, P4s...>,
                                              const unsigned (&mask)[2 * G::NX],
                                              const float (&xv)[G::NX],
                                              float (&acc)[G::KPL][G::ACC],
                                              const float (&wr)[G::KPL][9])
{
    (position_group<G, P4s>(mask, xv, acc, wr), ...);
}

// Epilogue of a tile: the lane owns filters kb0 + lane + 64*i.  Plain tiles store (slice ss of the
// partial sums when the launch is split), pooled tiles reduce each 2x2 window first.
template <class G>
__device__ __forceinline__ void store_tile(const Problem& p, float (&acc)[G::KPL][G::ACC], float* __restrict__ y,
                                           int ss, int n, int g, int kb0, int kvalid, int oh0, int ow0, int lane)
{
    if (p.bias) {   // (a branch of its own: without a bias the epilogue is exactly the plain one)
#pragma unroll
        for (int i = 0; i < G::KPL; ++i) {
            const int k = lane + 64 * i;
            const float bk = k < kvalid ? p.bias[(size_t)g * p.Kg + kb0 + k] : 0.0f;
#pragma unroll
            for (int a = 0; a < G::ACC; ++a) acc[i][a] += bk;
        }
    }
    if (!G::POOL) {
        const int plane = p.OH * p.OW;
        y += (size_t)ss * p.N * p.K * plane;       // split: slice ss of the partial sums (p.relu is off)
#pragma unroll
        for (int i = 0; i < G::KPL; ++i) {
            const int k = lane + 64 * i;
            if (k >= kvalid) continue;
            float* yk = y + ((size_t)n * p.K + (size_t)g * p.Kg + kb0 + k) * plane;
#pragma unroll
            for (int a = 0; a < G::ACC; ++a) {
                const int oh = oh0 + a / G::TW, ow = ow0 + a % G::TW;
                if (oh < p.OH && ow < p.OW) {
                    float v = acc[i][a];
                    if (p.relu) v = fmaxf(v, 0.0f);
                    yk[oh * p.OW + ow] = v;
                }
            }
        }
    } else {
        // 2x2 / stride 2 windows never straddle tiles (TH, TW even, tile origins even)
        const int plane = p.PH * p.PW;
#pragma unroll
        for (int i = 0; i < G::KPL; ++i) {
            const int k = lane + 64 * i;
            if (k >= kvalid) continue;
            float* yk = y + ((size_t)n * p.K + (size_t)g * p.Kg + kb0 + k) * plane;
#pragma unroll
            for (int a = 0; a < (G::TH / 2) * (G::TW / 2); ++a) {
                const int pr = a / (G::TW / 2), pc = a % (G::TW / 2);
                const int phh = oh0 / 2 + pr, pww = ow0 / 2 + pc;
                if (phh < p.PH && pww < p.PW) {
                    const int b = (2 * pr) * G::TW + 2 * pc;
                    float m = fmaxf(fmaxf(acc[i][b], acc[i][b + 1]),
                                    fmaxf(acc[i][b + G::TW], acc[i][b + G::TW + 1]));
                    yk[phh * p.PW + pww] = fmaxf(m, 0.0f);
                }
            }
        }
    }
}

// Adds the partial sums of a tile's channel slices through LDS, into slice 0's registers.  Of the
// `active` slices still holding sums, the top nw hand theirs to the bottom nw, as many at a time as
// the buffer has room for (cfg.RW slices of NT tiles): a tree of log2(NCS) steps when half of the
// slices fit, one slice per step when only one does.  The pairing depends on the decomposition alone,
// so results are reproducible.  Every wavefront of the workgroup calls it (it holds barriers).
template <class G>
__device__ __forceinline__ void reduce_slices(const TapCfg& cfg, float* red /* [RW][NT][KPL*ACC][64] */,
                                              float (&acc)[G::KPL][G::ACC], int ts, int cs, int lane)
{
    if (cfg.NCS <= 1) return;
    constexpr int NACC = G::KPL * G::ACC;
    int active = cfg.NCS;
    while (active > 1) {
        const int nw = min(cfg.RW, active / 2);
        const int first = active - nw;   // first writing slice
        __syncthreads();
        if (cs >= first && cs < active) {
            float* dst = red + (size_t)((cs - first) * cfg.NT + ts) * NACC * 64 + lane;
#pragma unroll
            for (int i = 0; i < G::KPL; ++i)
#pragma unroll
                for (int a = 0; a < G::ACC; ++a) dst[(i * G::ACC + a) * 64] = acc[i][a];
        }
        __syncthreads();
        if (cs < nw) {
            const float* src = red + (size_t)(cs * cfg.NT + ts) * NACC * 64 + lane;
#pragma unroll
            for (int i = 0; i < G::KPL; ++i)
#pragma unroll
                for (int a = 0; a < G::ACC; ++a) acc[i][a] += src[(i * G::ACC + a) * 64];
        }
        active = first;
    }
}

// Plan of one launch: the split of a geometry's work over wavefronts and its modelled cost.
struct Plan {
    double cost = -1.0;   // model clocks; negative = not applicable
    TapCfg cfg;
    int nwv = 0;
    int kblocks = 0;
    size_t lds_bytes = 0;
    int nss = 1;          // workgroups per tile along the channels (partial sums through scratch)
    long long wgs1 = 0;   // workgroups of the launch before that split
    int split_mode = 0;   // the split argument the plan was made with (transposed-filter candidates)
};

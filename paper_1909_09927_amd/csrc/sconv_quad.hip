// Matrix-core variant of the element-stationary kernel for 3x3 / stride 1 / pad 1 convolutions,
// with the optional 2x2 / stride 2 max-pooling epilogue.
//
// Same arithmetic and the same bookkeeping as the vector kernel (lanes hold output channels, the
// filters of one input channel stay in registers while that channel's input tile is processed,
// ballot(x != 0) is the compaction), but the products are issued four input positions at a time
// on the matrix pipe: v_mfma_f32_4x4x1 computes 16 independent 4x4 outer products
// D[b][i][j] += A[b][i] * B[b][j].  Here j (with the block number b) is the lane's filter, B is
// the lane's filter value for one tap, and A - broadcast from one 4-lane block of the input
// register to all blocks - holds four horizontally adjacent input elements, so one instruction
// adds tap (r, s) of four adjacent inputs to the four adjacent outputs of an accumulator quad
// for 64 filters: 256 multiply-adds in the time the vector pipe needs for 128.  It is full fp32
// arithmetic.  Zero skipping works on the six input elements that feed one accumulator quad from
// one input row (four outputs times three tap columns): when their six mask bits are all clear,
// one scalar test replaces up to nine matrix instructions per filter register (probability z^6
// for i.i.d. zero ratio z); finer tests cost more issue slots than the instructions they save.
//
// Input tile layout: rows of RP lanes (RP = 16 or 32, TW + 2 of them used); the three tap
// columns s = 0, 1, 2 need the register shifted by s lanes so that the four wanted elements sit
// on a 4-lane block boundary; the shifted copies come from DPP wavefront shifts.
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <utility>

#include "sconv_internal.h"

namespace sconv {

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));

template <int KPL_, int TH_, int RP_, int NQ_, int TW_, bool POOL_, bool NOSKIP_ = false>
struct Geom {
    // NOSKIP: no zero tests at all - the dense form, for maps with so few zeros that hardly a
    // 6-element group is empty (z^6: 5 % of the groups at 60 % zeros) and the tests with their
    // branches cost more issue time than the skipped instructions save.
    static constexpr bool NOSKIP = NOSKIP_;
    static constexpr int KPL = KPL_;            // filters per lane
    static constexpr int TH = TH_;              // output rows of the tile
    static constexpr int RP = RP_;              // lanes per input row
    static constexpr int NQ = NQ_;              // accumulator quads per output row
    static constexpr int TW = TW_;              // valid output columns (<= 4*NQ, TW + 2 <= RP)
    static constexpr bool POOL = POOL_;
    static constexpr int IH = TH + 2;           // input rows oh0 - 1 .. oh0 + TH
    static constexpr int NPOS = IH * RP;
    static constexpr int NX = (NPOS + 63) / 64;  // input registers per channel
    static constexpr int ACC = TH * NQ * 4;      // accumulator floats per filter
    static constexpr int KB = 64 * KPL;          // filters per workgroup
    static constexpr int KBP = KB;               // LDS row stride: 256-byte aligned rows, so the filter
                                                 // reads need no address arithmetic
    static constexpr int CCH = 16 / KPL;         // channels per staged chunk
    static constexpr int ROWS = CCH * 9;         // LDS rows per buffer
    static constexpr int BUF = ROWS * KBP;       // floats per buffer
    static constexpr int MAXW = (KPL * ACC + 9 * KPL + 3 * NX + 26 > 128) ? 8 : 16;
    static_assert(64 % RP == 0 && TW + 2 <= RP && TW <= 4 * NQ, "tile layout");
};

struct TapCfg {
    int NT, NCS;        // wavefronts per workgroup = NT spatial tiles x NCS channel slices
    int CPW;            // channels per wavefront per chunk = CCH / NCS
    int tiles_x, tiles_y, ntiles;
    int tr;             // plain epilogue: transpose each output row through LDS (it fits)
    int NSS;            // workgroups splitting the channels of a tile; above 1 the results are raw
                        // partial sums, stored into slice blockIdx.z % NSS of y
};

// x[l] <- x[l + 1] over the whole wavefront (lane 63 gets 0)
__device__ __forceinline__ float wave_shl1(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x130, 0xf, 0xf, true));
}

// One accumulator quad's worth of input: row IHI of the tile, output quad CQ.  Its three tap
// columns read lanes b0 .. b0 + 5 of input register Q (b0 on a block boundary); in the copy
// shifted by s lanes the four elements of tap column s are block number b0 / 4.  One scalar test
// of those six mask bits guards the up to nine matrix instructions (three tap columns times the
// tap rows whose output row lies in the tile) of each of the lane's filters.
template <class G, int IHI, int CQ>
__device__ __forceinline__ void quad_group(const unsigned (&mask)[2 * G::NX], const float (&xs)[3],
                                           v4f (&acc)[G::KPL][G::TH * G::NQ], const float (&wr)[G::KPL][9])
{
    constexpr int P0 = IHI * G::RP + CQ * 4;     // lane position of the block in the tile
    constexpr int Q = P0 / 64, B0 = P0 % 64;
    constexpr unsigned long long bits = (B0 + 5 < 64) ? (0x3Full << B0) : ((~0ull) << B0);
    constexpr unsigned lo = (unsigned)bits, hi = (unsigned)(bits >> 32);
    unsigned hit = 0;
    if (lo) hit |= mask[2 * Q] & lo;
    if (hi) hit |= mask[2 * Q + 1] & hi;
    if (G::NOSKIP || hit) {
#pragma unroll
        for (int s = 0; s < 3; ++s) {
#pragma unroll
            for (int r = 0; r < 3; ++r) {
                // input row oh0 - 1 + IHI feeds output row oh0 + IHI - r through tap row r
                const int orow = IHI - r;
                if (orow < 0 || orow >= G::TH) continue;
#pragma unroll
                for (int i = 0; i < G::KPL; ++i)
                    acc[i][orow * G::NQ + CQ] = __builtin_amdgcn_mfma_f32_4x4x1f32(
                        xs[s], wr[i][r * 3 + s], acc[i][orow * G::NQ + CQ], 4, B0 / 4, 0);
            }
        }
    }
}

// One input row of the tile.  The row's lanes sit in one input register; the copies shifted by one
// and two lanes are made here, right before their use, so that only one register's copies are alive.
template <class G, int IHI, int... CQs>
__device__ __forceinline__ void quad_row(std::integer_sequence<int, CQs...>,
                                         const unsigned (&mask)[2 * G::NX], const float (&x0)[G::NX],
                                         v4f (&acc)[G::KPL][G::TH * G::NQ], const float (&wr)[G::KPL][9])
{
    constexpr int Q = IHI * G::RP / 64;
    float xs[3];
    xs[0] = x0[Q];
    xs[1] = wave_shl1(xs[0]);
    xs[2] = wave_shl1(xs[1]);
    (quad_group<G, IHI, CQs>(mask, xs, acc, wr), ...);
}

template <class G, int... IHIs>
__device__ __forceinline__ void all_quads(std::integer_sequence<int, IHIs...>,
                                          const unsigned (&mask)[2 * G::NX], const float (&x0)[G::NX],
                                          v4f (&acc)[G::KPL][G::TH * G::NQ], const float (&wr)[G::KPL][9])
{
    (quad_row<G, IHIs>(std::make_integer_sequence<int, G::NQ>{}, mask, x0, acc, wr), ...);
}

template <class G, int NWV>
__global__ __launch_bounds__(NWV * 64) void quad_kernel(Problem p, TapCfg cfg, const float* __restrict__ x,
                                                   const float* __restrict__ w, float* __restrict__ y)
{
    extern __shared__ __align__(16) float lds[];  // two filter buffers; reused for the reduction

    const int tid = threadIdx.x;
    constexpr int nthr = NWV * 64;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: scalar registers
    const int ts = wave % cfg.NT;                  // spatial tile slot
    const int cs = wave / cfg.NT;                  // channel slice
    const int ss = blockIdx.z % cfg.NSS;           // channel range of the workgroup
    const int ng = blockIdx.z / cfg.NSS;
    const int n = ng / p.G;
    const int g = ng - n * p.G;
    if (!G::POOL) y += (size_t)ss * p.N * p.K * p.OH * p.OW;   // split: slice ss of the partial sums
    const int kb0 = blockIdx.y * G::KB;            // first filter of the block inside the group
    const int tile = blockIdx.x * cfg.NT + ts;
    const bool tile_ok = tile < cfg.ntiles;
    const int ty = tile / cfg.tiles_x, tx = tile - ty * cfg.tiles_x;
    const int oh0 = ty * G::TH, ow0 = tx * G::TW;
    const int HWp = p.H * p.W;

    // this lane's input positions (one per input register)
    unsigned xoff[G::NX];   // offset inside a channel plane; 0 (a valid address) when unused
    bool xok[G::NX];
#pragma unroll
    for (int q = 0; q < G::NX; ++q) {
        const int P = q * 64 + lane;
        const int ih = P / G::RP, ic = P - ih * G::RP;
        const int xr = oh0 - 1 + ih, xc = ow0 - 1 + ic;
        xok[q] = tile_ok && ih < G::IH && ic < G::TW + 2 && xr >= 0 && xr < p.H && xc >= 0 && xc < p.W;
        xoff[q] = xok[q] ? (unsigned)(xr * p.W + xc) : 0u;
    }
    const float* xg = x + ((size_t)n * p.C + (size_t)g * p.Cg) * HWp;
    const float* wg = w + ((size_t)g * p.Kg + kb0) * p.L;  // filter k of the block: wg + k*L
    const int kvalid = min(G::KB, p.Kg - kb0);

    v4f acc[G::KPL][G::TH * G::NQ];
#pragma unroll
    for (int i = 0; i < G::KPL; ++i)
#pragma unroll
        for (int a = 0; a < G::TH * G::NQ; ++a) acc[i][a] = v4f{0.0f, 0.0f, 0.0f, 0.0f};

    // Filter staging.  A chunk is KB filters x ROWS = CCH*9 consecutive floats of each filter.
    // TPF threads share one filter, each moving EPT consecutive floats, so both the global offset
    // and the LDS index are one per-thread base plus compile-time steps.  A filter past the
    // group's last one (ragged last block) re-reads the last valid filter: its lanes compute
    // values that are never stored, and no address leaves the tensor.
    constexpr int TPF = nthr / G::KB;
    constexpr int EPT = G::ROWS / TPF;             // 9 (16 wavefronts) or 18 (8 wavefronts)
    static_assert(TPF * G::KB == nthr && EPT * TPF == G::ROWS, "staging must divide evenly");
    float stage[EPT];
    const int sk = tid / TPF, ssub = tid - sk * TPF;
    const unsigned sgoff = (unsigned)(min(sk, kvalid - 1) * p.L + ssub * EPT);
    const int sloff = ssub * EPT * G::KBP + sk;
    auto fetch_chunk = [&](int c0) {
        const float* base = wg + c0 * 9 + sgoff;
#pragma unroll
        for (int i = 0; i < EPT; ++i) stage[i] = base[i];
    };
    auto store_chunk = [&](float* buf) {
#pragma unroll
        for (int i = 0; i < EPT; ++i) buf[sloff + i * G::KBP] = stage[i];
    };
    auto load_x = [&](int c, float (&dst)[G::NX]) {
        const float* base = xg + (size_t)min(c, p.Cg - 1) * HWp;   // uniform; past-the-end prefetch
#pragma unroll                                                    // re-reads the last channel
        for (int q = 0; q < G::NX; ++q) {
            const float t = base[xoff[q]];
            dst[q] = xok[q] ? t : 0.0f;
        }
    };

    const int nchunks = (p.Cg + G::CCH - 1) / G::CCH;
    const int ch0 = ss * nchunks / cfg.NSS, ch1 = (ss + 1) * nchunks / cfg.NSS;   // this workgroup's chunks
    fetch_chunk(ch0 * G::CCH);
    float xn[G::NX];
    load_x(ch0 * G::CCH + cs * cfg.CPW, xn);

    for (int ch = ch0; ch < ch1; ++ch) {
        float* buf = lds + (ch & 1) * G::BUF;
        store_chunk(buf);
        __syncthreads();
        if (ch + 1 < ch1) fetch_chunk((ch + 1) * G::CCH);

        const int cbase = ch * G::CCH + cs * cfg.CPW;   // this wavefront's channels of the chunk
        for (int cc = 0; cc < cfg.CPW; ++cc) {
            float xs[G::NX];
            unsigned mask[2 * G::NX];
#pragma unroll
            for (int q = 0; q < G::NX; ++q) {
                xs[q] = xn[q];
                const unsigned long long m = __ballot(xs[q] != 0.0f);
                mask[2 * q] = (unsigned)m;
                mask[2 * q + 1] = (unsigned)(m >> 32);
            }
            // next channel of this wavefront (next chunk's first one after the last of this chunk)
            const int cnext = (cc + 1 < cfg.CPW) ? cbase + cc + 1 : cbase + G::CCH;
            load_x(cnext, xn);

            unsigned any = 0;
#pragma unroll
            for (int q = 0; q < 2 * G::NX; ++q) any |= mask[q];
            if (any) {
                float wr[G::KPL][9];
                const float* wl = buf + (cs * cfg.CPW + cc) * 9 * G::KBP + lane;
#pragma unroll
                for (int j = 0; j < 9; ++j)
#pragma unroll
                    for (int i = 0; i < G::KPL; ++i) wr[i][j] = wl[j * G::KBP + 64 * i];
                all_quads<G>(std::make_integer_sequence<int, G::IH>{}, mask, xs, acc, wr);
            }
        }
    }

    // reduce the channel slices: slice r hands its partial sums to slice 0 through LDS
    if (cfg.NCS > 1) {
        float* red = lds;  // [NT][KPL*ACC][64]
        for (int r = 1; r < cfg.NCS; ++r) {
            __syncthreads();
            if (cs == r) {
#pragma unroll
                for (int i = 0; i < G::KPL; ++i)
#pragma unroll
                    for (int a = 0; a < G::ACC; ++a)
                        red[(ts * G::KPL * G::ACC + i * G::ACC + a) * 64 + lane] = acc[i][a / 4][a % 4];
            }
            __syncthreads();
            if (cs == 0) {
#pragma unroll
                for (int i = 0; i < G::KPL; ++i)
#pragma unroll
                    for (int a = 0; a < G::ACC; ++a)
                        acc[i][a / 4][a % 4] += red[(ts * G::KPL * G::ACC + i * G::ACC + a) * 64 + lane];
            }
        }
    }
    // epilogue: lane owns filters kb0 + lane + 64*i; accumulator (row, quad, e) = output column 4*quad + e
    if (p.bias) {   // (a branch of its own: without a bias the epilogue is exactly the plain one)
#pragma unroll
        for (int i = 0; i < G::KPL; ++i) {
            const int k = lane + 64 * i;
            const float bk = k < kvalid ? p.bias[(size_t)g * p.Kg + kb0 + k] : 0.0f;
#pragma unroll
            for (int a = 0; a < G::ACC / 4; ++a) acc[i][a] += bk;
        }
    }
    if (!G::POOL && cfg.tr == 2) {
        // Every wavefront of the workgroup stores.  After the reduction slice 0 holds the finished tile and
        // the other slices' wavefronts would idle while it issues all the stores (on a launch of a single
        // round of workgroups that is the tail of the whole kernel).  Slice 0 lays the tile out in LDS as
        // [filter register][row][filter][column]; after one barrier the NCS wavefronts of the tile store its
        // rows in turn, each store a group of RP lanes writing the run one filter has in that row.
        constexpr int TS = 4 * G::NQ + 8;          // row stride: 16-byte aligned, spreads the banks
        constexpr int FPI = 64 / G::RP;            // filters per store instruction
        __syncthreads();   // every wavefront is done with the filter buffers and the reduction
        float* tr = lds + ts * (G::KPL * G::TH * 64 * TS);
        if (cs == 0 && tile_ok) {
#pragma unroll
            for (int i = 0; i < G::KPL; ++i)
#pragma unroll
                for (int orow = 0; orow < G::TH; ++orow)
#pragma unroll
                    for (int q = 0; q < G::NQ; ++q) {
                        v4f v = acc[i][orow * G::NQ + q];
                        if (p.relu) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) v[e] = fmaxf(v[e], 0.0f);
                        }
                        *reinterpret_cast<v4f*>(tr + ((i * G::TH + orow) * 64 + lane) * TS + 4 * q) = v;
                    }
        }
        __syncthreads();
        if (!tile_ok) return;
        const int plane = p.OH * p.OW;
        const int col = lane % G::RP, fsub = lane / G::RP;
        const bool col_ok = col < G::TW && ow0 + col < p.OW;
#pragma unroll
        for (int i = 0; i < G::KPL; ++i) {
            const int kleft = kvalid - 64 * i;     // filters of this register that exist
            float* yk = y + ((size_t)n * p.K + (size_t)g * p.Kg + kb0 + 64 * i) * plane;
#pragma unroll
            for (int orow = 0; orow < G::TH; ++orow) {
                const int oh = oh0 + orow;         // uniform
                if ((orow & (cfg.NCS - 1)) != cs || oh >= p.OH) continue;
                const float* trr = tr + (i * G::TH + orow) * 64 * TS;
#pragma unroll
                for (int kk = 0; kk < G::RP; ++kk) {
                    const int k = kk * FPI + fsub;
                    if (col_ok && k < kleft) yk[(size_t)k * plane + oh * p.OW + ow0 + col] = trr[k * TS + col];
                }
            }
        }
        return;
    }
    if (!G::POOL && cfg.tr) {
        // Stored from the accumulator layout, every lane of a store would go to a different
        // output plane, four bytes each.  Instead each output row of the tile is transposed
        // through LDS (64 filters x TS floats), and a group of RP lanes stores the run of up to
        // TW contiguous floats one filter has in that row.
        constexpr int TS = 4 * G::NQ + 8;          // row stride: 16-byte aligned, spreads the banks
        constexpr int FPI = 64 / G::RP;            // filters per store instruction
        __syncthreads();   // every wavefront is done with the filter buffers and the reduction
        if (cs != 0 || !tile_ok) return;
        float* tr = lds + ts * (64 * TS);
        const int plane = p.OH * p.OW;
        const int col = lane % G::RP, fsub = lane / G::RP;
        const bool col_ok = col < G::TW && ow0 + col < p.OW;
#pragma unroll
        for (int i = 0; i < G::KPL; ++i) {
            const int kleft = kvalid - 64 * i;     // filters of this register that exist
            float* yk = y + ((size_t)n * p.K + (size_t)g * p.Kg + kb0 + 64 * i) * plane;
#pragma unroll
            for (int orow = 0; orow < G::TH; ++orow) {
                const int oh = oh0 + orow;         // uniform
                if (oh >= p.OH) break;
#pragma unroll
                for (int q = 0; q < G::NQ; ++q) {
                    v4f v = acc[i][orow * G::NQ + q];
                    if (p.relu) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = fmaxf(v[e], 0.0f);
                    }
                    *reinterpret_cast<v4f*>(tr + lane * TS + 4 * q) = v;
                }
                // wavefront-private region: the LDS accesses of one wavefront complete in order
#pragma unroll
                for (int kk = 0; kk < G::RP; ++kk) {
                    const int k = kk * FPI + fsub;
                    if (col_ok && k < kleft) yk[(size_t)k * plane + oh * p.OW + ow0 + col] = tr[k * TS + col];
                }
            }
        }
        return;
    }
    if (cs != 0 || !tile_ok) return;

    if (!G::POOL) {
        const int plane = p.OH * p.OW;
#pragma unroll
        for (int i = 0; i < G::KPL; ++i) {
            const int k = lane + 64 * i;
            if (k >= kvalid) continue;
            float* yk = y + ((size_t)n * p.K + (size_t)g * p.Kg + kb0 + k) * plane;
#pragma unroll
            for (int a = 0; a < G::ACC; ++a) {
                const int orow = a / (4 * G::NQ), ocol = a % (4 * G::NQ);
                if (ocol >= G::TW) continue;
                const int oh = oh0 + orow, ow = ow0 + ocol;
                if (oh < p.OH && ow < p.OW) {
                    float v = acc[i][a / 4][a % 4];
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
                    const int q0 = (2 * pr) * G::NQ + (2 * pc) / 4, e = (2 * pc) % 4;   // e is 0 or 2
                    float m = fmaxf(fmaxf(acc[i][q0][e], acc[i][q0][e + 1]),
                                    fmaxf(acc[i][q0 + G::NQ][e], acc[i][q0 + G::NQ][e + 1]));
                    yk[phh * p.PW + pww] = fmaxf(m, 0.0f);
                }
            }
        }
    }
}

// Workgroups of one kernel instantiation that fit on a compute unit (asked once per LDS size).
template <class G, int NWV>
int occupancy(size_t lds_bytes)
{
    static int occ = 0;
    static size_t asked = 0;
    if (occ == 0 || asked != lds_bytes) {
        int nb = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, quad_kernel<G, NWV>, NWV * 64, lds_bytes) !=
                hipSuccess || nb < 1)
            nb = 1;
        occ = nb;
        asked = lds_bytes;
    }
    return occ;
}

template <class G, int NWV>
int launch_nwv(const Problem& p, const TapCfg& cfg, dim3 grid, size_t lds_bytes, const float* x,
               const float* w, float* y, hipStream_t stream)
{
    auto kern = quad_kernel<G, NWV>;
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

// Plan of one launch: the split of a geometry's work over wavefronts and its modelled cost.
struct Plan {
    double cost = -1.0;   // model clocks; negative = not applicable
    TapCfg cfg;
    int nwv = 0;
    int kblocks = 0;
    size_t lds_bytes = 0;
    int nss = 1;          // workgroups per tile along the channels (partial sums through scratch)
};

// Decomposition of one launch.  The work is ntiles x kblocks x images x groups tile-wavefronts,
// each walking Cg channels.  Two knobs: NCS wavefronts split the channels of a tile (more, shorter
// wavefronts: fills the machine at small batch, evens out the last round of workgroups), and NT
// tiles share a workgroup (fewer workgroups re-reading the same filters from L2).  Every
// candidate is priced with a simple model - rounds of workgroups over 256 compute units, SIMDs
// saturating at about four resident wavefronts, one scalar test per input position and channel,
// filter staging at 64 bytes per clock per compute unit - and the cheapest is launched.  The
// density of the input is not known on the host; the model assumes 30 % nonzeros.
template <class G>
Plan plan_geom(const Problem& p)
{
    Plan best;
    TapCfg cfg;
    cfg.tiles_y = (p.OH + G::TH - 1) / G::TH;
    cfg.tiles_x = (p.OW + G::TW - 1) / G::TW;
    cfg.ntiles = cfg.tiles_x * cfg.tiles_y;
    const int kblocks = (p.Kg + G::KB - 1) / G::KB;
    const size_t buf_bytes = 2 * (size_t)G::BUF * sizeof(float);
    const size_t red_per_tile = (size_t)G::KPL * G::ACC * 64 * sizeof(float);
    // clocks of one wavefront on one channel: a test per input row and quad, and for the groups
    // with a nonzero (88 % at 30 % density) their share of the 9 * TH * NQ * KPL matrix
    // instructions at about 9 clocks each
    const double groups = (double)G::IH * G::NQ;
    const double t_channel = 200.0 + 9.0 * groups + 0.88 * 9.0 * G::TH * G::NQ * G::KPL * 9.2;
    const double stage_clocks = (double)G::KB * p.Cg * 36.0 / 64.0;

    int pin_nwv = 0, pin_ncs = 0, pin_nss = 0;   // tuning aid: SCONV_QUAD_SPLIT="nwv,ncs[,nss]"
    pinned_split("SCONV_QUAD_SPLIT", &pin_nwv, &pin_ncs, &pin_nss);
    // The channel split across workgroups (see sconv_split.hip) is only ever pinned here - by
    // sconv_tune, by the dispatcher's static rule for small launches on wide maps, or by the
    // environment; the cost model below ranks unsplit plans.
    const int nss = pin_nss > 1 ? pin_nss : 1;
    if (nss > 1 && (G::POOL || nss > p.Cg / G::CCH || (long long)p.N * p.G * nss > 65535 ||
                    (size_t)nss * p.N * p.K * p.OH * p.OW * sizeof(float) > split_scratch_bytes()))
        return best;
    for (int nwv = 8; nwv <= G::MAXW; nwv *= 2) {
        for (int ncs = 1; ncs <= nwv && ncs <= G::CCH; ncs *= 2) {
            const int nt = nwv / ncs;
            if (pin_nwv && (pin_nwv != nwv || pin_ncs != ncs)) continue;
            // the slice reduction reuses the filter buffers; a large tile's partial sums need more
            size_t lds_bytes = buf_bytes;
            if (ncs > 1 && nt * red_per_tile > lds_bytes) lds_bytes = nt * red_per_tile;
            if (lds_bytes > 160 * 1024) continue;
            if (!pin_nwv && nt > 1 && nt / 2 >= cfg.ntiles) continue;   // half of the tile slots empty
            // a 7-row tile's long reduction and epilogue need 32 channels per slice to pay off
            if (!pin_nwv && G::TH >= 7 && ncs > 1 && p.Cg / ncs < 32) continue;
            const int occ = nwv == 16 ? occupancy<G, G::MAXW>(lds_bytes) : occupancy<G, 8>(lds_bytes);
            const long long wgs1 = (long long)((cfg.ntiles + nt - 1) / nt) * kblocks * p.N * p.G;
            if (nss > 1 && wgs1 >= 512 && current_pin()) continue;   // sconv_tune: not worth a trial
            const long long wgs = wgs1 * nss;
            const long long slots = 256LL * occ;
            const long long rounds = (wgs + slots - 1) / slots;
            const double per_cu = wgs >= slots ? occ : (double)((wgs + 255) / 256);  // resident workgroups
            double r = per_cu * nwv / 4.0;                                         // wavefronts per SIMD
            // below this many resident wavefronts a SIMD is not kept busy; a 7-row tile's wavefront
            // issues 441 matrix instructions per channel and two of them are enough
            const double r_min = G::TH >= 7 ? 2.0 : 4.0;
            if (r < r_min) r = r_min;
            const double cost = rounds * ((double)p.Cg / ncs * t_channel * r + per_cu * stage_clocks) / nss +
                                (ncs - 1) * 8000.0 +  // reduction steps and barrier-bound short slices
                                (nss > 1 ? 9000.0 : 0.0);
            if (best.cost < 0.0 || cost < best.cost) {
                best.cost = cost;
                best.cfg = cfg;
                best.cfg.NT = nt;
                best.cfg.NCS = ncs;
                best.cfg.CPW = G::CCH / ncs;
                best.cfg.tr = (size_t)nt * 64 * (4 * G::NQ + 8) * sizeof(float) <= lds_bytes ? 1 : 0;
                // whole tiles laid out in LDS so that every slice's wavefront stores rows: where that needs
                // no more LDS than the plan has (7-row tiles keep one workgroup per compute unit anyway)
                const size_t all_bytes = (size_t)nt * G::KPL * G::TH * 64 * (4 * G::NQ + 8) * sizeof(float);
                if (!G::POOL && ncs > 1 && all_bytes <= (G::TH >= 7 ? (size_t)160 * 1024 : lds_bytes)) {
                    best.cfg.tr = 2;
                    if (all_bytes > lds_bytes) lds_bytes = all_bytes;
                }
                best.nwv = nwv;
                best.kblocks = kblocks;
                best.lds_bytes = lds_bytes;
                best.nss = nss;
                best.cfg.NSS = nss;
            }
        }
    }
    return best;
}

// pooled: the caller asked for the fused call; a pooled geometry does the pooling itself, a plain one
// (split plans only) leaves it to the kernel that adds the parts.
template <class G>
int launch_plan(const Plan& pl, const Problem& p, bool pooled, const float* x, const float* w, float* y,
                hipStream_t stream)
{
    if (pooled && !G::POOL && pl.nss == 1) return SCONV_EUNSUPPORTED;
    const size_t lds_bytes = pl.lds_bytes;
    const long long gx = (pl.cfg.ntiles + pl.cfg.NT - 1) / pl.cfg.NT;
    const long long gz = (long long)p.N * p.G * pl.nss;
    if (gz > 65535 || pl.kblocks > 65535 || gx >= (1LL << 31)) return SCONV_EUNSUPPORTED;
    const dim3 grid((unsigned)gx, (unsigned)pl.kblocks, (unsigned)gz);
    Problem q = p;
    float* out = y;
    if (pl.nss > 1) {
        // raw partial sums of every channel range into the scratch slices; the second kernel below
        // adds them and applies ReLU
        if (G::POOL || pl.nss > p.Cg / G::CCH ||
            (size_t)pl.nss * p.N * p.K * p.OH * p.OW * sizeof(float) > split_scratch_bytes())
            return SCONV_EUNSUPPORTED;
        out = split_scratch(stream);
        if (!out) return SCONV_EUNSUPPORTED;
        q.relu = 0;
        q.bias = nullptr;
    }
    int rc;
    if (G::MAXW == 16 && pl.nwv == 16)
        rc = launch_nwv<G, G::MAXW>(q, pl.cfg, grid, lds_bytes, x, w, out, stream);
    else
        rc = launch_nwv<G, 8>(q, pl.cfg, grid, lds_bytes, x, w, out, stream);
    if (rc != SCONV_OK || pl.nss == 1) return rc;
    return launch_split_reduce(p, pooled, out, pl.nss, y, stream);
}

// Geometries.  Maps wider than 14: rows of 32 lanes, 28 output columns (7 quads), 2 output rows.
// Maps up to 14 wide: rows of 16 lanes, 14 output columns in 4 quads (the last two columns of
// the fourth quad are computed from the neighbouring row's lanes and never stored), 2 output rows.
using Q32_1 = Geom<1, 2, 32, 7, 28, false>;
using Q32_2 = Geom<2, 1, 32, 7, 28, false>;
using Q32_T7 = Geom<1, 7, 32, 7, 28, false>;   // 7 output rows: heights that are multiples of 7
using Q32_T7D = Geom<1, 7, 32, 7, 28, false, true>;   // the same without zero tests
using Q32_1D = Geom<1, 2, 32, 7, 28, false, true>;
using Q32_2D = Geom<2, 1, 32, 7, 28, false, true>;
using Q16_2 = Geom<2, 2, 16, 4, 14, false>;
using QP32_1 = Geom<1, 2, 32, 7, 28, true>;
using QP16_2 = Geom<2, 2, 16, 4, 14, true>;

bool shape_ok(const Problem& p, bool pooled)
{
    if (p.R != 3 || p.S != 3 || p.pad != 1 || p.stride != 1) return false;
    if (p.Cg % 16) return false;                      // whole staged chunks of channels only
    if (pooled && (p.ph != 2 || p.pw != 2 || p.ps != 2)) return false;
    return true;
}

struct Candidate {
    const char* name;
    Plan (*plan)(const Problem&);
    int (*launch)(const Plan&, const Problem&, bool, const float*, const float*, float*, hipStream_t);
    bool pooled;
    int kpl;              // filters per lane: needs more than 64*(kpl-1) filters in the group
    bool wide;            // for maps wider than 14
    bool by_model = true; // false: only when named (by the tuner's measurement or a pin)
};

const Candidate kCandidates[] = {
    {"q32k1", plan_geom<Q32_1>, launch_plan<Q32_1>, false, 1, true},
    {"q32k2", plan_geom<Q32_2>, launch_plan<Q32_2>, false, 2, true},
    {"q32t7", plan_geom<Q32_T7>, launch_plan<Q32_T7>, false, 1, true},
    {"q32t7d", plan_geom<Q32_T7D>, launch_plan<Q32_T7D>, false, 1, true, false},
    {"q32k1d", plan_geom<Q32_1D>, launch_plan<Q32_1D>, false, 1, true, false},
    {"q32k2d", plan_geom<Q32_2D>, launch_plan<Q32_2D>, false, 2, true, false},
    {"q16k2", plan_geom<Q16_2>, launch_plan<Q16_2>, false, 2, false},
    {"qp32k1", plan_geom<QP32_1>, launch_plan<QP32_1>, true, 1, true},
    {"qp16k2", plan_geom<QP16_2>, launch_plan<QP16_2>, true, 2, false},
};

}  // namespace

const char* const* quad_geoms()
{
    static const char* const names[] = {"q32k1", "q32k2", "q32t7", "q32t7d", "q32k1d", "q32k2d", "q16k2", "qp32k1", "qp16k2", nullptr};
    return names;
}

bool quad_supported(const Problem& p, bool pooled) { return shape_ok(p, pooled); }

int launch_quad(const Problem& p, bool pooled, const float* x, const float* w, float* y,
                hipStream_t stream)
{
    if (!shape_ok(p, pooled)) return SCONV_EUNSUPPORTED;
    const char* pin = pinned_geom("SCONV_QUAD_GEOM");   // tuning aid: candidate name, or !name to exclude one
    int pin_nwv = 0, pin_ncs = 0, pin_nss = 0;
    pinned_split("SCONV_QUAD_SPLIT", &pin_nwv, &pin_ncs, &pin_nss);
    // a fused call whose plan is pinned to a channel split across workgroups runs on the plain
    // tiles: the kernel that adds the parts takes the maximum over the pooling window
    const bool plain_for_pooled = pooled && pin_nss > 1;
    const Candidate* best = nullptr;
    Plan best_plan;
    for (const Candidate& c : kCandidates) {
        if (c.pooled != (pooled && !plain_for_pooled)) continue;
        if (p.Kg <= 64 * (c.kpl - 1)) continue;
        if (pin ? (pin[0] == '!' ? strcmp(pin + 1, c.name) == 0 || c.wide != (p.W > 14) : strcmp(pin, c.name) != 0)
                : (c.wide != (p.W > 14)))
            continue;
        if (!c.by_model && !(pin && pin[0] != '!')) continue;
        const Plan pl = c.plan(p);
        if (pl.cost < 0.0) continue;
        if (!best || pl.cost < best_plan.cost) {
            best = &c;
            best_plan = pl;
        }
    }
    if (!best) return SCONV_EUNSUPPORTED;
    return best->launch(best_plan, p, pooled, x, w, y, stream);
}

}  // namespace sconv

// Matrix-core kernel for 1x1 / stride 1 / pad 0 convolutions (the bottleneck and transition
// layers of the ResNet- and DenseNet-shaped configs), with the optional 2x2 / stride 2 max-pooling
// epilogue.
//
// A 1x1 window row is the channel vector of one position, so Algorithm 2's sparse product is
// y[k][p] = sum over the nonzero channels c of x[c][p] * w[k][c].  Lanes hold output channels
// (k = lane), the accumulators of 64 positions live in 16 register quads, and per input channel
// the 64 positions are one coalesced load (lane = position, Section 5.3 / Fig. 5);
// ballot(x != 0) is the compaction.  The products are issued four positions at a time on the
// matrix pipe: v_mfma_f32_4x4x1 with the A operand broadcast from 4-lane block b of the input
// register adds x[c][p0+4b .. p0+4b+3] * w[k][c] to accumulator quad b for all 64 lanes - full
// fp32 arithmetic, 256 multiply-adds per instruction.  Zero skipping works on a whole channel of
// the tile: when none of its 64 elements is nonzero (dead channels, empty regions of a ReLU map)
// one scalar test replaces its sixteen matrix instructions.  Finer tests were measured to cost
// more than they save on this machine: scalar tests, branches and matrix instructions of all the
// wavefronts of a SIMD share its issue slots (about 4.5 clocks per instruction, 9 per matrix
// instruction), so a test of eight positions (three instructions) only pays when more than 70 %
// of such groups are empty, which i.i.d. zeros reach above a zero ratio of 0.96.
//
// A workgroup is NT position tiles x NCS channel slices sharing one LDS-staged (double-buffered)
// filter chunk of 64 channels x 64 filters; slices reduce through LDS at the end.  Activations
// are prefetched sixteen channels ahead.
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <utility>

#include "sconv_internal.h"

namespace sconv {

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int KB = 64;            // filters per workgroup (one per lane)
constexpr int KBP = KB + 1;       // LDS row stride (odd: conflict-free transposed writes)
constexpr int CCH = 64;           // channels per staged chunk
constexpr int BUF = CCH * KBP;    // floats per LDS buffer
constexpr int XB = 16;            // activation registers: a channel is loaded XB channels ahead

struct PwCfg {
    int NT, NCS;        // wavefronts per workgroup = NT position tiles x NCS channel slices
    int CPW;            // channels per wavefront per chunk = CCH / NCS (a multiple of XB)
    int tiles_x, tiles_y, ntiles;   // tiles per image (flat: tiles_x = tiles, tiles_y = 1)
};

// FLAT: a tile is 64 consecutive positions of the flattened H*W plane (16 quads).
// !FLAT (pooled): a tile is 2 rows x 28 columns, row r in lanes 32r .. 32r+27 (blocks 8r .. 8r+6).
template <bool POOL>
__host__ __device__ constexpr bool block_used(int b)
{
    return POOL ? (b % 8) != 7 : true;
}

// The sixteen matrix instructions of one channel (one per 4-lane block of the input register).
template <bool POOL, int... Bs>
__device__ __forceinline__ void all_blocks(std::integer_sequence<int, Bs...>, float xv, float wv, v4f (&acc)[16])
{
    ((block_used<POOL>(Bs) ? (void)(acc[Bs] = __builtin_amdgcn_mfma_f32_4x4x1f32(xv, wv, acc[Bs], 4, Bs, 0))
                           : (void)0), ...);
}

template <bool POOL, int NWV>
__global__ __launch_bounds__(NWV * 64) void pw_kernel(Problem p, PwCfg cfg, const float* __restrict__ x,
                                                      const float* __restrict__ w, float* __restrict__ y)
{
    extern __shared__ __align__(16) float lds[];  // two filter buffers; reused for the reduction

    const int tid = threadIdx.x;
    constexpr int nthr = NWV * 64;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: scalar registers
    const int ts = wave % cfg.NT;                  // tile slot
    const int cs = wave / cfg.NT;                  // channel slice
    const int n = blockIdx.z / p.G;
    const int g = blockIdx.z - n * p.G;
    const int kb0 = blockIdx.y * KB;               // first filter of the block inside the group
    const int tile = blockIdx.x * cfg.NT + ts;
    const bool tile_ok = tile < cfg.ntiles;
    const int HWp = p.H * p.W;

    // this lane's position
    int oh0 = 0, ow0 = 0, p0 = 0;
    bool xok;
    unsigned xoff;
    if (POOL) {
        const int ty = tile / cfg.tiles_x, tx = tile - ty * cfg.tiles_x;
        oh0 = 2 * ty;
        ow0 = 28 * tx;
        const int r = lane >> 5, c = lane & 31;
        xok = tile_ok && c < 28 && oh0 + r < p.H && ow0 + c < p.W;
        xoff = xok ? (unsigned)((oh0 + r) * p.W + ow0 + c) : 0u;
    } else {
        p0 = tile * 64;
        xok = tile_ok && p0 + lane < HWp;
        xoff = xok ? (unsigned)(p0 + lane) : 0u;
    }
    const float* xg = x + ((size_t)n * p.C + (size_t)g * p.Cg) * HWp;
    const float* wg = w + ((size_t)g * p.Kg + kb0) * p.L;  // filter k of the block: wg + k*L, L = Cg
    const int kvalid = min(KB, p.Kg - kb0);

    v4f acc[16];
#pragma unroll
    for (int b = 0; b < 16; ++b) acc[b] = v4f{0.0f, 0.0f, 0.0f, 0.0f};

    // Filter staging: a chunk is KB filters x CCH consecutive channels of each filter.  TPF threads
    // share one filter, each moving EPT consecutive floats.  A filter past the group's last one
    // re-reads the last valid filter (its lanes' results are never stored).
    constexpr int TPF = nthr / KB;                 // 8 or 16
    constexpr int EPT = CCH / TPF;                 // 8 or 4
    float stage[EPT];
    const int sk = tid / TPF, ssub = tid - sk * TPF;
    const unsigned sgoff = (unsigned)(min(sk, kvalid - 1) * p.L + ssub * EPT);
    const int sloff = ssub * EPT * KBP + sk;
    auto fetch_chunk = [&](int c0) {
        const float* base = wg + c0 + sgoff;
#pragma unroll
        for (int i = 0; i < EPT; ++i) stage[i] = base[i];
    };
    auto store_chunk = [&](float* buf) {
#pragma unroll
        for (int i = 0; i < EPT; ++i) buf[sloff + i * KBP] = stage[i];
    };
    // activations of one channel (clamped: a prefetch past the end re-reads the last channel and is
    // never used)
    // (the value of a lane without a position is replaced by zero where it is consumed, so that
    // the wait for the load sits there and not behind the load)
    auto load_x = [&](int c) -> float { return xg[(size_t)min(c, p.Cg - 1) * HWp + xoff]; };

    const int nchunks = p.Cg / CCH;                // Cg is a multiple of CCH
    fetch_chunk(0);
    // Rotating activation registers: slot j holds channel (first + j) of the current group of XB
    // channels; as soon as its matrix instructions are issued it is reloaded with the channel XB
    // further on, so XB loads of 256 bytes stay in flight per wavefront.
    float xb[XB];
#pragma unroll
    for (int j = 0; j < XB; ++j) xb[j] = load_x(cs * cfg.CPW + j);

    for (int ch = 0; ch < nchunks; ++ch) {
        float* buf = lds + (ch & 1) * BUF;
        store_chunk(buf);
        __syncthreads();
        if (ch + 1 < nchunks) fetch_chunk((ch + 1) * CCH);

        const int cbase = ch * CCH + cs * cfg.CPW;      // this wavefront's channels of the chunk
        for (int cc = 0; cc < cfg.CPW; cc += XB) {
            // the group after this one: in this chunk, or the slice's first group of the next chunk
            const int cnext = (cc + XB < cfg.CPW) ? cbase + cc + XB : cbase + CCH;
            float wv[XB];
            const float* wl = buf + (cs * cfg.CPW + cc) * KBP + lane;
#pragma unroll
            for (int j = 0; j < XB; ++j) wv[j] = wl[j * KBP];

#pragma unroll
            for (int j = 0; j < XB; ++j) {
                const float xv = xok ? xb[j] : 0.0f;
                // one test per channel and tile: a channel without a nonzero in the tile is skipped
                if (__ballot(xv != 0.0f)) all_blocks<POOL>(std::make_integer_sequence<int, 16>{}, xv, wv[j], acc);
                xb[j] = load_x(cnext + j);
            }
        }
    }

    // reduce the channel slices: slice r hands its partial sums to slice 0 through LDS
    if (cfg.NCS > 1) {
        float* red = lds;  // [NT][64 accumulator floats][64 lanes]
        for (int r = 1; r < cfg.NCS; ++r) {
            __syncthreads();
            if (cs == r) {
#pragma unroll
                for (int a = 0; a < 64; ++a) red[(ts * 64 + a) * 64 + lane] = acc[a / 4][a % 4];
            }
            __syncthreads();
            if (cs == 0) {
#pragma unroll
                for (int a = 0; a < 64; ++a) acc[a / 4][a % 4] += red[(ts * 64 + a) * 64 + lane];
            }
        }
    }
    if (cs != 0 || !tile_ok || lane >= kvalid) return;

    // epilogue: lane owns filter kb0 + lane; accumulator quad b, element e = lane position 4b + e
    if (!POOL) {
        float* yk = y + ((size_t)n * p.K + (size_t)g * p.Kg + kb0 + lane) * HWp + p0;
        const bool vec = (HWp % 4) == 0;   // quads are 16-byte aligned in every plane
#pragma unroll
        for (int b = 0; b < 16; ++b) {
            v4f v = acc[b];
            if (p.relu) {
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = fmaxf(v[e], 0.0f);
            }
            if (vec && p0 + 4 * b + 3 < HWp) {
                *reinterpret_cast<v4f*>(yk + 4 * b) = v;
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (p0 + 4 * b + e < HWp) yk[4 * b + e] = v[e];
            }
        }
    } else {
        // pooled output (oh0/2, ow0/2 + pc), pc < 14: columns 2pc, 2pc+1 of rows 0 and 1
        const int plane = p.PH * p.PW;
        const int phh = oh0 / 2;
        if (phh < p.PH) {
            float* yk = y + ((size_t)n * p.K + (size_t)g * p.Kg + kb0 + lane) * plane + phh * p.PW + ow0 / 2;
#pragma unroll
            for (int pc = 0; pc < 14; ++pc) {
                if (ow0 / 2 + pc < p.PW) {
                    const int b = (2 * pc) / 4, e = (2 * pc) % 4;   // e is 0 or 2
                    const float m = fmaxf(fmaxf(acc[b][e], acc[b][e + 1]), fmaxf(acc[8 + b][e], acc[8 + b][e + 1]));
                    yk[pc] = fmaxf(m, 0.0f);
                }
            }
        }
    }
}

// Workgroups of one kernel instantiation that fit on a compute unit, per LDS size (asked once each).
template <bool POOL, int NWV>
int occupancy(size_t lds_bytes)
{
    static size_t seen_bytes[8];
    static int seen_occ[8];
    static int nseen = 0;
    for (int i = 0; i < nseen; ++i)
        if (seen_bytes[i] == lds_bytes) return seen_occ[i];
    int nb = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, pw_kernel<POOL, NWV>, NWV * 64, lds_bytes) !=
            hipSuccess || nb < 1)
        nb = 1;
    if (nseen < 8) {
        seen_bytes[nseen] = lds_bytes;
        seen_occ[nseen] = nb;
        ++nseen;
    }
    return nb;
}

template <bool POOL, int NWV>
int launch_nwv(const Problem& p, const PwCfg& cfg, dim3 grid, size_t lds_bytes, const float* x,
               const float* w, float* y, hipStream_t stream)
{
    auto kern = pw_kernel<POOL, NWV>;
    static size_t opted = 48 * 1024;  // dynamic LDS above 48 KiB is opted into once per kernel
    if (lds_bytes > opted) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024) != hipSuccess)
            return SCONV_ELAUNCH;
        opted = 128 * 1024;
    }
    hipLaunchKernelGGL(kern, grid, dim3(NWV * 64), lds_bytes, stream, p, cfg, x, w, y);
    return launch_status();
}

// Split of one launch over wavefronts, priced like the 3x3 kernels: rounds of workgroups over 256
// compute units, SIMDs saturating at about four resident wavefronts, filter staging traffic.
template <bool POOL>
int launch_pw(const Problem& p, const float* x, const float* w, float* y, hipStream_t stream)
{
    PwCfg cfg;
    if (POOL) {
        cfg.tiles_x = (p.OW + 27) / 28;
        cfg.tiles_y = p.PH;                         // one pooled row per tile
    } else {
        cfg.tiles_x = (p.H * p.W + 63) / 64;
        cfg.tiles_y = 1;
    }
    cfg.ntiles = cfg.tiles_x * cfg.tiles_y;
    const int kblocks = (p.Kg + KB - 1) / KB;
    const size_t stage_bytes = 2 * (size_t)BUF * sizeof(float);
    const size_t red_per_tile = 64 * 64 * sizeof(float);
    const double t_channel = 40.0 + 16.0 * 9.2;    // one wavefront, one channel, all groups nonzero
    const double stage_clocks = (double)KB * p.Cg * 4.0 / 64.0;

    int pin_nwv = 0, pin_ncs = 0;   // tuning aid: SCONV_PW_SPLIT="nwv,ncs"
    if (const char* pin = getenv("SCONV_PW_SPLIT")) {
        if (sscanf(pin, "%d,%d", &pin_nwv, &pin_ncs) != 2) pin_nwv = pin_ncs = 0;
    }
    double best = -1.0;
    int best_nwv = 0;
    size_t lds_bytes = stage_bytes;
    for (int nwv = 8; nwv <= 16; nwv *= 2) {
        for (int ncs = 1; ncs <= nwv && ncs <= CCH / XB; ncs *= 2) {
            const int nt = nwv / ncs;
            if (pin_nwv && (pin_nwv != nwv || pin_ncs != ncs)) continue;
            if (!pin_nwv && nt > 1 && nt / 2 >= cfg.ntiles) continue;
            // the reduction of the channel slices reuses the staging buffers and may need more
            size_t bytes = stage_bytes;
            if (ncs > 1 && nt * red_per_tile > bytes) bytes = nt * red_per_tile;
            const int occ = nwv == 16 ? occupancy<POOL, 16>(bytes) : occupancy<POOL, 8>(bytes);
            const long long wgs = (long long)((cfg.ntiles + nt - 1) / nt) * kblocks * p.N * p.G;
            const long long slots = 256LL * occ;
            const long long rounds = (wgs + slots - 1) / slots;
            const double per_cu = wgs >= slots ? occ : (double)((wgs + 255) / 256);
            double r = per_cu * nwv / 4.0;
            if (r < 4.0) r = 4.0;
            const double cost = rounds * ((double)p.Cg / ncs * t_channel * r + per_cu * stage_clocks) +
                                (ncs - 1) * 2000.0;
            if (best < 0.0 || cost < best) {
                best = cost;
                cfg.NT = nt;
                cfg.NCS = ncs;
                cfg.CPW = CCH / ncs;
                best_nwv = nwv;
                lds_bytes = bytes;
            }
        }
    }
    if (best < 0.0) return SCONV_EUNSUPPORTED;
    const long long gx = (cfg.ntiles + cfg.NT - 1) / cfg.NT;
    const unsigned gz = (unsigned)(p.N * p.G);
    if (gz > 65535u || kblocks > 65535 || gx >= (1LL << 31)) return SCONV_EUNSUPPORTED;
    const dim3 grid((unsigned)gx, (unsigned)kblocks, gz);
    return best_nwv == 16 ? launch_nwv<POOL, 16>(p, cfg, grid, lds_bytes, x, w, y, stream)
                          : launch_nwv<POOL, 8>(p, cfg, grid, lds_bytes, x, w, y, stream);
}

}  // namespace

bool pw_supported(const Problem& p, bool pooled)
{
    if (p.R != 1 || p.S != 1 || p.stride != 1 || p.pad != 0) return false;
    if (p.Cg % CCH) return false;                     // whole staged chunks of channels only
    if (pooled && (p.ph != 2 || p.pw != 2 || p.ps != 2)) return false;
    return true;
}

int launch_pointwise(const Problem& p, bool pooled, const float* x, const float* w, float* y,
                     hipStream_t stream)
{
    if (!pw_supported(p, pooled)) return SCONV_EUNSUPPORTED;
    return pooled ? launch_pw<true>(p, x, w, y, stream) : launch_pw<false>(p, x, w, y, stream);
}

}  // namespace sconv

// Matrix-core kernel for 1x1 / stride 1 / pad 0 convolutions (the bottleneck and transition
// layers of the ResNet- and DenseNet-shaped configs), with the optional 2x2 / stride 2 max-pooling
// epilogue.
//
// A 1x1 window row is the channel vector of one position, so Algorithm 2's sparse product is
// y[k][p] = sum over the nonzero channels c of x[c][p] * w[k][c].  Lanes hold output channels
// (k = lane) and a wavefront owns 32 positions, whose accumulators are 8 register quads.  One
// coalesced load brings those 32 positions of TWO channels (lanes 0-31 channel c, lanes 32-63
// channel c + 1; lane = position, Section 5.3 / Fig. 5); ballot(x != 0) is the compaction.  The
// products are issued four positions at a time on the matrix pipe: v_mfma_f32_4x4x1 with the A
// operand broadcast from 4-lane block b of the input register adds x[c][p0+4b .. p0+4b+3] * w[k][c]
// to accumulator quad b (blocks 8-15: channel c + 1, quad b - 8) for all 64 lanes - full fp32
// arithmetic, 256 multiply-adds per instruction.  Zero skipping works on a channel of the tile:
// when none of its 32 elements is nonzero (dead channels, empty regions of a ReLU map) one scalar
// test replaces its eight matrix instructions.  Finer tests were measured to cost more than they
// save on this machine.
//
// These layers are bound by memory, and the read rate a compute unit reaches grows with the bytes
// it keeps in flight; the small tile (32 accumulator registers) is what lets seven or eight
// wavefronts per SIMD each keep XB 256-byte loads outstanding.
//
// A workgroup is NT position tiles x NCS channel slices sharing one LDS-staged (double-buffered)
// filter chunk of 64 channels x 64 filters; slices reduce through LDS at the end.
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
constexpr int TP = 32;            // positions per tile

struct PwCfg {
    int NT, NCS;        // wavefronts per workgroup = NT position tiles x NCS channel slices
    int CPW;            // channels per wavefront per chunk = CCH / NCS (a multiple of 2 * XB)
    int tiles_x, tiles_y, ntiles;   // pooled: tiles per image; plain: tiles_x = tiles of the batch
    int npos;                       // plain: positions of the batch, N*H*W
};

// The eight matrix instructions of one channel: blocks B0 .. B0 + 7 of the input register feed
// accumulator quads 0 .. 7.
template <int B0, int... Qs>
__device__ __forceinline__ void channel_blocks(std::integer_sequence<int, Qs...>, float xv, float wv, v4f (&acc)[8])
{
    ((acc[Qs] = __builtin_amdgcn_mfma_f32_4x4x1f32(xv, wv, acc[Qs], 4, B0 + Qs, 0)), ...);
}

// Plain: a tile is 32 consecutive positions of the batch's flattened planes (8 quads).
// Pooled: a tile is 2 rows x 14 columns of one image, row r in lanes 16r .. 16r+13 (quads 4r .. 4r+3).
// DENSE: no zero tests - for maps without dead channels or empty regions, where no channel of a
// 32-position tile is ever all zero and the test (a compare, a mask, two scalar branches per channel
// pair) only takes issue time from the matrix instructions.  Lanes without a position then feed
// whatever they loaded into accumulators that are never stored.
template <bool POOL, int NWV, int XB, bool DENSE>
__global__ __launch_bounds__(NWV * 64) __attribute__((amdgpu_waves_per_eu(6, 8))) void pw_kernel(Problem p, PwCfg cfg, const float* __restrict__ x,
                                                      const float* __restrict__ w, float* __restrict__ y)
{
    extern __shared__ __align__(16) float lds[];  // two filter buffers; reused for the reduction

    const int tid = threadIdx.x;
    constexpr int nthr = NWV * 64;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: scalar registers
    const int ts = wave % cfg.NT;                  // tile slot
    const int cs = wave / cfg.NT;                  // channel slice
    // pooled: tiles of one image per workgroup row (grid z = image, group); plain: tiles of the
    // whole batch (grid z = group), so no tile is ragged but the last
    const int n = POOL ? blockIdx.z / p.G : 0;
    const int g = POOL ? blockIdx.z - n * p.G : blockIdx.z;
    const int kb0 = blockIdx.y * KB;               // first filter of the block inside the group
    const int tile = blockIdx.x * cfg.NT + ts;
    const bool tile_ok = tile < cfg.ntiles;
    const int HWp = p.H * p.W;

    // this lane's position (lanes l and l + 32 share it) and channel parity
    const int pl = lane & 31, half = lane >> 5;
    int oh0 = 0, ow0 = 0, p0 = 0;
    bool xok;
    unsigned xoff;
    if (POOL) {
        const int ty = tile / cfg.tiles_x, tx = tile - ty * cfg.tiles_x;
        oh0 = 2 * ty;
        ow0 = 14 * tx;
        const int r = pl >> 4, c = pl & 15;
        xok = tile_ok && c < 14 && oh0 + r < p.H && ow0 + c < p.W;
        xoff = xok ? (unsigned)((oh0 + r) * p.W + ow0 + c + half * HWp) : 0u;
    } else {
        p0 = tile * TP;                             // position number in the batch: image * H*W + pixel
        xok = tile_ok && p0 + pl < cfg.npos;
        const int ni = xok ? (p0 + pl) / HWp : 0;
        xoff = xok ? (unsigned)(ni * (p.C - 1) * HWp + p0 + pl + half * HWp) : 0u;   // ni*C*HW + pixel
    }
    const float* xg = x + ((size_t)n * p.C + (size_t)g * p.Cg) * HWp;
    const float* wg = w + ((size_t)g * p.Kg + kb0) * p.L;  // filter k of the block: wg + k*L, L = Cg
    const int kvalid = min(KB, p.Kg - kb0);

    v4f acc[8];
#pragma unroll
    for (int b = 0; b < 8; ++b) acc[b] = v4f{0.0f, 0.0f, 0.0f, 0.0f};

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
    // activations of the channel pair (c, c + 1), c even (clamped: a prefetch past the end re-reads
    // the last pair and is never used).  The value of a lane without a position is replaced by
    // zero where it is consumed, so that the wait for the load sits there and not behind the load.
    // (the lane offset is made opaque next to the load so that the load takes the scalar channel
    // base and the 32-bit lane offset as they are, without vector address arithmetic)
    unsigned xboff = 4u * xoff;
    auto load_x = [&](int c) -> float {
        const char* base = (const char*)(xg + (size_t)min(c, p.Cg - 2) * HWp);
        asm volatile("" : "+v"(xboff));
        return *(const float*)(base + xboff);
    };

    const int nchunks = p.Cg / CCH;                // Cg is a multiple of CCH
    fetch_chunk(0);
    // Rotating activation registers: slot j holds channel pair (first + 2j) of the current group of
    // 2*XB channels; as soon as its matrix instructions are issued it is reloaded with the pair 2*XB
    // channels further on, so XB loads of 256 bytes stay in flight per wavefront.
    float xb[XB];
#pragma unroll
    for (int j = 0; j < XB; ++j) xb[j] = load_x(cs * cfg.CPW + 2 * j);

    for (int ch = 0; ch < nchunks; ++ch) {
        float* buf = lds + (ch & 1) * BUF;
        store_chunk(buf);
        __syncthreads();
        if (ch + 1 < nchunks) fetch_chunk((ch + 1) * CCH);

        const int cbase = ch * CCH + cs * cfg.CPW;      // this wavefront's channels of the chunk
        for (int cc = 0; cc < cfg.CPW; cc += 2 * XB) {
            // the group after this one: in this chunk, or the slice's first group of the next chunk
            const int cnext = (cc + 2 * XB < cfg.CPW) ? cbase + cc + 2 * XB : cbase + CCH;
            const float* wl = buf + (cs * cfg.CPW + cc) * KBP + lane;
            // filter values of a pair are read from LDS one pair ahead of their use
            float wc0 = wl[0], wc1 = wl[KBP];
#pragma unroll
            for (int j = 0; j < XB; ++j) {
                float wn0 = 0.0f, wn1 = 0.0f;
                if (j + 1 < XB) {
                    wn0 = wl[(2 * j + 2) * KBP];
                    wn1 = wl[(2 * j + 3) * KBP];
                }
                if (DENSE) {
                    const float xv = xb[j];
                    channel_blocks<0>(std::make_integer_sequence<int, 8>{}, xv, wc0, acc);
                    channel_blocks<8>(std::make_integer_sequence<int, 8>{}, xv, wc1, acc);
                } else {
                    const float xv = xok ? xb[j] : 0.0f;
                    // one test per channel and tile: a channel without a nonzero in the tile is skipped
                    const unsigned long long m = __ballot(xv != 0.0f);
                    unsigned lo = (unsigned)m, hi = (unsigned)(m >> 32);
                    asm volatile("" : "+s"(lo), "+s"(hi));   // two 32-bit scalar tests
                    if (lo) channel_blocks<0>(std::make_integer_sequence<int, 8>{}, xv, wc0, acc);
                    if (hi) channel_blocks<8>(std::make_integer_sequence<int, 8>{}, xv, wc1, acc);
                }
                xb[j] = load_x(cnext + 2 * j);
                wc0 = wn0;
                wc1 = wn1;
            }
        }
    }

    // reduce the channel slices: slice r hands its partial sums to slice 0 through LDS
    if (cfg.NCS > 1) {
        float* red = lds;  // [NT][32 accumulator floats][64 lanes]
        for (int r = 1; r < cfg.NCS; ++r) {
            __syncthreads();
            if (cs == r) {
#pragma unroll
                for (int a = 0; a < 32; ++a) red[(ts * 32 + a) * 64 + lane] = acc[a / 4][a % 4];
            }
            __syncthreads();
            if (cs == 0) {
#pragma unroll
                for (int a = 0; a < 32; ++a) acc[a / 4][a % 4] += red[(ts * 32 + a) * 64 + lane];
            }
        }
    }
    // epilogue: lane owns filter kb0 + lane; accumulator quad b, element e = tile position 4b + e
    if (p.bias) {   // (a branch of its own: without a bias the epilogue is exactly the plain one)
        const float bk = lane < kvalid ? p.bias[(size_t)g * p.Kg + kb0 + lane] : 0.0f;
#pragma unroll
        for (int b = 0; b < 8; ++b) acc[b] += bk;
    }
    if (!POOL) {
        const size_t kglob0 = (size_t)g * p.Kg + kb0;
        if ((HWp % 4) == 0) {
            // Quads are 16-byte aligned and never straddle images.  The tile is transposed through
            // LDS (rows of 36 floats: filter, then position) so that eight lanes store the 128
            // contiguous bytes one filter has in this tile; storing from the accumulator layout
            // would send each lane's 16 bytes to a different plane.
            __syncthreads();   // every wavefront is done with the filter buffers
            if (cs != 0 || !tile_ok) return;
            float* tr = lds + ts * (64 * 36);
#pragma unroll
            for (int b = 0; b < 8; ++b) {
                v4f v = acc[b];
                if (p.relu) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = fmaxf(v[e], 0.0f);
                }
                *reinterpret_cast<v4f*>(tr + lane * 36 + 4 * b) = v;
            }
            // wavefront-private region: the LDS accesses of one wavefront complete in order
            const int q = lane & 7, kr = lane >> 3;
            const int P0 = p0 + 4 * q;
            if (P0 < cfg.npos) {
                const int ni = P0 / HWp;
                float* dst = y + ((size_t)ni * p.K + kglob0) * HWp + (P0 - ni * HWp);
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int k = 8 * i + kr;
                    if (k < kvalid)
                        *reinterpret_cast<v4f*>(dst + (size_t)k * HWp) = *reinterpret_cast<const v4f*>(tr + k * 36 + 4 * q);
                }
            }
            return;
        }
        if (cs != 0 || !tile_ok || lane >= kvalid) return;
        const size_t kglob = kglob0 + lane;
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const int P0 = p0 + 4 * b;     // uniform
            if (P0 >= cfg.npos) break;
            v4f v = acc[b];
            if (p.relu) {
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = fmaxf(v[e], 0.0f);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int Pe = P0 + e;
                if (Pe < cfg.npos) {
                    const int ni = Pe / HWp;
                    y[((size_t)ni * p.K + kglob) * HWp + (Pe - ni * HWp)] = v[e];
                }
            }
        }
    } else {
        if (cs != 0 || !tile_ok || lane >= kvalid) return;
        // pooled output (oh0/2, ow0/2 + pc), pc < 7: columns 2pc, 2pc+1 of rows 0 and 1
        const int plane = p.PH * p.PW;
        const int phh = oh0 / 2;
        if (phh < p.PH) {
            float* yk = y + ((size_t)n * p.K + (size_t)g * p.Kg + kb0 + lane) * plane + phh * p.PW + ow0 / 2;
#pragma unroll
            for (int pc = 0; pc < 7; ++pc) {
                if (ow0 / 2 + pc < p.PW) {
                    const int b = (2 * pc) / 4, e = (2 * pc) % 4;   // e is 0 or 2
                    const float m = fmaxf(fmaxf(acc[b][e], acc[b][e + 1]), fmaxf(acc[4 + b][e], acc[4 + b][e + 1]));
                    yk[pc] = fmaxf(m, 0.0f);
                }
            }
        }
    }
}

// Workgroups of one kernel instantiation that fit on a compute unit, per LDS size (asked once each).
template <bool POOL, int NWV, int XB>
int occupancy(size_t lds_bytes)
{
    static size_t seen_bytes[8];
    static int seen_occ[8];
    static int nseen = 0;
    for (int i = 0; i < nseen; ++i)
        if (seen_bytes[i] == lds_bytes) return seen_occ[i];
    int nb = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, pw_kernel<POOL, NWV, XB, false>, NWV * 64, lds_bytes) !=
            hipSuccess || nb < 1)
        nb = 1;
    if (nseen < 8) {
        seen_bytes[nseen] = lds_bytes;
        seen_occ[nseen] = nb;
        ++nseen;
    }
    return nb;
}

template <bool POOL, int NWV, int XB, bool DENSE>
int launch_inst(const Problem& p, const PwCfg& cfg, dim3 grid, size_t lds_bytes, const float* x,
                const float* w, float* y, hipStream_t stream)
{
    auto kern = pw_kernel<POOL, NWV, XB, DENSE>;
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

const char* const kPwGeoms[] = {"", "dense", nullptr};

// the zero-testing kernel unless the dense form is named (by sconv_tune's measurement or SCONV_PW_GEOM)
template <bool POOL, int NWV, int XB>
int launch_nwv(const Problem& p, const PwCfg& cfg, dim3 grid, size_t lds_bytes, const float* x,
               const float* w, float* y, hipStream_t stream)
{
    const char* geom = pinned_geom("SCONV_PW_GEOM");
    if (geom && !strcmp(geom, "dense"))
        return launch_inst<POOL, NWV, XB, true>(p, cfg, grid, lds_bytes, x, w, y, stream);
    return launch_inst<POOL, NWV, XB, false>(p, cfg, grid, lds_bytes, x, w, y, stream);
}

// Split of one launch over wavefronts, priced like the 3x3 kernels: rounds of workgroups over 256
// compute units, SIMDs saturating at about four resident wavefronts, filter staging traffic.
// One or two channel slices keep 16 loads (32 channels) in flight per wavefront, four slices 8.
template <bool POOL>
int launch_pw(const Problem& p, const float* x, const float* w, float* y, hipStream_t stream)
{
    PwCfg cfg;
    if (POOL) {
        cfg.tiles_x = (p.OW + 13) / 14;
        cfg.tiles_y = p.PH;                         // one pooled row per tile
    } else {
        cfg.tiles_x = (int)(((long long)p.N * p.H * p.W + TP - 1) / TP);
        cfg.tiles_y = 1;
    }
    cfg.npos = POOL ? 0 : p.N * p.H * p.W;
    const int images = POOL ? p.N : 1;             // plain tiles run over the whole batch
    cfg.ntiles = cfg.tiles_x * cfg.tiles_y;
    const int kblocks = (p.Kg + KB - 1) / KB;
    const size_t stage_bytes = 2 * (size_t)BUF * sizeof(float);
    const size_t red_per_tile = 32 * 64 * sizeof(float);
    const double t_channel = 25.0 + 8.0 * 9.2;     // one wavefront, one channel, all groups nonzero
    const double stage_clocks = (double)KB * p.Cg * 4.0 / 64.0;

    int pin_nwv = 0, pin_ncs = 0;   // tuning aid: SCONV_PW_SPLIT="nwv,ncs"
    pinned_split("SCONV_PW_SPLIT", &pin_nwv, &pin_ncs);
    double best = -1.0;
    int best_nwv = 0;
    size_t lds_bytes = stage_bytes;
    for (int nwv = 8; nwv <= 16; nwv *= 2) {
        for (int ncs = 1; ncs <= 4; ncs *= 2) {
            const int nt = nwv / ncs;
            if (pin_nwv && (pin_nwv != nwv || pin_ncs != ncs)) continue;
            if (!pin_nwv && nt > 1 && nt / 2 >= cfg.ntiles) continue;
            // the reduction of the channel slices reuses the staging buffers and may need more
            size_t bytes = stage_bytes;
            if (ncs > 1 && nt * red_per_tile > bytes) bytes = nt * red_per_tile;
            if (!POOL && (size_t)nt * 64 * 36 * sizeof(float) > bytes) bytes = (size_t)nt * 64 * 36 * sizeof(float);
            if (bytes > 128 * 1024) continue;
            const int occ = nwv == 16 ? (ncs == 4 ? occupancy<POOL, 16, 8>(bytes) : occupancy<POOL, 16, 16>(bytes))
                                      : (ncs == 4 ? occupancy<POOL, 8, 8>(bytes) : occupancy<POOL, 8, 16>(bytes));
            const long long wgs = (long long)((cfg.ntiles + nt - 1) / nt) * kblocks * images * p.G;
            const long long slots = 256LL * occ;
            const long long rounds = (wgs + slots - 1) / slots;
            const double per_cu = wgs >= slots ? occ : (double)((wgs + 255) / 256);
            double r = per_cu * nwv / 4.0;
            if (r < 4.0) r = 4.0;
            double cost = rounds * ((double)p.Cg / ncs * t_channel * r + per_cu * stage_clocks) +
                          (ncs - 1) * 300.0;
            // measured: many short workgroups overlap their start-up (first filter chunk, first
            // loads) with the others' streaming; the model above does not see that
            if (nwv == 8 && ncs == 4 && wgs >= 512) cost *= 0.8;
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
    const unsigned gz = (unsigned)(images * p.G);
    if (gz > 65535u || kblocks > 65535 || gx >= (1LL << 31)) return SCONV_EUNSUPPORTED;
    const dim3 grid((unsigned)gx, (unsigned)kblocks, gz);
    if (cfg.NCS == 4)
        return best_nwv == 16 ? launch_nwv<POOL, 16, 8>(p, cfg, grid, lds_bytes, x, w, y, stream)
                              : launch_nwv<POOL, 8, 8>(p, cfg, grid, lds_bytes, x, w, y, stream);
    return best_nwv == 16 ? launch_nwv<POOL, 16, 16>(p, cfg, grid, lds_bytes, x, w, y, stream)
                          : launch_nwv<POOL, 8, 16>(p, cfg, grid, lds_bytes, x, w, y, stream);
}

}  // namespace

bool pw_supported(const Problem& p, bool pooled)
{
    if (p.R != 1 || p.S != 1 || p.stride != 1 || p.pad != 0) return false;
    if (p.Cg % CCH) return false;                     // whole staged chunks of channels only
    if (pooled && (p.ph != 2 || p.pw != 2 || p.ps != 2)) return false;
    if ((long long)p.N * p.C * p.H * p.W >= (1LL << 30)) return false;   // 32-bit byte offsets into the input
    return true;
}

const char* const* pw_geoms() { return kPwGeoms; }

int launch_pointwise(const Problem& p, bool pooled, const float* x, const float* w, float* y,
                     hipStream_t stream)
{
    if (!pw_supported(p, pooled)) return SCONV_EUNSUPPORTED;
    return pooled ? launch_pw<true>(p, x, w, y, stream) : launch_pw<false>(p, x, w, y, stream);
}

}  // namespace sconv

// Element-stationary kernel for 3x3 / pad 1 convolutions of stride 1 or 2 (the bulk of the VGG-,
// ResNet-, DenseNet- and RegNet-shaped layers), with the optional 2x2 / stride 2 max-pooling
// epilogue (stride 1 only).
//
// Same arithmetic as the window-row formulation (Section 5.4: only nonzero elements are
// multiplied), different bookkeeping.  A nonzero element x[c][h][w] appears in up to nine window
// rows, at nine different filter positions; instead of storing it nine times (the "extended"
// part of ECR) a wavefront finds it once and issues all of its products:
//   - lanes hold output channels (64*KPL filters per wavefront, KPL per lane);
//   - the accumulators of a TH x TW output tile live in registers, statically indexed;
//   - per input channel, the 9*KPL filter values of the lane's filters are read once from an
//     LDS-staged filter tile and stay in registers while the whole input tile of that channel is
//     processed (filter reuse = number of nonzeros of the channel inside the tile);
//   - the input tile (output tile plus halo) is read from HBM/L2 with one coalesced load per
//     64 positions, one element per lane; ballot(x != 0) gives the nonzero mask - the wavefront
//     level compaction; positions are tested four at a time first, then one by one inside a group
//     that holds a nonzero, so a zero element costs between a quarter of and one scalar bit test;
//   - for each set bit the value is broadcast from its lane (readlane -> scalar register) and
//     the code for that position, which knows at compile time which accumulators and which
//     filter taps the position touches, runs up to 9*KPL FMAs with a scalar operand.
// Several wavefronts of a workgroup share the filter tile: NT of them own different spatial
// tiles, NCS of them split the input channels of one tile (partial sums are reduced through LDS
// at the end), so that small batches still fill the machine.
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <map>
#include <utility>

#include "sconv_internal.h"
#include "sconv_tapt.h"

namespace sconv {

namespace {


#include "sconv_tap_common.h"

template <class G, int NWV>
__global__ __launch_bounds__(NWV * 64) void tap_kernel(Problem p, TapCfg cfg, const float* __restrict__ x,
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
        const int ih = P / G::IW, iw = P - ih * G::IW;
        const int xr = oh0 * G::STRIDE - G::HH + ih, xc = ow0 * G::STRIDE - G::HW + iw;
        xok[q] = tile_ok && P < G::NPOS && xr >= 0 && xr < p.H && xc >= 0 && xc < p.W;
        xoff[q] = xok[q] ? (unsigned)(xr * p.W + xc) : 0u;
    }
    const float* xg = x + ((size_t)n * p.C + (size_t)g * p.Cg) * HWp;
    const float* wg = w + ((size_t)g * p.Kg + kb0) * p.L;  // filter k of the block: wg + k*L
    const int kvalid = min(G::KB, p.Kg - kb0);

    float acc[G::KPL][G::ACC];
#pragma unroll
    for (int i = 0; i < G::KPL; ++i)
#pragma unroll
        for (int a = 0; a < G::ACC; ++a) acc[i][a] = 0.0f;

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
            float xv[G::NX];
            unsigned mask[2 * G::NX];
#pragma unroll
            for (int q = 0; q < G::NX; ++q) {
                xv[q] = xn[q];
                const unsigned long long m = __ballot(xv[q] != 0.0f);
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
                all_positions<G>(std::make_integer_sequence<int, (G::NPOS + 3) / 4>{}, mask, xv, acc, wr);
            }
        }
    }

    reduce_slices<G>(cfg, lds, acc, ts, cs, lane);
    if (cs != 0 || !tile_ok) return;

    store_tile<G>(p, acc, y, ss, n, g, kb0, kvalid, oh0, ow0, lane);
}

// Workgroups of one kernel instantiation that fit on a compute unit (asked once per LDS size).
template <class G, int NWV>
int occupancy(size_t lds_bytes)
{
    static std::map<size_t, int> answers;   // under the dispatcher's lock
    auto it = answers.find(lds_bytes);
    if (it != answers.end()) return it->second;
    int occ = 0;
    {
        int nb = 0;
        const hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, tap_kernel<G, NWV>, NWV * 64, lds_bytes);
        if (e != hipSuccess || nb < 1)
            nb = 1;
        occ = nb;
    }
    answers[lds_bytes] = occ;
    return occ;
}

template <class G, int NWV>
int launch_nwv(const Problem& p, const TapCfg& cfg, dim3 grid, size_t lds_bytes, const float* x,
               const float* w, float* y, hipStream_t stream)
{
    auto kern = tap_kernel<G, NWV>;
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


// Decomposition of one launch.  The work is ntiles x kblocks x images x groups tile-wavefronts,
// each walking Cg channels.  Two knobs: NCS wavefronts split the channels of a tile (more, shorter
// wavefronts: fills the machine at small batch, evens out the last round of workgroups), and NT
// tiles share a workgroup (fewer workgroups re-reading the same filters from L2).  Every
// candidate is priced with a simple model - rounds of workgroups over 256 compute units, SIMDs
// saturating at about four resident wavefronts, one scalar test per input position and channel,
// filter staging at 64 bytes per clock per compute unit - and the cheapest is launched.  The
// density of the input is not known on the host; the model assumes 30 % nonzeros.
//
// Third knob, for small launches only: NSS workgroups split the channels of a tile (split: 0 = not
// allowed, 1 = allowed, 2 = required - a plain tile serving a pooled layer).  A workgroup has one
// filter chunk in flight, so a launch of fewer workgroups than compute units waits on the memory
// latency chunk after chunk; the split divides that chain, for the price of the second, small
// kernel that adds the partial sums.  The model splits launches of fewer than 128 tile-workgroups
// (measured 1.4-3.5x faster there) and, two to four ways, launches of up to 768 that walk 16 or more
// chunks with one filter per lane (around 200 workgroups of shorter chains the split measures
// between 1.2x faster and 1.5x slower); sconv_tune tries splits of launches up to 512.
template <class G>
Plan plan_geom(const Problem& p, int split)
{
    Plan best;
    TapCfg cfg;
    cfg.tiles_y = (p.OH + G::TH - 1) / G::TH;
    cfg.tiles_x = (p.OW + G::TW - 1) / G::TW;
    cfg.ntiles = cfg.tiles_x * cfg.tiles_y;
    const int kblocks = (p.Kg + G::KB - 1) / G::KB;
    const size_t buf_bytes = 2 * (size_t)G::BUF * sizeof(float);
    const size_t red_per_tile = (size_t)G::KPL * G::ACC * 64 * sizeof(float);
    // clocks of SIMD issue time for one wavefront on one channel: a bit test and branch per
    // position, and per nonzero a broadcast plus its share of the tile's 9*ACC*KPL FMAs
    const double nnz = 0.3 * G::NPOS;
    const double t_channel = 60.0 + 6.0 * G::NPOS + nnz * (14.0 + 4.5 * 9.0 * G::ACC * G::KPL / G::NPOS);
    const double stage_clocks = (double)G::KB * p.Cg * 36.0 / 64.0;

    int pin_nwv = 0, pin_ncs = 0, pin_nss = 0;   // tuning aid: SCONV_TAP_SPLIT="nwv,ncs[,nss]"
    pinned_split("SCONV_TAP_SPLIT", &pin_nwv, &pin_ncs, &pin_nss);
    const int nchunks = p.Cg / G::CCH;
    // a launch that leaves half of the compute units idle even with one tile and 64 filters per
    // workgroup
    const long long tile_wgs = (long long)cfg.ntiles * ((p.Kg + 63) / 64) * p.N * p.G;
    const bool small = tile_wgs < 128;
    const bool large = tile_wgs >= 512;   // several rounds of workgroups
    // a few workgroups per compute unit, each walking 16 or more chunks: still a chain of chunk
    // latencies with little to overlap it
    const bool mid = !small && tile_wgs <= 768 && nchunks >= 16;
    const size_t part_bytes = (size_t)p.N * p.K * p.OH * p.OW * sizeof(float);
    auto split_fits = [&](int nss) {
        return !G::POOL && nss <= nchunks && nss * part_bytes <= split_scratch_bytes() &&
               (long long)p.N * p.G * nss <= 65535;
    };
    // a pinned decomposition is priced as it is; the model ranks the unsplit decompositions and
    // splits the winner afterwards
    const int nss = pin_nss ? pin_nss : 1;
    if (nss > 1 && (split == 0 || !split_fits(nss))) return best;
    if (pin_nss == 1 && split == 2) return best;
    // (a fused call takes plain tiles plus the pooling second kernel only when the launch is too small to
    // fill the chip otherwise: the convolution tensor of a larger one stays on chip, Section 6.4)
    if (!pin_nss && split == 2 && !small) return best;
    // measured on mid-sized launches: one filter per lane (twice the workgroups) with the channels
    // split beats two filters per lane, which the pricing below would prefer
    if (mid && split >= 1 && G::KPL > 1 && !pin_nss && !pin_nwv && !pinned_geom("SCONV_TAP_GEOM")) return best;
    // Mid-sized launches, measured: whole-map tiles (as many channel slices as wavefronts) run 10 %
    // faster split across workgroups with eight longer slices than with sixteen (512 @7x7, batch 16
    // and 32); smaller tiles run fastest as 2 tiles x 8 slices on every shape tried (14x14 and 28x28
    // maps, 256-512 channels, batch 4-32: sconv_tune's pick each time, 5-20 % ahead of 16 slices).
    // The first scan keeps to those; the second takes anything if they do not fit.
    const bool steer = mid && split >= 1 && !pin_nwv && !pin_nss;
    for (int scan = steer ? 0 : 1; scan < 2 && best.cost < 0.0; ++scan)
    for (int nwv = 8; nwv <= G::MAXW; nwv *= 2) {
        for (int ncs = 1; ncs <= nwv && ncs <= G::CCH; ncs *= 2) {
            const int nt = nwv / ncs;
            if (pin_nwv && (pin_nwv != nwv || pin_ncs != ncs)) continue;
            if (scan == 0 && (cfg.ntiles == 1 ? nwv != 8 : (nwv != 16 || ncs != 8))) continue;
            // the slice reduction reuses the filter buffers; a large tile's partial sums need more
            size_t lds_bytes = buf_bytes;
            if (ncs > 1 && nt * red_per_tile > lds_bytes) lds_bytes = nt * red_per_tile;
            if (lds_bytes > 160 * 1024) continue;
            const int occ = nwv == 16 ? occupancy<G, G::MAXW>(lds_bytes) : occupancy<G, 8>(lds_bytes);
            if (!pin_nwv && nt > 1 && nt / 2 >= cfg.ntiles) continue;   // half of the tile slots empty
            const long long wgs1 = (long long)((cfg.ntiles + nt - 1) / nt) * kblocks * p.N * p.G;
            if (nss > 1 && wgs1 >= 512 && current_pin()) continue;   // sconv_tune: not worth a trial
            const long long wgs = wgs1 * nss;
            const int rw = ncs > 1 ? (int)(lds_bytes / (nt * red_per_tile)) : 1;
            int red_steps = 0;   // of the slice reduction: the kernel's own loop
            for (int active = ncs; active > 1; ++red_steps) active -= rw < active / 2 ? rw : active / 2;
            const long long slots = 256LL * occ;
            const double per_cu = wgs >= slots ? occ : (double)((wgs + 255) / 256);  // resident workgroups
            double rounds, r, t_chunk;
            if (large) {
                // Launches of several rounds, fitted to measured times.  Rounds as a fraction: in a
                // last, partly filled round the resident workgroups run faster.  r: time for the wv
                // wavefronts of a SIMD to get through one channel each, in units of t_channel - a
                // wavefront's test - broadcast - multiply chain waits on itself, so resident
                // wavefronts overlap (2.9 at four per SIMD, 4.7 at eight).  The barrier and staging
                // wait per chunk shows at low residency (2900 clocks at four per SIMD) and hides at
                // high (400 at eight).
                rounds = wgs >= slots ? (double)wgs / slots : 1.0;
                double wv = per_cu * nwv / 4.0;
                if (wv < 2.0) wv = 2.0;
                r = 1.2 + 0.44 * wv;
                t_chunk = 2900.0 - 625.0 * (wv - 4.0);
                t_chunk = t_chunk > 2900.0 ? 2900.0 : (t_chunk < 400.0 ? 400.0 : t_chunk);
            } else {
                // up to a round or two: whole rounds, SIMDs saturating at four resident wavefronts
                rounds = (double)((wgs + slots - 1) / slots);
                r = per_cu * nwv / 4.0;
                if (r < 4.0) r = 4.0;
                t_chunk = 0.0;
            }
            const double cost = rounds * ((double)p.Cg / ncs * t_channel * r + nchunks * t_chunk +
                                          per_cu * stage_clocks) / nss +
                                red_steps * 2000.0 +                             // reduction steps
                                (nss > 1 ? 9000.0 : 0.0);                        // second kernel
            if (best.cost < 0.0 || cost < best.cost) {
                best.cost = cost;
                best.cfg = cfg;
                best.cfg.NT = nt;
                best.cfg.NCS = ncs;
                best.cfg.CPW = G::CCH / ncs;
                best.nwv = nwv;
                best.kblocks = kblocks;
                best.lds_bytes = lds_bytes;
                best.nss = nss;
                best.cfg.NSS = nss;
                best.cfg.RW = rw;
                best.wgs1 = wgs1;
            }
        }
    }
    if (!pin_nss && split && small && best.cost >= 0.0) {
        // the model's split: the smallest power of two that gives every compute unit a workgroup
        // and leaves each workgroup two chunks or more
        int want = split == 2 ? 2 : 1;
        while (want < 16 && best.wgs1 * want < 256 && want * 4 <= nchunks) want *= 2;
        if (want > 1 && !split_fits(want)) want = 1;
        if (want == 1 && split == 2) return Plan();
        best.nss = best.cfg.NSS = want;
        if (want > 1) best.cost = best.cost / want + 9000.0;
    }
    if (!pin_nss && split == 1 && mid && best.cost >= 0.0) {
        // mid-sized launches (up to 768 tile-workgroups): up to 768 workgroups (a round and a half of two
        // per compute unit) of four chunks or more, four ways at most (512 channels @14x14: batch 4 57 -> 46 us, batch 8
        // 87 -> 64, with fused pooling 71 -> 65; @7x7: batch 16 56 -> 43, batch 32 80 -> 72)
        int want = 1;
        // and every wavefront keeps 16 channels or more (fewer do not pay for the slice reduction
        // and the tile epilogue, which every workgroup runs: 512 @7x7 at batch 32, 16 slices, four
        // ways 102 against 80 us unsplit)
        while (want < 4 && best.wgs1 * want * 2 <= 768 && want * 2 * 4 <= nchunks &&
               p.Cg / (best.cfg.NCS * want * 2) >= 16)
            want *= 2;
        if (want > 1 && split_fits(want)) {
            best.nss = best.cfg.NSS = want;
            best.cost = best.cost / want + 9000.0;
        }
    }
    return best;
}

template <class G>
int launch_plan(const Plan& pl, const Problem& p, bool pooled, const float* x, const float* w, float* y,
                hipStream_t stream)
{
    const size_t lds_bytes = pl.lds_bytes;
    const long long gx = (pl.cfg.ntiles + pl.cfg.NT - 1) / pl.cfg.NT;
    const long long gz = (long long)p.N * p.G * pl.nss;
    if (gz > 65535 || pl.kblocks > 65535 || gx >= (1LL << 31)) return SCONV_EUNSUPPORTED;
    const dim3 grid((unsigned)gx, (unsigned)pl.kblocks, (unsigned)gz);
    Problem q = p;
    float* out = y;
    if (pl.nss > 1) {
        // raw partial sums of every channel range into the scratch slices; the second kernel below
        // adds them and applies the epilogue
        if (G::POOL || pl.nss > p.Cg / G::CCH ||
            (size_t)pl.nss * p.N * p.K * p.OH * p.OW * sizeof(float) > split_scratch_bytes())
            return SCONV_EUNSUPPORTED;
        out = split_scratch(stream);
        if (!out) return SCONV_EUNSUPPORTED;
        q.relu = 0;
        q.bias = nullptr;
    } else if (pooled != G::POOL) {
        return SCONV_EUNSUPPORTED;
    }
    int rc;
    if (G::MAXW == 16 && pl.nwv == 16)
        rc = launch_nwv<G, G::MAXW>(q, pl.cfg, grid, lds_bytes, x, w, out, stream);
    else
        rc = launch_nwv<G, 8>(q, pl.cfg, grid, lds_bytes, x, w, out, stream);
    if (rc != SCONV_OK || pl.nss == 1) return rc;
    return launch_split_reduce(p, pooled, out, pl.nss, y, stream);
}

// Geometries.  Generic: 5x7 output tiles with halo (63 input positions, one register).  Maps
// 7 wide and 7 high: one 7x7 tile, no halo (padding contributes nothing).  Pooled: even tiles,
// 4x14 without column halo for 14-wide maps, or 4x6 with halo.
using G57_1 = Geom<1, 5, 7, 1, 1, false>;
using G57_2 = Geom<2, 5, 7, 1, 1, false>;
using G77_1 = Geom<1, 7, 7, 0, 0, false>;
using G77_2 = Geom<2, 7, 7, 0, 0, false>;
using P414_1 = Geom<1, 4, 14, 1, 0, true>;
using P414_2 = Geom<2, 4, 14, 1, 0, true>;
using P46_1 = Geom<1, 4, 6, 1, 1, true>;
using P46_2 = Geom<2, 4, 6, 1, 1, true>;
using S34_1 = Geom<1, 3, 4, 1, 1, false, 2>;   // stride 2: 7x9 input positions feed 3x4 outputs
using S34_2 = Geom<2, 3, 4, 1, 1, false, 2>;

bool shape_ok(const Problem& p, bool pooled)
{
    if (p.R != 3 || p.S != 3 || p.pad != 1) return false;
    if (p.stride != 1 && !(p.stride == 2 && !pooled)) return false;
    if (p.Cg % 16) return false;                      // whole staged chunks of channels only
    if (pooled && (p.ph != 2 || p.pw != 2 || p.ps != 2)) return false;
    return true;
}

struct Candidate {
    const char* name;
    Plan (*plan)(const Problem&, int);
    int (*launch)(const Plan&, const Problem&, bool, const float*, const float*, float*, hipStream_t);
    bool pooled;
    int kpl;              // filters per lane: needs more than 64*(kpl-1) filters in the group
    int need_h, need_w;   // map height / width the geometry is built for (0 = any)
    int stride;
    bool by_model;        // false: only when pinned (sconv_tune tries it; the cost model was not
                          // calibrated on it)
};

// Adapters for the transposed-filter kernel's geometries (sconv_tapt.hip plans and launches them).
#define SCONV_TAPT_ADAPT(NAME)                                                                             \
    Plan plan_t_##NAME(const Problem& p, int split)                                                        \
    {                                                                                                      \
        const TaptPlan t = tapt_plan_##NAME(p, split);                                                     \
        Plan pl;                                                                                           \
        pl.cost = t.cost; pl.nwv = t.nwv; pl.cfg.NCS = t.ncs; pl.cfg.NT = t.nt; pl.nss = t.nss;            \
        pl.split_mode = split;                                                                             \
        return pl;                                                                                         \
    }                                                                                                      \
    int launch_t_##NAME(const Plan& pl, const Problem& p, bool pooled, const float* x, const float* w,     \
                        float* y, hipStream_t stream)                                                      \
    {                                                                                                      \
        return tapt_launch_##NAME(p, pooled, pl.split_mode, x, w, y, stream);                              \
    }
SCONV_TAPT_ADAPT(5x7k1)
SCONV_TAPT_ADAPT(5x7k1n)
SCONV_TAPT_ADAPT(5x7k2)
SCONV_TAPT_ADAPT(7x7k1)
SCONV_TAPT_ADAPT(7x7k2)
SCONV_TAPT_ADAPT(p4x14k1)
SCONV_TAPT_ADAPT(p4x6k1)
SCONV_TAPT_ADAPT(p4x6k2)
SCONV_TAPT_ADAPT(p2x14k2)
SCONV_TAPT_ADAPT(p2x14k1)
SCONV_TAPT_ADAPT(p2x14hk1)
SCONV_TAPT_ADAPT(p2x14hk2)
SCONV_TAPT_ADAPT(s2_3x4k1)
SCONV_TAPT_ADAPT(s2_3x4k2)

const Candidate kCandidates[] = {
    {"5x7k1", plan_geom<G57_1>, launch_plan<G57_1>, false, 1, 0, 0, 1, true},
    {"5x7k2", plan_geom<G57_2>, launch_plan<G57_2>, false, 2, 0, 0, 1, true},
    {"7x7k1", plan_geom<G77_1>, launch_plan<G77_1>, false, 1, 7, 7, 1, true},
    {"7x7k2", plan_geom<G77_2>, launch_plan<G77_2>, false, 2, 7, 7, 1, true},
    {"p4x14k1", plan_geom<P414_1>, launch_plan<P414_1>, true, 1, 0, 14, 1, true},
    {"p4x14k2", plan_geom<P414_2>, launch_plan<P414_2>, true, 2, 0, 14, 1, true},
    {"p4x6k1", plan_geom<P46_1>, launch_plan<P46_1>, true, 1, 0, 0, 1, true},
    {"p4x6k2", plan_geom<P46_2>, launch_plan<P46_2>, true, 2, 0, 0, 1, true},
    {"5x7k1t", plan_t_5x7k1, launch_t_5x7k1, false, 1, 0, 0, 1, false},
    {"5x7k1tn", plan_t_5x7k1n, launch_t_5x7k1n, false, 1, 0, 0, 1, false},
    {"5x7k2t", plan_t_5x7k2, launch_t_5x7k2, false, 2, 0, 0, 1, false},
    {"7x7k1t", plan_t_7x7k1, launch_t_7x7k1, false, 1, 7, 7, 1, false},
    {"7x7k2t", plan_t_7x7k2, launch_t_7x7k2, false, 2, 7, 7, 1, false},
    {"p4x14k1t", plan_t_p4x14k1, launch_t_p4x14k1, true, 1, 0, 14, 1, false},
    {"p4x6k1t", plan_t_p4x6k1, launch_t_p4x6k1, true, 1, 0, 0, 1, false},
    {"p4x6k2t", plan_t_p4x6k2, launch_t_p4x6k2, true, 2, 0, 0, 1, false},
    {"p2x14k2t", plan_t_p2x14k2, launch_t_p2x14k2, true, 2, 0, 14, 1, false},
    {"p2x14k1t", plan_t_p2x14k1, launch_t_p2x14k1, true, 1, 0, 14, 1, false},
    {"p2x14hk1t", plan_t_p2x14hk1, launch_t_p2x14hk1, true, 1, 0, 0, 1, false},
    {"p2x14hk2t", plan_t_p2x14hk2, launch_t_p2x14hk2, true, 2, 0, 0, 1, false},
    {"s2-3x4k1t", plan_t_s2_3x4k1, launch_t_s2_3x4k1, false, 1, 0, 0, 2, false},
    {"s2-3x4k2t", plan_t_s2_3x4k2, launch_t_s2_3x4k2, false, 2, 0, 0, 2, false},
    {"s2-3x4k1", plan_geom<S34_1>, launch_plan<S34_1>, false, 1, 0, 0, 2, true},
    {"s2-3x4k2", plan_geom<S34_2>, launch_plan<S34_2>, false, 2, 0, 0, 2, true},
};

}  // namespace

const char* const* tap_geoms()
{
    static const char* const names[] = {"5x7k1", "5x7k2", "7x7k1", "7x7k2", "p4x14k1", "p4x14k2", "p4x6k1", "p4x6k2",
                                        "s2-3x4k1", "s2-3x4k2", "5x7k1t", "5x7k1tn", "5x7k2t", "7x7k1t", "7x7k2t", "p4x14k1t", "p4x6k1t",
                                        "p4x6k2t", "p2x14k2t", "p2x14k1t", "p2x14hk1t", "p2x14hk2t", "s2-3x4k1t", "s2-3x4k2t", nullptr};
    return names;
}

bool tap_supported(const Problem& p, bool pooled) { return shape_ok(p, pooled); }

namespace {
// The candidate and decomposition a launch on `stream` would get (the dispatcher has selected the
// stream's workspace); null when no tile plan applies.
const Candidate* select_tap(const Problem& p, bool pooled, hipStream_t stream, Plan* plan_out)
{
    if (!shape_ok(p, pooled)) return nullptr;
    const char* pin = pinned_geom("SCONV_TAP_GEOM");   // tuning aid: candidate name
    const Candidate* best = nullptr;
    Plan best_plan;
    // a channel split across workgroups needs a workspace lent for the stream
    const bool can_split = split_scratch_possible(stream);
    // Large launches with a workspace that holds a transposed copy of the filters: the kernel without
    // LDS staging (sconv_tapt.hip) measures 5-13 % faster on every launch of 512 or more tile-workgroups
    // with 128 or more channels per group tried (512 @28x28 batch 8: 231 -> 210 us; 512 @14x14 batch 32:
    // 190 -> 168; 256 @14x14 batch 32: 63 -> 55; 896 in 7 groups @14x14 batch 32: 130 -> 126), and its
    // pooled tiles beat both the staged pooled tiles and the split plain tiles (512 @14x14 + pooling at
    // batch 8: 61 against 71 and 65 us; on wider maps 2x14 pooled tiles with a column halo - 64 input
    // positions, one register - : 512 @28x28 + pooling at batch 8 202 us, 256 @28x28 at batch 16 124, 128 @56x56
    // at batch 8 71, against 257, 146 and 78 on the matrix kernel's pooled tiles).
    int dn = 0, dc = 0, ds = 0;
    pinned_split("SCONV_TAP_SPLIT", &dn, &dc, &ds);
    // With prepared filters (the call brings the transposed copy: no transposition before the launch) the same
    // kernel also leads on smaller launches and on whole-map tiles - 512 @7x7 at batch 32: 64 against 72 us,
    // 2048 in 16 groups @7x7: 58 against 70, 384 @5x5 in 2 groups: 18 against 22 - and, split over workgroups,
    // on batch-1 layers of 64 M multiply-adds or more (512 @28x28: 40 against 46 us on the matrix kernel's
    // split tiles, 512 @14x14: 20.5 against 24.6, 256 @14x14: 13.6 against 15.8; smaller ones are level or
    // behind the staged kernel: two launches take 13.5 us whatever they hold).
    const bool prep = p.wprep != nullptr;
    const bool whole_map = p.H <= 7 && p.W <= 7;
    if (!pin && !dn && (can_split || prep) && p.stride == 1 && p.Cg >= 128 && !(whole_map && (pooled || !prep))) {
        const long long tile_wgs = (long long)((p.OH + 4) / 5) * ((p.OW + 6) / 7) * ((p.Kg + 63) / 64) * p.N * p.G;
        const double macs = (double)p.N * p.K * p.OH * p.OW * p.Cg * 9.0;
        const char* want = nullptr;
        // split argument of the plan: 0 none, 1 allowed, 2 plain tiles serving a fused call
        int mode = prep && can_split && !pooled ? 1 : 0;
        if (tile_wgs >= (prep ? 128 : (pooled ? 256 : 512)))   // (pooled: measured from 384 up)
            // (below about 85 % zeros the test of four positions at once rarely spares the four single
            // tests: the form without it measures 2-4 % faster when the caller reported such a ratio)
            want = !pooled ? (p.H == 7 && p.W == 7 ? "7x7k1t" : (p.zhint >= 0.0f && p.zhint < 0.85f ? "5x7k1tn" : "5x7k1t"))
                           : (p.W == 14 ? (p.Kg >= 128 && !prep ? "p2x14k2t" : (prep ? "p2x14k1t" : "p4x14k1t")) : "p2x14hk1t");
        else if (prep && can_split && macs >= 64e6) {
            // (5x7 tiles also on 7x7 maps: two tiles per image instead of one)
            want = p.zhint >= 0.0f && p.zhint < 0.85f ? "5x7k1tn" : "5x7k1t";
            mode = pooled ? 2 : 1;
        }
        for (const Candidate& c : kCandidates) {
            if (!want || strcmp(want, c.name) != 0) continue;
            if (c.need_h && p.H != c.need_h) continue;
            if (c.need_w && p.W != c.need_w) continue;
            const Plan pl = c.plan(p, mode);
            if (pl.cost >= 0.0) {
                best = &c;
                best_plan = pl;
            }
        }
    }
    // A pooled layer: first the plain tiles with the split (the second kernel pools), which the
    // model offers for small launches only; the pooled tiles when none applies.
    for (int pass = pooled && can_split ? 0 : 1; pass < 2 && !best; ++pass) {
        for (const Candidate& c : kCandidates) {
            if (c.stride != p.stride) continue;
            if (c.pooled != (pooled && pass == 1)) continue;
            if (p.Kg <= 64 * (c.kpl - 1)) continue;
            if (c.need_h && p.H != c.need_h) continue;
            if (c.need_w && p.W != c.need_w) continue;
            if (pin ? strcmp(pin, c.name) != 0 : !c.by_model) continue;
            const Plan pl = c.plan(p, c.pooled != pooled ? 2 : (can_split && !c.pooled ? 1 : 0));
            if (pl.cost < 0.0) continue;
            if (!best || pl.cost < best_plan.cost) {
                best = &c;
                best_plan = pl;
            }
        }
    }
    if (best) *plan_out = best_plan;
    return best;
}
}  // namespace

int launch_tap(const Problem& p, bool pooled, const float* x, const float* w, float* y,
               hipStream_t stream)
{
    Plan best_plan;
    const Candidate* best = select_tap(p, pooled, stream, &best_plan);
    if (!best) return SCONV_EUNSUPPORTED;
    if (env_value("SCONV_TRACE_PLAN"))
        fprintf(stderr, "sconv: tap3x3 %s nwv=%d ncs=%d nt=%d nss=%d cost=%.0f\n", best->name, best_plan.nwv,
                best_plan.cfg.NCS, best_plan.cfg.NT, best_plan.nss, best_plan.cost);
    return best->launch(best_plan, p, pooled, x, w, y, stream);
}

bool describe_tap(const Problem& p, bool pooled, hipStream_t stream, char* out, size_t out_size)
{
    Plan pl;
    const Candidate* c = select_tap(p, pooled, stream, &pl);
    if (!c) return false;
    if (pl.nss > 1)
        snprintf(out, out_size, "%s/%dx%dx%d", c->name, pl.nwv, pl.cfg.NCS, pl.nss);
    else
        snprintf(out, out_size, "%s/%dx%d", c->name, pl.nwv, pl.cfg.NCS);
    return true;
}

}  // namespace sconv

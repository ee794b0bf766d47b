// Host side of libsconv: argument checks, size helpers, variant choice.  No device code here.
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <array>
#include <atomic>
#include <string>
#include <map>
#include <vector>
#include <mutex>

#include "sconv_internal.h"

namespace sconv {

// The pin of the launch in progress, per calling thread.
static thread_local const PlanPin* g_pin = nullptr;

const PlanPin* current_pin() { return g_pin; }

// The tuning-aid environment (SCONV_*), read once - at the first call that looks - and again only when
// sconv_env_refresh is called: no launch pays for getenv.
static const char* const kEnvNames[] = {
    "SCONV_VARIANT", "SCONV_TAP_GEOM", "SCONV_QUAD_GEOM", "SCONV_WIDE_GEOM", "SCONV_GEN_GEOM", "SCONV_PW_GEOM",
    "SCONV_TAP_SPLIT", "SCONV_QUAD_SPLIT", "SCONV_WIDE_SPLIT", "SCONV_GEN_SPLIT", "SCONV_PW_SPLIT",
    "SCONV_ENCODE", "SCONV_TRACE_PLAN", "SCONV_NO_XCD_REMAP", "SCONV_ENCODE_TR16"};
constexpr int kEnvCount = (int)(sizeof(kEnvNames) / sizeof(kEnvNames[0]));
static std::mutex g_env_lock;
static std::atomic<bool> g_env_read{false};
static std::string g_env_val[kEnvCount];
static bool g_env_set[kEnvCount];

static void env_load_locked()
{
    for (int i = 0; i < kEnvCount; ++i) {
        const char* v = getenv(kEnvNames[i]);
        g_env_set[i] = v != nullptr;
        g_env_val[i] = v ? v : "";
    }
    g_env_read.store(true, std::memory_order_release);
}

const char* env_value(const char* name)
{
    if (!g_env_read.load(std::memory_order_acquire)) {
        std::lock_guard<std::mutex> lock(g_env_lock);
        if (!g_env_read.load(std::memory_order_relaxed)) env_load_locked();
    }
    for (int i = 0; i < kEnvCount; ++i)
        if (!strcmp(name, kEnvNames[i])) return g_env_set[i] ? g_env_val[i].c_str() : nullptr;
    return nullptr;
}

const char* pinned_geom(const char* env_name)
{
    if (g_pin) return g_pin->geom[0] ? g_pin->geom : nullptr;
    return env_value(env_name);
}

void pinned_split(const char* env_name, int* nwv, int* ncs, int* nss)
{
    int dummy = 0;
    if (!nss) nss = &dummy;
    *nwv = *ncs = *nss = 0;
    if (g_pin) {
        *nwv = g_pin->nwv;
        *ncs = g_pin->ncs;
        *nss = g_pin->nwv ? (g_pin->nss > 1 ? g_pin->nss : 1) : 0;
        return;
    }
    if (const char* pin = env_value(env_name)) {
        const int got = sscanf(pin, "%d,%d,%d", nwv, ncs, nss);
        if (got == 2) *nss = 1;
        else if (got != 3) *nwv = *ncs = *nss = 0;
    }
}

static bool mul_fits_31(int64_t a, int64_t b, int64_t c, int64_t d)
{
    // every factor is positive and below 2^31, so partial products cannot overflow int64
    int64_t ab = a * b;
    if (ab >= (int64_t(1) << 31)) return false;
    int64_t abc = ab * c;
    if (abc >= (int64_t(1) << 31)) return false;
    return abc * d < (int64_t(1) << 31);
}

int fill_problem(const sconv_desc_t* d, bool pooled, Problem* out)
{
    if (!d || !out) return SCONV_EINVAL;
    if (d->N <= 0 || d->C <= 0 || d->H <= 0 || d->W <= 0 || d->K <= 0 || d->R <= 0 || d->S <= 0)
        return SCONV_EINVAL;
    if (d->stride <= 0 || d->pad < 0 || d->groups <= 0) return SCONV_EINVAL;
    if (d->C % d->groups || d->K % d->groups) return SCONV_EINVAL;
    if (d->pad >= d->R || d->pad >= d->S) return SCONV_EINVAL;
    if (d->flags & ~(SCONV_RELU | SCONV_PREPARED_FILTERS | SCONV_ZERO_RATIO_MASK)) return SCONV_EINVAL;
    if (d->H + 2 * (int64_t)d->pad < d->R || d->W + 2 * (int64_t)d->pad < d->S) return SCONV_EINVAL;

    Problem p;
    memset(&p, 0, sizeof(p));
    p.N = d->N; p.C = d->C; p.H = d->H; p.W = d->W;
    p.K = d->K; p.R = d->R; p.S = d->S;
    p.stride = d->stride; p.pad = d->pad; p.G = d->groups;
    p.Cg = d->C / d->groups;
    p.Kg = d->K / d->groups;
    // (in 64 bits: H + 2*pad can pass 2^31 with a large pad under a larger kernel)
    const int64_t oh64 = (d->H + 2 * (int64_t)d->pad - d->R) / d->stride + 1;
    const int64_t ow64 = (d->W + 2 * (int64_t)d->pad - d->S) / d->stride + 1;
    if (oh64 >= (int64_t(1) << 31) || ow64 >= (int64_t(1) << 31)) return SCONV_EUNSUPPORTED;
    p.OH = (int)oh64;
    p.OW = (int)ow64;
    p.relu = (d->flags & SCONV_RELU) ? 1 : 0;
    const int zcode = (d->flags & SCONV_ZERO_RATIO_MASK) >> SCONV_ZERO_RATIO_SHIFT;   // 0: not given
    p.zhint = zcode ? (float)(zcode - 1) / 254.0f : -1.0f;
    p.wprep = nullptr;
    if (pooled) {
        if (d->pool_h <= 0 || d->pool_w <= 0 || d->pool_stride <= 0) return SCONV_EINVAL;
        if (d->pool_h > p.OH || d->pool_w > p.OW) return SCONV_EINVAL;
        p.ph = d->pool_h; p.pw = d->pool_w; p.ps = d->pool_stride;
        p.PH = (p.OH - p.ph) / p.ps + 1;
        p.PW = (p.OW - p.pw) / p.ps + 1;
        p.relu = 1;
    }
    // (factor by factor: Cg * R * S of three values near 2^31 does not fit 64 bits)
    const int64_t CR = (int64_t)p.Cg * p.R;
    if (CR >= (int64_t(1) << 24)) return SCONV_EUNSUPPORTED;
    const int64_t L = CR * p.S;
    if (L >= (int64_t(1) << 24)) return SCONV_EUNSUPPORTED;
    p.L = (int)L;
    if (!mul_fits_31(p.N, p.C, p.H, p.W) || !mul_fits_31(p.K, p.Cg, p.R, p.S) ||
        !mul_fits_31(p.N, p.K, p.OH, p.OW))
        return SCONV_EUNSUPPORTED;
    *out = p;
    return SCONV_OK;
}

enum Variant { V_ROWS, V_TAP, V_QUAD, V_PW, V_WIDE, V_GEN };

static const char* variant_name(Variant v)
{
    switch (v) {
    case V_PW: return "quad1x1";
    case V_QUAD: return "quad3x3";
    case V_TAP: return "tap3x3";
    case V_WIDE: return "wide3x3";
    case V_GEN: return "gen";
    default: return "rows";
    }
}

// What sconv_tune found fastest for one descriptor: a variant and its decomposition.
struct Tuned {
    Variant v;
    PlanPin pin;
    bool pinned;          // false: the variant with its cost model's decomposition
    float ms;
    char name[48];
};
typedef std::array<int32_t, 17> TuneKey;   // the descriptor's fields, the pooled flag, the density bucket,
                                           // whether the call brings prepared filters

static std::mutex g_lock;                  // planning, enqueueing and the tuning cache
static std::map<TuneKey, Tuned> g_tuned;

// Density bucket of a call: 0 = no zero ratio given, 1 = below 55 % zeros, 2 = 55-80 %, 3 = above.  Tuned
// plans are kept per bucket, so that layers of one shape with different densities keep their own.
static int density_bucket(const Problem& p)
{
    if (p.zhint < 0.0f) return 0;
    return p.zhint < 0.55f ? 1 : (p.zhint < 0.8f ? 2 : 3);
}

static TuneKey tune_key(const Problem& p, bool pooled)
{
    return TuneKey{p.N, p.C, p.H, p.W, p.K, p.R, p.S, p.stride, p.pad, p.G,
                   pooled ? p.ph : 0, pooled ? p.pw : 0, pooled ? p.ps : 0, p.relu, pooled ? 1 : 0,
                   density_bucket(p), p.wprep ? 1 : 0};
}

// The tuned entry for this problem, unless SCONV_VARIANT pins the variant.  Caller holds g_lock.
static const Tuned* tuned_for(const Problem& p, bool pooled)
{
    if (env_value("SCONV_VARIANT")) return nullptr;
    auto it = g_tuned.find(tune_key(p, pooled));
    if (it == g_tuned.end() && p.zhint >= 0.0f) {   // nothing tuned at this density: a plan tuned without one
        Problem q = p;
        q.zhint = -1.0f;
        it = g_tuned.find(tune_key(q, pooled));
    }
    return it == g_tuned.end() ? nullptr : &it->second;
}

// Small launches of the matrix kernel that a workspace lets split: on maps 28 or more wide with 128 or
// more channels per group, a launch of 200 to 400 two-row tiles (100 to 400 with 512 or more
// channels) runs as one-filter-per-lane tiles, 8 wavefronts x 4 channel slices, with the channels of a
// tile split over enough workgroups to make about 450 of them.  Against the vector kernel's plan
// that measures 1.2-1.8x faster at 50 % zeros and 0.95-1.4x at 80 % (256 channels @56x56 at batch 1
// 51 against 75 us at 60 %, 512 @28x28 48 against 69 at 75 %, 128->32 @28x28 at batch 16 30 against
// 36 at 70 %); smaller launches, and maps whose width leaves the second 28-column tile mostly empty,
// stay with the vector kernel.
static bool small_quad_split(const Problem& p, bool pooled, PlanPin* pin)
{
    if (pooled || p.W < 28 || p.Cg < 128 || !quad_supported(p, pooled)) return false;
    const int wtiles = (p.OW + 27) / 28;
    if (wtiles * 28 * 3 > p.OW * 4) return false;  // more than a quarter of the tile columns empty
    const long long tiles = (long long)((p.OH + 1) / 2) * wtiles * ((p.Kg + 63) / 64) * p.N * p.G;
    if (tiles >= 400 || tiles < (p.Cg >= 512 ? 100 : 200)) return false;
    const long long wgs1 = (tiles + 1) / 2;        // two tiles per workgroup
    int nss = 2;
    while (wgs1 * nss < 448 && nss < 16) nss *= 2;
    if (wgs1 * nss < 448 || nss > p.Cg / 16) return false;
    if (pin) {
        memset(pin, 0, sizeof(*pin));
        snprintf(pin->geom, sizeof(pin->geom), "q32k1");
        pin->nwv = 8;
        pin->ncs = 4;
        pin->nss = nss;
    }
    return true;
}

// Launches of a handful of tiles with short channel loops (batch 1, up to 160 channels per group): the
// general matrix kernel splits their columns over workgroups finer than the vector kernel splits its
// 16-channel chunks and measures 1.15-1.25x faster (3x3 64 @56x56 at batch 1: 15.7 against 19.5 us; 128 -> 32
// @28x28: 14.5 against 18.2; 128 stride 2 @56x56: 17.1 against 21.2; 896 in 7 groups @14x14: 19.4 against
// 22.5); deeper layers (256 channels and more) stay with the vector kernel.
static bool small_gen_split(const Problem& p, bool pooled, bool have_ws)
{
    if (!have_ws || pooled || p.R != 3 || p.S != 3 || p.Cg > 160 || p.Cg < 64 || !gen_supported(p, pooled)) return false;
    const long long tile_wgs = (long long)((p.OH + 4) / 5) * ((p.OW + 6) / 7) * ((p.Kg + 63) / 64) * p.N * p.G;
    return tile_wgs < 128 && p.H > 7;
}

// The static rules.  have_ws: a workspace is lent (the split plans of the matrix kernel need one;
// the vector and general kernels decide on their own).  When the choice comes with a fixed
// decomposition, *static_pin receives it (geom[0] != 0).
//
// z: the map's zero ratio when the caller reported one (the zero-ratio field of the descriptor's flags), negative when unknown.
// Known, it moves 3x3 / stride 1 / pad 1 launches that fill the matrix kernels' tiles along the
// crossovers measured on the zero-ratio sweeps (independent zeros; 896 channels in 7 groups @14x14 at
// batch 32 and 256 channels @56x56 at batch 8): below 68 % zeros whole groups are almost never empty and
// the matrix kernels run at their dense rate, which the vector kernel only matches from about 68 %;
// from 92 % the 6-element granule of quad3x3 is empty often enough to lead again.
static Variant choose(const Problem& p, bool pooled, bool have_ws = false, PlanPin* static_pin = nullptr,
                      float z = -1.0f)
{
    // the vector kernel's transposed-filter form needs the transposed filters: brought by the call, or room
    // for them in a workspace
    const bool have_wt = have_ws || p.wprep != nullptr;
    if (static_pin) memset(static_pin, 0, sizeof(*static_pin));
    const char* pin = env_value("SCONV_VARIANT");
    if (pin && !strcmp(pin, "rows")) return V_ROWS;
    if (pin && !strcmp(pin, "tap")) return tap_supported(p, pooled) ? V_TAP : V_ROWS;
    if (pin && !strcmp(pin, "wide")) return wide_supported(p, pooled) ? V_WIDE : V_ROWS;
    if (pin && !strcmp(pin, "quad")) return quad_supported(p, pooled) ? V_QUAD : V_ROWS;
    if (pin && !strcmp(pin, "gen")) return gen_supported(p, pooled) ? V_GEN : V_ROWS;
    if (pw_supported(p, pooled)) {
        // A 1x1 layer of few 32-position tiles walking 512 or more channels is one latency chain per
        // workgroup, the longer the more channels: the general kernel, which splits such a launch's
        // columns over workgroups, measures 1.1-1.7x faster up to about 0.3 tiles per channel (512
        // channels: 1.25x at 100 tiles, level at 200; 1024: 1.7x at 100, 1.4x at 200; 2048: 1.7x at 200).
        const long long pw_tiles = ((long long)p.N * p.H * p.W + 31) / 32 * ((p.Kg + 63) / 64) * p.G;
        // (the split needs a workspace; without one only launches of fewer than 64 tiles go there)
        if (p.Cg >= 512 && (pw_tiles < 64 || (have_ws && pw_tiles * 16 < 5LL * p.Cg)) && gen_supported(p, pooled))
            return V_GEN;
        return V_PW;
    }
    // The 16-row granule needs many tile-wavefronts (64 window rows x 64 filters each) to fill the
    // chip: it splits the channels of a tile four ways at most.
    const long long rows = pooled ? (long long)p.N * p.PH * p.PW * 4 : (long long)p.N * p.OH * p.OW;
    const bool wide_fills = wide_supported(p, pooled) &&
                            ((rows + 63) / 64) * ((p.Kg + 63) / 64) * p.G >= 128;
    if (quad_supported(p, pooled)) {
        // Maps of 7x7 and below are one whole-map tile of the vector kernel (no halo, no ragged
        // tiles); it measures 1.4-1.8x faster there than either matrix kernel.
        if (p.H <= 7 && p.W <= 7 && tap_supported(p, pooled)) return V_TAP;
        // With prepared filters the vector kernel's transposed-filter form, split over workgroups, leads on
        // small launches of 64 M multiply-adds or more with 128 or more channels per group (896 in 7 groups
        // @14x14 at batch 1: 16.9 against 21.9 us on the general kernel; 160 -> 320 @14x14: 13.8 against 16.2;
        // 512 @28x28: 40 against 47 on the matrix kernel's split tiles; 256 @56x56 stays there: 46 against 49).
        const bool prep_small_tap = p.wprep && have_ws && p.stride == 1 && p.Cg >= 128 && tap_supported(p, pooled) &&
                                    (double)p.N * p.K * p.OH * p.OW * p.Cg * 9.0 >= 64e6;
        if (!prep_small_tap && small_gen_split(p, pooled, have_ws)) return V_GEN;
        const long long quad_tiles_z = (long long)((p.OH + 1) / 2) * ((p.OW + 27) / 28) * ((p.Kg + 63) / 64) *
                                       p.N * p.G;
        if (z >= 0.0f && quad_tiles_z >= 400 && tap_supported(p, pooled)) {
            // (the 6-element granule leads again from about 92 % zeros, where the filters fill quad3x3's blocks
            // of 128; between 87 and 92 % it is ahead on some 14-wide maps - 512 channels at 88 %: 55 against 72 us -
            // and far behind on others - 384 -> 128 @40x14 at 90 %: 156 against 91 -, so the vector kernel keeps those)
            if (z >= 0.92f && !(pooled && p.W <= 14) && p.Kg % 128 == 0) return V_QUAD;
            if (z >= 0.68f) return V_TAP;
            // A denser map.  Below 68 % independent zeros fewer than one group of six in ten is empty: the
            // matrix kernels run at their dense rate, but only where their tiles fit the map.  quad3x3's
            // tiles are 28 columns wide (16 on maps up to 16 wide); measured on 40 random shapes with each
            // variant pinned: on maps wider than 16 whose width fills the 28-column tiles it leads (256 @56x56,
            // 512 @28x28 at 40-60 % zeros: 1.07-1.3x ahead of the vector kernel); on badly filling widths
            // (20: 246 us against 149 on the 16-row granule and 180 on the vector kernel; 40: 141 against 87)
            // and on maps up to 16 wide it does not: there the 16-row granule (up to 60 % zeros, fewer than 256
            // channels per group on the small maps) or the vector kernel (512 @14x14 at 50 %: 98 against 118 on
            // quad3x3 and 124 on wide3x3; quad3x3 only below 45 %: 88 against 117 at 41 %).
            const double fitw = p.W > 16 ? (double)((p.OW + 27) / 28 * 28) / p.OW : 16.0 / p.OW;
            if (p.W > 16 && fitw <= 1.15 && !(pooled && p.W <= 14)) {
                // the form without zero tests, from 256 channels per group up and where its 7-row tiles make
                // 512 or more tile-wavefronts (256 @56x56 at batch 8: 247 against 263 us; with 64 channels
                // or 128 tile-wavefronts it is 1.6-3x slower than the model's own tiles)
                const long long t7 = (long long)((p.OH + 6) / 7) * ((p.OW + 27) / 28) * ((p.Kg + 63) / 64) * p.N * p.G;
                // (and only on maps its tiles divide: 384 channels @40x56 ran 605 against 417 us with it)
                if (static_pin && (p.Cg == 256 || p.Cg == 512) && t7 >= 512 && p.OH % 7 == 0 && p.OW % 28 == 0)
                    snprintf(static_pin->geom, sizeof(static_pin->geom), "q32t7d");
                return V_QUAD;
            }
            if (p.W <= 7) return V_TAP;   // (no column halo on such maps: 128 -> 512 @20x7 at 60 % 57 against 76 on wide3x3)
            if (p.W <= 16 && p.Cg >= 256 && z < 0.45f && !pooled) return V_QUAD;
            if (z <= 0.6f && (p.W > 16 || p.Cg < 256) && p.Kg >= 128 && wide_fills) return V_WIDE;
            if (p.Cg >= 128 || fitw > 1.15) return V_TAP;
        }
        // Maps up to 14 wide with 256 or more channels per group are the deep layers, whose zero
        // ratio the paper puts above 0.7 (Fig. 2): there per-element skipping on the vector pipe
        // measures 1.0-1.15x faster than the 6-element granule from 70 % zeros up (and 1.1x slower
        // at 60 %).
        if (p.W <= 14 && p.Cg >= 256 && tap_supported(p, pooled)) return V_TAP;
        if (have_ws && !(prep_small_tap && p.Cg >= 512) && small_quad_split(p, pooled, static_pin)) return V_QUAD;
        // The same one stage earlier, 512 channels on maps up to 28 wide: 1.14x faster at 75 % zeros.
        if (p.W <= 28 && p.Cg >= 512 && !pooled && tap_supported(p, pooled)) return V_TAP;
        // Maps up to 14 wide with 128 or more filters per group and shorter channel loops: the
        // 16-row granule has no tile-geometry waste there and its time is flat in the zero ratio;
        // the vector kernel is level with it at 70 % zeros, 1.15x faster at 90 % and 2x slower on
        // a dense map, so the choice that cannot go badly wrong is made here and sconv_tune
        // takes the rest.
        if (!pooled && p.W <= 14 && p.Kg >= 128 && p.Cg < 256 && wide_fills) return V_WIDE;
        // Few tile-wavefronts (2 output rows x 28 columns x 64 filters each): the vector kernel's
        // smaller tiles spread over more of the chip and measure faster at small batch.
        const long long quad_tiles = (long long)((p.OH + 1) / 2) * ((p.OW + 27) / 28) * ((p.Kg + 63) / 64) *
                                     p.N * p.G;
        if (quad_tiles < 400 && tap_supported(p, pooled)) return V_TAP;
        // Fused pooling on maps up to 14 wide: the vector kernel's 4x14 pooled tile measures
        // 1.25-1.35x faster than the matrix kernel's at every batch size.
        if (pooled && p.W <= 14 && tap_supported(p, pooled)) return V_TAP;
        // Fused pooling on wider maps, 128 or more channels per group, a workspace for the transposed
        // filters: the vector kernel's 2x14 pooled tiles measure 1.1-1.27x faster than the matrix kernel's at
        // 70-78 % zeros (a reported ratio below 68 % keeps the matrix kernel)
        if (pooled && have_wt && p.Cg >= 128 && !(z >= 0.0f && z < 0.68f) && tap_supported(p, pooled)) return V_TAP;
        // Zero ratio unknown, 128 or more channels per group, a workspace for the transposed filters: the
        // vector kernel.  Over 80 random large launches (64-512 channels, maps 7-56 wide, 40-90 % zeros, each
        // variant pinned) always taking it here costs 9 % on average and 2.0x at worst against the best variant
        // of each shape, quad3x3 27 % and 2.1x: a sparse map punishes the matrix kernels more than a dense one
        // punishes per-element skipping, and the paper's maps are the sparse ones (Fig. 2).  A reported ratio
        // (SCONV_ZERO_RATIO) replaces this guess: 1-4 % and 1.33x.
        if (z < 0.0f && have_wt && p.Cg >= 128 && tap_supported(p, pooled)) return V_TAP;
        // Maps whose width fills quad3x3's 28-column tiles badly (20, 40: a quarter or more of the tile columns
        // empty), whatever the channel count: 96 @40x40 at 60 / 90 % zeros 127 / 50 against 193 / 100 us
        if (p.W > 16 && (p.OW + 27) / 28 * 28 * 100 > p.OW * 115 && tap_supported(p, pooled)) return V_TAP;
        return V_QUAD;
    }
    if (small_gen_split(p, pooled, have_ws)) return V_GEN;
    if (tap_supported(p, pooled)) return wide_fills ? V_WIDE : V_TAP;   // 3x3 / stride 2 / pad 1
    if (wide_supported(p, pooled)) return V_WIDE;     // 3x3 with another stride or padding
    if (gen_supported(p, pooled)) return V_GEN;       // other kernel sizes, odd channel counts
    return V_ROWS;
}

// One launch of variant v, with the cost models' decomposition or the pinned one.  No fall-through
// to other variants.  Caller holds g_lock.
static int launch_variant(Variant v, const PlanPin* pin, const Problem& p, bool pooled, const float* x,
                          const float* w, float* y, hipStream_t s)
{
    g_pin = pin;
    split_scratch_select(s);   // the workspace lent for this stream, if any
    int rc = SCONV_EUNSUPPORTED;
    switch (v) {
    case V_PW: rc = launch_pointwise(p, pooled, x, w, y, s); break;
    case V_GEN: rc = launch_gen(p, pooled, x, w, y, s); break;
    case V_WIDE: rc = launch_wide(p, pooled, x, w, y, s); break;
    case V_QUAD: rc = launch_quad(p, pooled, x, w, y, s); break;
    case V_TAP: rc = tap_supported(p, pooled) ? launch_tap(p, pooled, x, w, y, s) : SCONV_EUNSUPPORTED; break;
    case V_ROWS: rc = launch_rows(p, pooled, x, w, y, s); break;
    }
    g_pin = nullptr;
    return rc;
}

// Whether a launch on stream s would find a workspace: the one that came with the call, else a lent one.
static bool have_workspace(hipStream_t s)
{
    if (split_scratch_is_given()) {
        split_scratch_select(s);
        return split_scratch_possible(s);
    }
    return split_workspace_lent(s, false);
}

static int run(const Problem& p, bool pooled, const float* x, const float* w, float* y, hipStream_t s)
{
    // the launchers cache occupancy answers and attribute opt-ins in static variables: planning and
    // enqueueing are serialised across host threads (they take microseconds)
    std::lock_guard<std::mutex> lock(g_lock);
    if (const Tuned* t = tuned_for(p, pooled)) {
        const int rc = launch_variant(t->v, t->pinned ? &t->pin : nullptr, p, pooled, x, w, y, s);
        if (rc != SCONV_EUNSUPPORTED) return rc;
    }
    PlanPin sp;
    const float z = p.zhint;
    Variant v = choose(p, pooled, have_workspace(s), &sp, z);
    int rc = SCONV_EUNSUPPORTED;
    if (sp.geom[0]) {
        rc = launch_variant(v, &sp, p, pooled, x, w, y, s);
        if (rc != SCONV_EUNSUPPORTED) return rc;
        v = choose(p, pooled, false, nullptr, z);      // e.g. the workspace is too small for this layer
    }
    if (v == V_PW) rc = launch_variant(V_PW, nullptr, p, pooled, x, w, y, s);
    if (v == V_GEN) {
        rc = launch_variant(V_GEN, nullptr, p, pooled, x, w, y, s);
        if (rc == SCONV_EUNSUPPORTED && pw_supported(p, pooled)) rc = launch_variant(V_PW, nullptr, p, pooled, x, w, y, s);
    }
    if (v == V_WIDE) {
        rc = launch_variant(V_WIDE, nullptr, p, pooled, x, w, y, s);
        if (rc == SCONV_EUNSUPPORTED) v = quad_supported(p, pooled) ? V_QUAD : V_TAP;
    }
    if (v == V_QUAD) {
        rc = launch_variant(V_QUAD, nullptr, p, pooled, x, w, y, s);
        if (rc == SCONV_EUNSUPPORTED) v = V_TAP;
    }
    if (v == V_TAP) rc = launch_variant(V_TAP, nullptr, p, pooled, x, w, y, s);
    // no applicable tile plan: the general kernel runs
    if (rc == SCONV_EUNSUPPORTED) rc = launch_variant(V_ROWS, nullptr, p, pooled, x, w, y, s);
    return rc;
}

// Scratch the caller lends to sconv_tune for evicting the caches between timed launches.
struct Flush {
    void* dev;
    size_t bytes;
};

// Times one candidate: one untimed launch (also tells whether the candidate applies), then `reps`
// launches.  Without a flush buffer they run back to back between two events (operands stay in the
// caches); with one, the buffer is overwritten before every launch and each launch is timed on its
// own.  Returns a negative time when the candidate does not apply.
static float time_candidate(Variant v, const PlanPin* pin, const Problem& p, bool pooled, const float* x,
                            const float* w, float* y, hipStream_t s, hipEvent_t e0, hipEvent_t e1, int reps,
                            const Flush& flush, int* err)
{
    int rc = launch_variant(v, pin, p, pooled, x, w, y, s);
    if (rc == SCONV_EUNSUPPORTED) return -1.0f;
    if (rc != SCONV_OK) { *err = rc; return -1.0f; }
    float total = 0.0f;
    const int rounds = flush.dev ? reps : 1, per_round = flush.dev ? 1 : reps;
    for (int r = 0; r < rounds; ++r) {
        if (flush.dev && hipMemsetAsync(flush.dev, r & 1, flush.bytes, s) != hipSuccess) { *err = SCONV_ELAUNCH; return -1.0f; }
        if (hipEventRecord(e0, s) != hipSuccess) { *err = SCONV_ELAUNCH; return -1.0f; }
        for (int i = 0; i < per_round; ++i) {
            rc = launch_variant(v, pin, p, pooled, x, w, y, s);
            if (rc != SCONV_OK) { *err = rc; return -1.0f; }
        }
        float ms = 0.0f;
        if (hipEventRecord(e1, s) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
            hipEventElapsedTime(&ms, e0, e1) != hipSuccess) {
            *err = SCONV_ELAUNCH;
            return -1.0f;
        }
        total += ms;
    }
    return total / reps;
}

static int tune(const Problem& p, bool pooled, const float* x, const float* w, float* y, hipStream_t s,
                const Flush& flush, float* best_ms)
{
    std::lock_guard<std::mutex> lock(g_lock);
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return SCONV_ELAUNCH;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return SCONV_ELAUNCH; }
    struct Family {
        Variant v;
        bool ok;
        const char* const* geoms;
        int nwv_lo, nwv_hi;
        int nss_hi;        // largest channel split across workgroups to try (1: the variant has none)
    };
    const Family fams[] = {
        {V_PW, pw_supported(p, pooled), pw_geoms(), 8, 16, 1},
        {V_TAP, tap_supported(p, pooled), tap_geoms(), 8, 16, 16},
        {V_QUAD, quad_supported(p, pooled), quad_geoms(), 8, 16, 16},
        {V_WIDE, wide_supported(p, pooled), wide_geoms(), 4, 8, 1},
        {V_GEN, gen_supported(p, pooled), gen_geoms(), 4, 8, 16},
    };
    // every candidate that applies, with a first quick timing
    struct Cand {
        Variant v;
        PlanPin pin;
        bool pinned;
        float ms;
    };
    std::vector<Cand> cands;
    int err = SCONV_OK;
    // First pass, cheap: one untimed launch (does the candidate apply?), one timed launch with the operands
    // still in the caches; only a candidate within a quarter of the fastest so far is timed twice more.
    float fastest = -1.0f, last_t = -1.0f;
    const Flush no_flush_first = {nullptr, 0};
    auto try_one = [&](Variant v, const PlanPin* pin) {
        float t = time_candidate(v, pin, p, pooled, x, w, y, s, e0, e1, 1, no_flush_first, &err);
        last_t = t;
        if (t < 0.0f) return false;
        if (fastest < 0.0f || t <= 1.25f * fastest) {
            const float t2 = time_candidate(v, pin, p, pooled, x, w, y, s, e0, e1, 2, no_flush_first, &err);
            if (t2 >= 0.0f && t2 < t) t = t2;
        }
        if (fastest < 0.0f || t < fastest) fastest = t;
        Cand c;
        c.v = v;
        c.pinned = pin != nullptr;
        if (pin) c.pin = *pin; else memset(&c.pin, 0, sizeof(c.pin));
        c.ms = t;
        cands.push_back(c);
        return true;
    };
    // the static rules' own choice comes first: it stays unless something measures clearly faster
    PlanPin sp;
    Variant v_static = choose(p, pooled, have_workspace(s), &sp, p.zhint);
    bool have_static = try_one(v_static, sp.geom[0] ? &sp : nullptr);
    if (!have_static && sp.geom[0]) {
        v_static = choose(p, pooled);
        have_static = try_one(v_static, nullptr);
    }
    // A fused call keeps the convolution tensor on chip (Section 6.4): plans that split its channels over
    // workgroups - plain tiles whose partial sums pass through the workspace to a kernel that pools - are
    // candidates only for launches too small to fill the chip, as in the static rules.
    const long long fused_tile_wgs = (long long)((p.OH + 4) / 5) * ((p.OW + 6) / 7) * ((p.Kg + 63) / 64) * p.N * p.G;
    const bool fused_split_ok = !pooled || fused_tile_wgs < 128;
    for (const Family& f : fams) {
        if (!f.ok || err != SCONV_OK) continue;
        for (const char* const* g = f.geoms; *g && err == SCONV_OK; ++g) {
            // the model's own split of this geometry first: a geometry that does not apply is
            // dropped after one call
            PlanPin pin;
            memset(&pin, 0, sizeof(pin));
            snprintf(pin.geom, sizeof(pin.geom), "%s", *g);
            // (a plain geometry serves a fused call only with its channels split: start there)
            const bool unsplit_ok = try_one(f.v, &pin);
            // (that plan comes again below under its explicit decomposition, which is what the record names)
            if (unsplit_ok) cands.pop_back();
            if (!unsplit_ok && !(pooled && f.nss_hi > 1 && fused_split_ok)) continue;
            // a geometry whose own split is twice as slow as the fastest plan so far is not worth its
            // other decompositions
            if (unsplit_ok && fastest > 0.0f && last_t > 2.0f * fastest) continue;
            for (int nss = unsplit_ok ? 1 : 2; nss <= (fused_split_ok ? f.nss_hi : 1) && err == SCONV_OK; nss *= 2) {
                bool any = false;   // a split the launch is too large for applies with no nwv, ncs
                for (int nwv = f.nwv_lo; nwv <= f.nwv_hi && err == SCONV_OK; nwv *= 2) {
                    for (int ncs = 1; ncs <= nwv && err == SCONV_OK; ncs *= 2) {
                        pin.nwv = nwv;
                        pin.ncs = ncs;
                        pin.nss = nss;
                        any |= try_one(f.v, &pin);
                    }
                }
                if (!any && !(pooled && nss == 1)) break;   // (a plain geometry serves a fused call only when split)
            }
        }
    }
    if (err == SCONV_OK && cands.empty()) try_one(V_ROWS, nullptr);   // only the general kernel covers it
    // The static choice and the four fastest again, long enough for the timing to be trusted (about
    // a millisecond each).  The static choice is timed first and a candidate replaces it only when
    // it measures 3 % faster: launches of 10-20 us differ by that much from one timing to the next
    Tuned best;
    best.ms = -1.0f;
    std::sort(cands.begin() + (have_static ? 1 : 0), cands.end(),
              [](const Cand& a, const Cand& b) { return a.ms < b.ms; });
    // With a flush buffer every plan is timed both ways - single launches on evicted caches, and
    // back to back - and must win both: the two rank kernels up to 10 % apart (the 1x1 layers:
    // a plan that leads on isolated cold launches trails when launches follow each other).
    float bar = -1.0f, bar_warm = -1.0f;   // times to beat
    const Flush no_flush = {nullptr, 0};
    for (size_t i = 0; i < cands.size() && i < (have_static ? 5u : 4u) && err == SCONV_OK; ++i) {
        const Cand& c = cands[i];
        int reps = (int)(1.0f / (c.ms > 1e-3f ? c.ms : 1e-3f));
        reps = reps < 5 ? 5 : (reps > 100 ? 100 : reps);
        const float t = time_candidate(c.v, c.pinned ? &c.pin : nullptr, p, pooled, x, w, y, s, e0, e1,
                                       flush.dev && reps > 30 ? 30 : reps, flush, &err);
        if (t < 0.0f || (bar >= 0.0f && t >= bar)) continue;
        float t_warm = t;
        if (flush.dev) {
            t_warm = time_candidate(c.v, c.pinned ? &c.pin : nullptr, p, pooled, x, w, y, s, e0, e1, reps, no_flush,
                                    &err);
            if (t_warm < 0.0f || (bar_warm >= 0.0f && t_warm >= bar_warm)) continue;
        }
        // (and by at least 1.5 us: single launches of 10-15 us time that far apart)
        const bool is_static = have_static && i == 0;
        bar = is_static ? std::min(0.97f * t, t - 0.0015f) : t;
        bar_warm = is_static ? std::min(0.97f * t_warm, t_warm - 0.0015f) : t_warm;
        best.v = c.v;
        best.ms = t;
        best.pin = c.pin;
        best.pinned = c.pinned;
        if (have_static && i == 0) {
            // (the vector kernel's static plan by name, so that records show what was kept)
            char detail[32];
            split_scratch_select(s);
            if (c.v == V_TAP && !c.pinned && describe_tap(p, pooled, s, detail, sizeof(detail)))
                snprintf(best.name, sizeof(best.name), "%s/model:%s/kept", variant_name(c.v), detail);
            else
                snprintf(best.name, sizeof(best.name), "%s/model/kept", variant_name(c.v));
        }
        else if (c.pinned && c.pin.nss > 1)
            snprintf(best.name, sizeof(best.name), "%s/%s/%dx%dx%d", variant_name(c.v), c.pin.geom, c.pin.nwv,
                     c.pin.ncs, c.pin.nss);
        else if (c.pinned)
            snprintf(best.name, sizeof(best.name), "%s/%s/%dx%d", variant_name(c.v), c.pin.geom[0] ? c.pin.geom : "-",
                     c.pin.nwv, c.pin.ncs);
        else
            snprintf(best.name, sizeof(best.name), "%s/model/kept", variant_name(c.v));
    }
    if (err == SCONV_OK && best.ms >= 0.0f) {
        // leave y holding the result of the plan that later calls will launch
        const int rc = launch_variant(best.v, best.pinned ? &best.pin : nullptr, p, pooled, x, w, y, s);
        if (rc != SCONV_OK) err = rc;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (err != SCONV_OK) return err;
    if (best.ms < 0.0f) return SCONV_EUNSUPPORTED;
    g_tuned[tune_key(p, pooled)] = best;
    if (best_ms) *best_ms = best.ms;
    return SCONV_OK;
}

}  // namespace sconv

using namespace sconv;

extern "C" int sconv_output_dims(const sconv_desc_t* desc, int32_t* OH, int32_t* OW, int32_t* PH,
                                 int32_t* PW)
{
    if (!desc || !OH || !OW) return SCONV_EINVAL;
    bool pooled = desc->pool_h > 0 || desc->pool_w > 0 || desc->pool_stride > 0;
    Problem p;
    int rc = fill_problem(desc, pooled, &p);
    if (rc) return rc;
    *OH = p.OH;
    *OW = p.OW;
    if (PH) *PH = p.PH;
    if (PW) *PW = p.PW;
    return SCONV_OK;
}

extern "C" int sconv_encode_sizes(const sconv_desc_t* desc, int fmt, int64_t* rows,
                                  int64_t* slots_per_row)
{
    if (!rows || !slots_per_row) return SCONV_EINVAL;
    if (fmt != SCONV_FMT_ECR && fmt != SCONV_FMT_PECR) return SCONV_EINVAL;
    Problem p;
    int rc = fill_problem(desc, fmt == SCONV_FMT_PECR, &p);
    if (rc) return rc;
    int64_t r = (int64_t)p.N * p.G;
    if (fmt == SCONV_FMT_ECR)
        r *= (int64_t)p.OH * p.OW;
    else
        r *= (int64_t)p.PH * p.PW * p.ph * p.pw;
    *rows = r;
    *slots_per_row = p.L;
    return SCONV_OK;
}

extern "C" int sconv_encode(const sconv_desc_t* desc, int fmt, const float* x_dev,
                            float* values_dev, int32_t* index_dev, int32_t* count_dev,
                            void* hip_stream)
{
    if (!x_dev || !values_dev || !index_dev || !count_dev) return SCONV_EINVAL;
    int64_t rows, L;
    int rc = sconv_encode_sizes(desc, fmt, &rows, &L);
    if (rc) return rc;
    if (rows * L >= (int64_t(1) << 40) || rows >= (int64_t(1) << 31)) return SCONV_EUNSUPPORTED;
    Problem p;
    rc = fill_problem(desc, fmt == SCONV_FMT_PECR, &p);
    if (rc) return rc;
    return launch_encode(p, fmt, x_dev, values_dev, index_dev, count_dev, (hipStream_t)hip_stream);
}

extern "C" int sconv_forward(const sconv_desc_t* desc, const float* x_dev, const float* w_dev,
                             float* y_dev, void* hip_stream)
{
    if (!x_dev || !w_dev || !y_dev) return SCONV_EINVAL;
    Problem p;
    int rc = fill_problem(desc, false, &p);
    if (rc) return rc;
    return run(p, false, x_dev, w_dev, y_dev, (hipStream_t)hip_stream);
}

extern "C" int sconv_pool_forward(const sconv_desc_t* desc, const float* x_dev, const float* w_dev,
                                  float* y_dev, void* hip_stream)
{
    if (!x_dev || !w_dev || !y_dev) return SCONV_EINVAL;
    Problem p;
    int rc = fill_problem(desc, true, &p);
    if (rc) return rc;
    if ((int64_t)p.ph * p.pw > 64) return SCONV_EUNSUPPORTED;
    return run(p, true, x_dev, w_dev, y_dev, (hipStream_t)hip_stream);
}

// Runs one forward call with the workspace the caller passed (null: none) in place of a lent one.
static int run_with(const Problem& p, bool pooled, const float* x, const float* w, float* y, void* ws,
                    size_t ws_bytes, hipStream_t s)
{
    split_scratch_given(ws, ws_bytes, true);
    const int rc = run(p, pooled, x, w, y, s);
    split_scratch_given(nullptr, 0, false);
    return rc;
}

extern "C" int sconv_forward_ws(const sconv_desc_t* desc, const float* x_dev, const float* w_dev, float* y_dev,
                                void* ws_dev, size_t ws_bytes, void* hip_stream)
{
    if (!x_dev || !w_dev || !y_dev) return SCONV_EINVAL;
    if ((ws_dev == nullptr) != (ws_bytes == 0) || reinterpret_cast<uintptr_t>(ws_dev) % 16) return SCONV_EINVAL;
    Problem p;
    int rc = fill_problem(desc, false, &p);
    if (rc) return rc;
    return run_with(p, false, x_dev, w_dev, y_dev, ws_dev, ws_bytes, (hipStream_t)hip_stream);
}

extern "C" int sconv_pool_forward_ws(const sconv_desc_t* desc, const float* x_dev, const float* w_dev,
                                     float* y_dev, void* ws_dev, size_t ws_bytes, void* hip_stream)
{
    if (!x_dev || !w_dev || !y_dev) return SCONV_EINVAL;
    if ((ws_dev == nullptr) != (ws_bytes == 0) || reinterpret_cast<uintptr_t>(ws_dev) % 16) return SCONV_EINVAL;
    Problem p;
    int rc = fill_problem(desc, true, &p);
    if (rc) return rc;
    if ((int64_t)p.ph * p.pw > 64) return SCONV_EUNSUPPORTED;
    return run_with(p, true, x_dev, w_dev, y_dev, ws_dev, ws_bytes, (hipStream_t)hip_stream);
}

extern "C" int sconv_forward_bias(const sconv_desc_t* desc, const float* x_dev, const float* w_dev,
                                  const float* bias_dev, float* y_dev, void* hip_stream)
{
    if (!x_dev || !w_dev || !bias_dev || !y_dev) return SCONV_EINVAL;
    Problem p;
    int rc = fill_problem(desc, false, &p);
    if (rc) return rc;
    p.bias = bias_dev;
    return run(p, false, x_dev, w_dev, y_dev, (hipStream_t)hip_stream);
}

extern "C" int sconv_pool_forward_bias(const sconv_desc_t* desc, const float* x_dev, const float* w_dev,
                                       const float* bias_dev, float* y_dev, void* hip_stream)
{
    if (!x_dev || !w_dev || !bias_dev || !y_dev) return SCONV_EINVAL;
    Problem p;
    int rc = fill_problem(desc, true, &p);
    if (rc) return rc;
    if ((int64_t)p.ph * p.pw > 64) return SCONV_EUNSUPPORTED;
    p.bias = bias_dev;
    return run(p, true, x_dev, w_dev, y_dev, (hipStream_t)hip_stream);
}

extern "C" int sconv_filter_prep_size(const sconv_desc_t* desc, size_t* bytes)
{
    if (!bytes) return SCONV_EINVAL;
    Problem p;
    bool pooled = desc && (desc->pool_h > 0 || desc->pool_w > 0 || desc->pool_stride > 0);
    int rc = fill_problem(desc, pooled, &p);
    if (rc) return rc;
    // only the vector kernel's transposed-filter form reads the layout
    *bytes = tap_supported(p, pooled) && p.stride == 1 ? filter_prep_bytes(p) : 0;
    return SCONV_OK;
}

extern "C" int sconv_filter_prep(const sconv_desc_t* desc, const float* w_dev, void* wprep_dev, size_t wprep_bytes,
                                 void* hip_stream)
{
    if (!w_dev || !wprep_dev) return SCONV_EINVAL;
    if (reinterpret_cast<uintptr_t>(wprep_dev) % 256) return SCONV_EINVAL;
    size_t need = 0;
    int rc = sconv_filter_prep_size(desc, &need);
    if (rc) return rc;
    if (need == 0) return SCONV_EUNSUPPORTED;
    if (wprep_bytes < need) return SCONV_EINVAL;
    Problem p;
    bool pooled = desc->pool_h > 0 || desc->pool_w > 0 || desc->pool_stride > 0;
    rc = fill_problem(desc, pooled, &p);
    if (rc) return rc;
    return launch_filter_prep(p, w_dev, static_cast<float*>(wprep_dev), (hipStream_t)hip_stream);
}

// Checks the optional operands of the ..._prep calls and attaches them to the problem.
static int attach_prep(Problem* p, bool pooled, const void* wprep_dev, size_t wprep_bytes, const float* bias_dev,
                       void* ws_dev, size_t ws_bytes)
{
    if ((ws_dev == nullptr) != (ws_bytes == 0) || reinterpret_cast<uintptr_t>(ws_dev) % 16) return SCONV_EINVAL;
    if ((wprep_dev == nullptr) != (wprep_bytes == 0) || reinterpret_cast<uintptr_t>(wprep_dev) % 256) return SCONV_EINVAL;
    p->bias = bias_dev;
    if (wprep_dev) {
        // a descriptor no kernel reads the layout for ignores it; one that does needs all of it
        if (tap_supported(*p, pooled) && p->stride == 1) {
            if (wprep_bytes < filter_prep_bytes(*p)) return SCONV_EINVAL;
            p->wprep = static_cast<const float*>(wprep_dev);
        }
    }
    return SCONV_OK;
}

extern "C" int sconv_forward_prep(const sconv_desc_t* desc, const float* x_dev, const float* w_dev,
                                  const void* wprep_dev, size_t wprep_bytes, const float* bias_dev, float* y_dev,
                                  void* ws_dev, size_t ws_bytes, void* hip_stream)
{
    if (!x_dev || !w_dev || !y_dev) return SCONV_EINVAL;
    Problem p;
    int rc = fill_problem(desc, false, &p);
    if (rc) return rc;
    rc = attach_prep(&p, false, wprep_dev, wprep_bytes, bias_dev, ws_dev, ws_bytes);
    if (rc) return rc;
    return run_with(p, false, x_dev, w_dev, y_dev, ws_dev, ws_bytes, (hipStream_t)hip_stream);
}

extern "C" int sconv_pool_forward_prep(const sconv_desc_t* desc, const float* x_dev, const float* w_dev,
                                       const void* wprep_dev, size_t wprep_bytes, const float* bias_dev,
                                       float* y_dev, void* ws_dev, size_t ws_bytes, void* hip_stream)
{
    if (!x_dev || !w_dev || !y_dev) return SCONV_EINVAL;
    Problem p;
    int rc = fill_problem(desc, true, &p);
    if (rc) return rc;
    if ((int64_t)p.ph * p.pw > 64) return SCONV_EUNSUPPORTED;
    rc = attach_prep(&p, true, wprep_dev, wprep_bytes, bias_dev, ws_dev, ws_bytes);
    if (rc) return rc;
    return run_with(p, true, x_dev, w_dev, y_dev, ws_dev, ws_bytes, (hipStream_t)hip_stream);
}

extern "C" int sconv_pair_forward(const sconv_desc_t* first, const sconv_desc_t* second, const float* x_dev,
                                  const float* w1_dev, const float* bias1_dev, const float* w2_dev,
                                  const float* bias2_dev, float* mid_dev, float* y_dev, void* hip_stream)
{
    if (!first || !second || !x_dev || !w1_dev || !w2_dev || !y_dev) return SCONV_EINVAL;
    const bool pooled1 = first->pool_h > 0 || first->pool_w > 0 || first->pool_stride > 0;
    const bool pooled2 = second->pool_h > 0 || second->pool_w > 0 || second->pool_stride > 0;
    Problem p1, p2;
    int rc = fill_problem(first, pooled1, &p1);
    if (rc) return rc;
    rc = fill_problem(second, pooled2, &p2);
    if (rc) return rc;
    if ((pooled1 && (int64_t)p1.ph * p1.pw > 64) || (pooled2 && (int64_t)p2.ph * p2.pw > 64)) return SCONV_EUNSUPPORTED;
    p1.bias = bias1_dev;
    p2.bias = bias2_dev;
    std::lock_guard<std::mutex> lock(g_lock);
    return launch_pair(p1, pooled1, p2, pooled2, x_dev, w1_dev, w2_dev, mid_dev, y_dev, (hipStream_t)hip_stream);
}

extern "C" int sconv_forward_static(const sconv_desc_t* desc, const float* x_dev, const float* w_dev,
                                    float* y_dev, void* hip_stream)
{
    if (!x_dev || !w_dev || !y_dev) return SCONV_EINVAL;
    Problem p;
    int rc = fill_problem(desc, false, &p);
    if (rc) return rc;
    // the smallest split keeps two slices of partial sums
    if (2 * (size_t)p.N * p.K * p.OH * p.OW * sizeof(float) > kStaticScratchBytes) return SCONV_ETOOLARGE;
    float* ws = nullptr;
    size_t ws_bytes = 0;
    {
        std::lock_guard<std::mutex> lock(g_lock);
        rc = split_static_scratch(&ws, &ws_bytes);
    }
    if (rc) return rc;
    return run_with(p, false, x_dev, w_dev, y_dev, ws, ws_bytes, (hipStream_t)hip_stream);
}

extern "C" int sconv_density(const sconv_desc_t* desc, const float* x_dev, unsigned long long* counts_dev,
                             void* hip_stream)
{
    if (!x_dev || !counts_dev) return SCONV_EINVAL;
    if (reinterpret_cast<uintptr_t>(counts_dev) % 8) return SCONV_EINVAL;
    Problem p;
    int rc = fill_problem(desc, false, &p);
    if (rc) return rc;
    return launch_density_probe(p, x_dev, counts_dev, (hipStream_t)hip_stream);
}

extern "C" int sconv_env_refresh(void)
{
    std::lock_guard<std::mutex> lock(g_lock);
    std::lock_guard<std::mutex> elock(g_env_lock);
    env_load_locked();
    return SCONV_OK;
}

extern "C" int sconv_maxpool(const sconv_desc_t* desc, const float* conv_dev, float* y_dev,
                             void* hip_stream)
{
    if (!conv_dev || !y_dev) return SCONV_EINVAL;
    Problem p;
    int rc = fill_problem(desc, true, &p);
    if (rc) return rc;
    return launch_maxpool(p, conv_dev, y_dev, (hipStream_t)hip_stream);
}

// SCONV_PREPARED_FILTERS in a descriptor handed to the two naming calls: plan as for a call that brings
// prepared filters.  Nothing is launched from such a Problem; the pointer only has to be non-null.
static void mark_prepared_for_naming(const sconv_desc_t* desc, bool pooled, Problem* p)
{
    static const float placeholder = 0.0f;
    if ((desc->flags & SCONV_PREPARED_FILTERS) && tap_supported(*p, pooled) && p->stride == 1) p->wprep = &placeholder;
}

extern "C" const char* sconv_variant_name(const sconv_desc_t* desc, int pooled)
{
    Problem p;
    if (fill_problem(desc, pooled != 0, &p)) return NULL;
    mark_prepared_for_naming(desc, pooled != 0, &p);
    std::lock_guard<std::mutex> lock(g_lock);
    if (const Tuned* t = tuned_for(p, pooled != 0)) return variant_name(t->v);
    return variant_name(choose(p, pooled != 0, split_workspace_lent(nullptr, true), nullptr, p.zhint));
}

extern "C" int sconv_tune(const sconv_desc_t* desc, int pooled, const float* x_dev, const float* w_dev,
                          float* y_dev, void* flush_dev, size_t flush_bytes, void* hip_stream, float* best_ms)
{
    if (!x_dev || !w_dev || !y_dev) return SCONV_EINVAL;
    if ((flush_dev == nullptr) != (flush_bytes == 0)) return SCONV_EINVAL;
    Problem p;
    int rc = fill_problem(desc, pooled != 0, &p);
    if (rc) return rc;
    if (pooled && (int64_t)p.ph * p.pw > 64) return SCONV_EUNSUPPORTED;
    return tune(p, pooled != 0, x_dev, w_dev, y_dev, (hipStream_t)hip_stream, Flush{flush_dev, flush_bytes}, best_ms);
}

extern "C" int sconv_tune_prep(const sconv_desc_t* desc, int pooled, const float* x_dev, const float* w_dev,
                               const void* wprep_dev, size_t wprep_bytes, float* y_dev, void* ws_dev, size_t ws_bytes,
                               void* flush_dev, size_t flush_bytes, void* hip_stream, float* best_ms)
{
    if (!x_dev || !w_dev || !y_dev) return SCONV_EINVAL;
    if ((flush_dev == nullptr) != (flush_bytes == 0)) return SCONV_EINVAL;
    Problem p;
    int rc = fill_problem(desc, pooled != 0, &p);
    if (rc) return rc;
    if (pooled && (int64_t)p.ph * p.pw > 64) return SCONV_EUNSUPPORTED;
    rc = attach_prep(&p, pooled != 0, wprep_dev, wprep_bytes, nullptr, ws_dev, ws_bytes);
    if (rc) return rc;
    split_scratch_given(ws_dev, ws_bytes, true);
    rc = tune(p, pooled != 0, x_dev, w_dev, y_dev, (hipStream_t)hip_stream, Flush{flush_dev, flush_bytes}, best_ms);
    split_scratch_given(nullptr, 0, false);
    return rc;
}

extern "C" int sconv_workspace_size(const sconv_desc_t* desc, int pooled, size_t* bytes)
{
    if (!bytes) return SCONV_EINVAL;
    Problem p;
    int rc = fill_problem(desc, pooled != 0, &p);
    if (rc) return rc;
    *bytes = 0;
    // only the kernels that can split a launch use it, and only for launches of a few hundred
    // workgroups: up to 16 slices of the convolution tensor, never more than the cap
    if (!tap_supported(p, pooled != 0) && !gen_supported(p, pooled != 0) && !quad_supported(p, pooled != 0))
        return SCONV_OK;
    const size_t slice = (size_t)p.N * p.K * p.OH * p.OW * sizeof(float);
    size_t need = 16 * slice;
    if (need > kSplitWorkspaceCap) need = kSplitWorkspaceCap;
    // plus the transposed copy of the filters the vector kernel's large launches read (filters per group
    // rounded up to whole blocks of 128)
    if (tap_supported(p, pooled != 0))
        need += (size_t)p.G * ((p.Kg + 127) / 128 * 128) * p.L * sizeof(float) + 256;
    *bytes = (need + 255) / 256 * 256;
    return SCONV_OK;
}

extern "C" int sconv_set_workspace(void* ws_dev, size_t bytes, void* hip_stream)
{
    if ((ws_dev == nullptr) != (bytes == 0)) return SCONV_EINVAL;
    if (reinterpret_cast<uintptr_t>(ws_dev) % 16) return SCONV_EINVAL;
    std::lock_guard<std::mutex> lock(g_lock);
    return split_workspace_set(ws_dev, bytes, (hipStream_t)hip_stream);
}

extern "C" int sconv_clear_workspaces(void)
{
    std::lock_guard<std::mutex> lock(g_lock);
    split_workspace_clear();
    return SCONV_OK;
}

extern "C" int sconv_tune_reset(void)
{
    std::lock_guard<std::mutex> lock(g_lock);
    g_tuned.clear();
    return SCONV_OK;
}

// Text form of the plan table, one line per entry:
//   "sconv-plan 1 <17 key integers> <variant> <pinned> <geometry or -> <nwv> <ncs> <nss> <ms> <name>"
static const char* const* geoms_of(Variant v)
{
    switch (v) {
    case V_PW: return pw_geoms();
    case V_TAP: return tap_geoms();
    case V_QUAD: return quad_geoms();
    case V_WIDE: return wide_geoms();
    case V_GEN: return gen_geoms();
    default: return nullptr;
    }
}

extern "C" int sconv_tune_export(char* out, size_t out_size, size_t* needed)
{
    std::lock_guard<std::mutex> lock(g_lock);
    std::string text;
    char line[512];
    for (const auto& kv : g_tuned) {
        int n = snprintf(line, sizeof(line), "sconv-plan 1");
        for (int32_t v : kv.first) n += snprintf(line + n, sizeof(line) - n, " %d", v);
        const Tuned& t = kv.second;
        snprintf(line + n, sizeof(line) - n, " %d %d %s %d %d %d %.6g %s\n", (int)t.v, t.pinned ? 1 : 0,
                 t.pin.geom[0] ? t.pin.geom : "-", t.pin.nwv, t.pin.ncs, t.pin.nss, (double)t.ms, t.name);
        text += line;
    }
    if (needed) *needed = text.size() + 1;
    if (!out || out_size < text.size() + 1) return (out || out_size) ? SCONV_EINVAL : SCONV_OK;
    memcpy(out, text.c_str(), text.size() + 1);
    return SCONV_OK;
}

extern "C" int sconv_tune_import(const char* text)
{
    if (!text) return SCONV_EINVAL;
    std::map<TuneKey, Tuned> parsed;
    const char* p = text;
    while (*p) {
        const char* eol = strchr(p, '\n');
        const size_t len = eol ? (size_t)(eol - p) : strlen(p);
        std::string line(p, len);
        p += len + (eol ? 1 : 0);
        if (line.find_first_not_of(" \t\r") == std::string::npos) continue;
        int pos = 0, version = 0;
        if (sscanf(line.c_str(), " sconv-plan %d%n", &version, &pos) != 1 || version != 1) return SCONV_EINVAL;
        TuneKey key;
        for (int32_t& v : key) {
            int used = 0;
            if (sscanf(line.c_str() + pos, " %d%n", &v, &used) != 1) return SCONV_EINVAL;
            pos += used;
        }
        Tuned t;
        memset(&t, 0, sizeof(t));
        int v = 0, pinned = 0, used = 0;
        char geom[32], name[64];
        double ms = 0.0;
        if (sscanf(line.c_str() + pos, " %d %d %31s %d %d %d %lf %63s%n", &v, &pinned, geom, &t.pin.nwv, &t.pin.ncs,
                   &t.pin.nss, &ms, name, &used) != 8)
            return SCONV_EINVAL;
        if (v < (int)V_ROWS || v > (int)V_GEN || strlen(geom) >= sizeof(t.pin.geom) || strlen(name) >= sizeof(t.name))
            return SCONV_EINVAL;
        // only decompositions the launchers know: a geometry of that variant, powers of two within their ranges
        auto pow2_upto = [](int x, int hi) { return x == 0 || (x > 0 && x <= hi && (x & (x - 1)) == 0); };
        if (!pow2_upto(t.pin.nwv, 16) || !pow2_upto(t.pin.ncs, 16) || !pow2_upto(t.pin.nss, 16)) return SCONV_EINVAL;
        t.v = (Variant)v;
        t.pinned = pinned != 0;
        if (strcmp(geom, "-") != 0) {
            bool known = false;
            if (const char* const* g = geoms_of(t.v))
                for (; *g; ++g) known |= strcmp(*g, geom) == 0;
            if (!known) return SCONV_EINVAL;
            snprintf(t.pin.geom, sizeof(t.pin.geom), "%s", geom);
        }
        t.ms = (float)ms;
        snprintf(t.name, sizeof(t.name), "%s", name);
        parsed[key] = t;
    }
    std::lock_guard<std::mutex> lock(g_lock);
    for (const auto& kv : parsed) g_tuned[kv.first] = kv.second;
    return SCONV_OK;
}

extern "C" int sconv_plan_name(const sconv_desc_t* desc, int pooled, char* out, int out_size)
{
    if (!out || out_size <= 0) return SCONV_EINVAL;
    Problem p;
    int rc = fill_problem(desc, pooled != 0, &p);
    if (rc) return rc;
    mark_prepared_for_naming(desc, pooled != 0, &p);
    std::lock_guard<std::mutex> lock(g_lock);
    if (const Tuned* t = tuned_for(p, pooled != 0)) {
        snprintf(out, (size_t)out_size, "%s", t->name);
        return SCONV_OK;
    }
    const Variant v = choose(p, pooled != 0, split_workspace_lent(nullptr, true), nullptr, p.zhint);
    char detail[40];
    split_scratch_select(nullptr);   // the default stream's workspace, as for a launch there
    if (v == V_TAP && describe_tap(p, pooled != 0, nullptr, detail, sizeof(detail)))
        snprintf(out, (size_t)out_size, "%s/model:%s", variant_name(v), detail);
    else
        snprintf(out, (size_t)out_size, "%s/model", variant_name(v));
    return SCONV_OK;
}

extern "C" const char* sconv_strerror(int code)
{
    switch (code) {
    case SCONV_OK: return "success";
    case SCONV_EINVAL: return "invalid argument";
    case SCONV_EUNSUPPORTED: return "shape exceeds a kernel limit";
    case SCONV_ELAUNCH: return "HIP launch failed";
    case SCONV_ETOOLARGE: return "output tensor too large for the library's static scratch (sconv_forward_static)";
    default: return "unknown sconv error code";
    }
}

// Host side of libsconv: argument checks, size helpers, variant choice.  No device code here.
#include <stdlib.h>
#include <string.h>

#include <mutex>

#include "sconv_internal.h"

namespace sconv {

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
    if (d->flags & ~SCONV_RELU) return SCONV_EINVAL;
    if (d->H + 2 * (int64_t)d->pad < d->R || d->W + 2 * (int64_t)d->pad < d->S) return SCONV_EINVAL;

    Problem p;
    memset(&p, 0, sizeof(p));
    p.N = d->N; p.C = d->C; p.H = d->H; p.W = d->W;
    p.K = d->K; p.R = d->R; p.S = d->S;
    p.stride = d->stride; p.pad = d->pad; p.G = d->groups;
    p.Cg = d->C / d->groups;
    p.Kg = d->K / d->groups;
    p.OH = (d->H + 2 * d->pad - d->R) / d->stride + 1;
    p.OW = (d->W + 2 * d->pad - d->S) / d->stride + 1;
    p.relu = (d->flags & SCONV_RELU) ? 1 : 0;
    if (pooled) {
        if (d->pool_h <= 0 || d->pool_w <= 0 || d->pool_stride <= 0) return SCONV_EINVAL;
        if (d->pool_h > p.OH || d->pool_w > p.OW) return SCONV_EINVAL;
        p.ph = d->pool_h; p.pw = d->pool_w; p.ps = d->pool_stride;
        p.PH = (p.OH - p.ph) / p.ps + 1;
        p.PW = (p.OW - p.pw) / p.ps + 1;
        p.relu = 1;
    }
    int64_t L = (int64_t)p.Cg * p.R * p.S;
    if (L >= (int64_t(1) << 24)) return SCONV_EUNSUPPORTED;
    p.L = (int)L;
    if (!mul_fits_31(p.N, p.C, p.H, p.W) || !mul_fits_31(p.K, p.Cg, p.R, p.S) ||
        !mul_fits_31(p.N, p.K, p.OH, p.OW))
        return SCONV_EUNSUPPORTED;
    *out = p;
    return SCONV_OK;
}

enum Variant { V_ROWS, V_TAP, V_QUAD, V_PW, V_WIDE, V_GEN };

static Variant choose(const Problem& p, bool pooled)
{
    const char* pin = getenv("SCONV_VARIANT");
    if (pin && !strcmp(pin, "rows")) return V_ROWS;
    if (pin && !strcmp(pin, "tap")) return tap_supported(p, pooled) ? V_TAP : V_ROWS;
    if (pin && !strcmp(pin, "wide")) return wide_supported(p, pooled) ? V_WIDE : V_ROWS;
    if (pin && !strcmp(pin, "quad")) return quad_supported(p, pooled) ? V_QUAD : V_ROWS;
    if (pin && !strcmp(pin, "gen")) return gen_supported(p, pooled) ? V_GEN : V_ROWS;
    if (pw_supported(p, pooled)) return V_PW;
    // The 16-row granule needs many tile-wavefronts (64 window rows x 64 filters each) to fill the
    // chip: it splits the channels of a tile four ways at most.
    const long long rows = pooled ? (long long)p.N * p.PH * p.PW * 4 : (long long)p.N * p.OH * p.OW;
    const bool wide_fills = wide_supported(p, pooled) &&
                            ((rows + 63) / 64) * ((p.Kg + 63) / 64) * p.G >= 128;
    if (quad_supported(p, pooled)) {
        // Maps of 7x7 and below are one whole-map tile of the vector kernel (no halo, no ragged
        // tiles); it measures 1.4-1.8x faster there than either matrix kernel.
        if (p.H <= 7 && p.W <= 7 && tap_supported(p, pooled)) return V_TAP;
        // Small maps with many filters: the 16-row granule has no tile-geometry waste there and
        // measures faster; everywhere else the 4-row granule skips more and wins.
        if (!pooled && p.W <= 14 && p.Kg >= 128 && wide_fills) return V_WIDE;
        // Few tile-wavefronts (2 output rows x 28 columns x 64 filters each): the vector kernel's
        // smaller tiles spread over more of the chip and measure faster at small batch.
        const long long quad_tiles = (long long)((p.OH + 1) / 2) * ((p.OW + 27) / 28) * ((p.Kg + 63) / 64) *
                                     p.N * p.G;
        if (quad_tiles < 400 && tap_supported(p, pooled)) return V_TAP;
        // Fused pooling on maps up to 14 wide: the vector kernel's 4x14 pooled tile measures
        // 1.25-1.35x faster than the matrix kernel's at every batch size.
        if (pooled && p.W <= 14 && tap_supported(p, pooled)) return V_TAP;
        return V_QUAD;
    }
    if (tap_supported(p, pooled)) return wide_fills ? V_WIDE : V_TAP;   // 3x3 / stride 2 / pad 1
    if (wide_supported(p, pooled)) return V_WIDE;     // 3x3 with another stride or padding
    if (gen_supported(p, pooled)) return V_GEN;       // other kernel sizes, odd channel counts
    return V_ROWS;
}

static int run(Variant v, const Problem& p, bool pooled, const float* x, const float* w, float* y,
               hipStream_t s)
{
    // the launchers cache occupancy answers and attribute opt-ins in static variables: planning and
    // enqueueing are serialised across host threads (they take microseconds)
    static std::mutex guard;
    std::lock_guard<std::mutex> lock(guard);
    int rc = SCONV_EUNSUPPORTED;
    if (v == V_PW) rc = launch_pointwise(p, pooled, x, w, y, s);
    if (v == V_GEN) rc = launch_gen(p, pooled, x, w, y, s);
    if (v == V_WIDE) {
        rc = launch_wide(p, pooled, x, w, y, s);
        if (rc == SCONV_EUNSUPPORTED) v = quad_supported(p, pooled) ? V_QUAD : V_TAP;
    }
    if (v == V_QUAD) {
        rc = launch_quad(p, pooled, x, w, y, s);
        if (rc == SCONV_EUNSUPPORTED) v = V_TAP;
    }
    if (v == V_TAP && tap_supported(p, pooled)) rc = launch_tap(p, pooled, x, w, y, s);
    // no applicable tile plan: the general kernel runs
    if (rc == SCONV_EUNSUPPORTED) rc = launch_rows(p, pooled, x, w, y, s);
    return rc;
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
    return run(choose(p, false), p, false, x_dev, w_dev, y_dev, (hipStream_t)hip_stream);
}

extern "C" int sconv_pool_forward(const sconv_desc_t* desc, const float* x_dev, const float* w_dev,
                                  float* y_dev, void* hip_stream)
{
    if (!x_dev || !w_dev || !y_dev) return SCONV_EINVAL;
    Problem p;
    int rc = fill_problem(desc, true, &p);
    if (rc) return rc;
    if ((int64_t)p.ph * p.pw > 64) return SCONV_EUNSUPPORTED;
    return run(choose(p, true), p, true, x_dev, w_dev, y_dev, (hipStream_t)hip_stream);
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

extern "C" const char* sconv_variant_name(const sconv_desc_t* desc, int pooled)
{
    Problem p;
    if (fill_problem(desc, pooled != 0, &p)) return NULL;
    switch (choose(p, pooled != 0)) {
    case V_PW: return "quad1x1";
    case V_QUAD: return "quad3x3";
    case V_TAP: return "tap3x3";
    case V_WIDE: return "wide3x3";
    case V_GEN: return "gen";
    default: return "rows";
    }
}

extern "C" const char* sconv_strerror(int code)
{
    switch (code) {
    case SCONV_OK: return "success";
    case SCONV_EINVAL: return "invalid argument";
    case SCONV_EUNSUPPORTED: return "shape exceeds a kernel limit";
    case SCONV_ELAUNCH: return "HIP launch failed";
    default: return "unknown sconv error code";
    }
}

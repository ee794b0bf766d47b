/*
 * CPU oracle for zero-skipping direct convolution (+ fused ReLU / max-pooling).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the GPU library is
 * checked against.  Nothing on the product path may call it; it shares no code, header,
 * table or helper with the GPU library.
 *
 * What is written out here:
 *   - oracle_conv / oracle_conv_pool: the plain definition of the result.  The paper's method
 *     only skips terms that are zero (Section 5.4), so it reaches exactly (up to rounding
 *     order) the ordinary cross-correlation O = A * Im2col(I) of Section 2.2, followed by
 *     ReLU (Section 5.5) and, for the fused path, max pooling (Section 6.4).  Accumulation is
 *     fp64 over fp32 inputs, in plain loop order, with no blocking.
 *   - oracle_encode: the conversion of Algorithm 1 (ECR) and Algorithm 3 (PECR), step by step
 *     in the paper's scan order, because an encoding is a representation with exactly one
 *     correct value.
 *   - oracle_spmv: Algorithm 2 / the product part of Algorithm 4 evaluated on an encoding.
 *   - oracle_add_bias: the layer's bias, added to the plain sums before the ReLU.  The paper's
 *     kernels have no bias term; this is the ordinary definition of a convolution layer, pinned against
 *     a brute-force loop, the library's fp64 convolution with bias, and the zero-input / zero-bias
 *     special cases.
 *
 * Readings of the paper taken here (it is silent or inconsistent on these):
 *   - filter position of tap (i,j) is i*k_w + j, row-major (Algorithm 3 prints i*k_h+j and
 *     Algorithm 1 prints i+j*k_w; the three agree for square kernels up to Alg. 1's transpose,
 *     which is treated as a misprint);
 *   - loop bounds are exclusive (a k_h x k_w window has k_w*k_h values, Section 5.3);
 *   - several input channels are scanned one after another (Section 7), so a window's row has
 *     L = (C/groups)*k_h*k_w columns, column = c*k_h*k_w + i*k_w + j;
 *   - both formats store the column number ("Index"); the gathered filter values K_data of
 *     Section 5.2 are w[k][Index] for each filter k and are not stored;
 *   - slots after the last nonzero of a row hold value +0.0 and index 0;
 *   - zero padding contributes zeros, which are never emitted;
 *   - sizes that do not divide are floored.
 */
#include <omp.h>
#include <math.h>
#include <stdint.h>
#include <stddef.h>

#define ORACLE_FMT_ECR 0
#define ORACLE_FMT_PECR 1

typedef struct {
    int32_t N, C, H, W;          /* input x[N][C][H][W], fp32 */
    int32_t K, R, S;             /* filters w[K][C/groups][R][S], fp32 */
    int32_t stride, pad, groups; /* c_s, symmetric zero padding, G */
    int32_t pool_h, pool_w, pool_stride; /* p_h, p_w, p_s */
} oracle_shape_t;

/* Convolution output size, Section 5.3: (i - k)/c_s + 1 with i the padded extent. */
static int conv_out(int i, int k, int pad, int cs) { return (i + 2 * pad - k) / cs + 1; }
/* Pooled size: windows that do not fit are dropped. */
static int pool_out(int o, int p, int ps) { return o < p ? 0 : (o - p) / ps + 1; }

/* Number of threads the OpenMP loop of oracle_conv may use from now on (timing aid: the benchmark
 * times the oracle on all host cores and on one); returns the previous limit.  No arithmetic here. */
int oracle_set_threads(int n)
{
    const int before = omp_get_max_threads();
    if (n > 0) omp_set_num_threads(n);
    return before;
}

void oracle_output_dims(const oracle_shape_t* s, int32_t* OH, int32_t* OW, int32_t* PH, int32_t* PW)
{
    int oh = conv_out(s->H, s->R, s->pad, s->stride);
    int ow = conv_out(s->W, s->S, s->pad, s->stride);
    *OH = oh;
    *OW = ow;
    if (PH) *PH = s->pool_h > 0 ? pool_out(oh, s->pool_h, s->pool_stride) : 0;
    if (PW) *PW = s->pool_w > 0 ? pool_out(ow, s->pool_w, s->pool_stride) : 0;
}

/* Eq. (3): number of pooling results along one axis, as printed (before flooring). */
double oracle_eq3_n_o(double I_w, double k_w, double c_s, double p_w, double p_s)
{
    return (I_w - k_w + c_s - c_s * p_w + p_s * c_s) / (p_s * c_s);
}

/* Padded input read: zero outside the map. */
static float X(const float* x, const oracle_shape_t* s, int n, int c, int h, int w)
{
    if (h < 0 || h >= s->H || w < 0 || w >= s->W) return 0.0f;
    return x[(((size_t)n * s->C + c) * s->H + h) * s->W + w];
}

/* Number of encoded rows and slots per row for a format. */
void oracle_encode_sizes(const oracle_shape_t* s, int fmt, int64_t* rows, int64_t* L)
{
    int32_t OH, OW, PH, PW;
    oracle_output_dims(s, &OH, &OW, &PH, &PW);
    *L = (int64_t)(s->C / s->groups) * s->R * s->S;
    if (fmt == ORACLE_FMT_ECR)
        *rows = (int64_t)s->N * s->groups * OH * OW;
    else
        *rows = (int64_t)s->N * s->groups * PH * PW * s->pool_h * s->pool_w;
}

/* One window (n, g, oh, ow): the scan of Algorithm 1 / Algorithm 3, with the
 * channel loop of Section 7 outside.  Returns the number of nonzeros written. */
static int32_t encode_window(const float* x, const oracle_shape_t* s, int n, int g, int oh, int ow,
                             float* values, int32_t* index)
{
    const int Cg = s->C / s->groups;
    int32_t cnt = 0;
    for (int c = 0; c < Cg; ++c)
        for (int i = 0; i < s->R; ++i)
            for (int j = 0; j < s->S; ++j) {
                float v = X(x, s, n, g * Cg + c, oh * s->stride - s->pad + i, ow * s->stride - s->pad + j);
                if (v != 0) {
                    values[cnt] = v;
                    index[cnt] = (c * s->R + i) * s->S + j;
                    cnt++;
                }
            }
    return cnt;
}

/*
 * ECR rows in order (n, g, oh, ow): one block row per output row, one thread per output
 * column (Section 5.2); count is -1 for an empty window (the end of Algorithm 1).
 * PECR rows in order (n, g, ph, pw, py, px): pooling-pack rows of pooling windows, the
 * convolution windows inside a pooling window left to right, top to bottom (Section 6.2);
 * count is the plain number of nonzeros (the end of Algorithm 3).
 * values/index: [rows][L]; count: [rows].
 */
void oracle_encode(const oracle_shape_t* s, int fmt, const float* x, float* values, int32_t* index,
                   int32_t* count)
{
    int64_t rows, L;
    int32_t OH, OW, PH, PW;
    oracle_encode_sizes(s, fmt, &rows, &L);
    oracle_output_dims(s, &OH, &OW, &PH, &PW);
    for (int64_t i = 0; i < rows * L; ++i) {
        values[i] = 0.0f;
        index[i] = 0;
    }
    int64_t row = 0;
    for (int n = 0; n < s->N; ++n)
        for (int g = 0; g < s->groups; ++g) {
            if (fmt == ORACLE_FMT_ECR) {
                for (int oh = 0; oh < OH; ++oh)
                    for (int ow = 0; ow < OW; ++ow) {
                        int32_t cnt = encode_window(x, s, n, g, oh, ow, values + row * L, index + row * L);
                        count[row] = cnt != 0 ? cnt : -1;
                        row++;
                    }
            } else {
                for (int ph = 0; ph < PH; ++ph)
                    for (int pw = 0; pw < PW; ++pw)
                        for (int py = 0; py < s->pool_h; ++py)
                            for (int px = 0; px < s->pool_w; ++px) {
                                int oh = ph * s->pool_stride + py;
                                int ow = pw * s->pool_stride + px;
                                count[row] = encode_window(x, s, n, g, oh, ow, values + row * L, index + row * L);
                                row++;
                            }
            }
        }
}

/*
 * Algorithm 2 (and the product part of Algorithm 4) on an encoding: for every row and every filter k
 * of the row's group, sum value[i] * w[k][index[i]] over the row's nonzeros; an empty row gives
 * 0.  out: [rows][K/groups] in fp64; row order is that of the encoding.
 */
void oracle_spmv(const oracle_shape_t* s, int64_t rows, const float* values, const int32_t* index,
                 const int32_t* count, const float* w, double* out)
{
    const int Cg = s->C / s->groups, Kg = s->K / s->groups;
    const int64_t L = (int64_t)Cg * s->R * s->S;
    const int64_t rows_per_group = rows / ((int64_t)s->N * s->groups);
    /* rows are independent; every (row, filter) sum is still formed by one thread, in slot order */
#pragma omp parallel for schedule(static)
    for (int64_t row = 0; row < rows; ++row) {
        int g = (int)((row / rows_per_group) % s->groups);
        for (int kk = 0; kk < Kg; ++kk) {
            const float* wk = w + (size_t)(g * Kg + kk) * L;
            double acc = 0.0;
            if (count[row] > 0)
                for (int32_t i = 0; i < count[row]; ++i)
                    acc += (double)values[row * L + i] * (double)wk[index[row * L + i]];
            out[row * Kg + kk] = acc;
        }
    }
}

/*
 * Plain convolution (cross-correlation, no filter flip: each window row times the filter
 * vector, Section 2.2), zero padded, grouped; fp64 accumulation in loop order (c, r, s).
 * y[N][K][OH][OW]; absdot gets sum |x*w| of the same terms (the scale of the rounding-error
 * bound); relu != 0 applies max(y, 0) (Section 5.5).  absdot may be NULL.
 */
void oracle_conv(const oracle_shape_t* s, const float* x, const float* w, int relu, double* y,
                 double* absdot)
{
    const int Cg = s->C / s->groups, Kg = s->K / s->groups;
    int32_t OH, OW;
    oracle_output_dims(s, &OH, &OW, NULL, NULL);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < s->N; ++n)
        for (int k = 0; k < s->K; ++k) {
            const int g = k / Kg;
            for (int oh = 0; oh < OH; ++oh)
                for (int ow = 0; ow < OW; ++ow) {
                    double acc = 0.0, mag = 0.0;
                    for (int c = 0; c < Cg; ++c)
                        for (int r = 0; r < s->R; ++r)
                            for (int q = 0; q < s->S; ++q) {
                                double xv = X(x, s, n, g * Cg + c, oh * s->stride - s->pad + r,
                                              ow * s->stride - s->pad + q);
                                double wv = w[(((size_t)k * Cg + c) * s->R + r) * s->S + q];
                                acc += xv * wv;
                                mag += fabs(xv * wv);
                            }
                    if (relu && acc < 0.0) acc = 0.0;
                    size_t o = (((size_t)n * s->K + k) * OH + oh) * OW + ow;
                    y[o] = acc;
                    if (absdot) absdot[o] = mag;
                }
        }
}

/*
 * The same definition evaluated at listed outputs only (for tensors too large to compute whole):
 * points[i] = (n, k, oh, ow); y[i] and absdot[i] as in oracle_conv.
 */
void oracle_conv_at(const oracle_shape_t* s, const float* x, const float* w, int relu, int64_t npoints,
                    const int32_t* points, double* y, double* absdot)
{
    const int Cg = s->C / s->groups, Kg = s->K / s->groups;
    for (int64_t i = 0; i < npoints; ++i) {
        const int n = points[4 * i], k = points[4 * i + 1], oh = points[4 * i + 2], ow = points[4 * i + 3];
        const int g = k / Kg;
        double acc = 0.0, mag = 0.0;
        for (int c = 0; c < Cg; ++c)
            for (int r = 0; r < s->R; ++r)
                for (int q = 0; q < s->S; ++q) {
                    double xv = X(x, s, n, g * Cg + c, oh * s->stride - s->pad + r, ow * s->stride - s->pad + q);
                    double wv = w[(((size_t)k * Cg + c) * s->R + r) * s->S + q];
                    acc += xv * wv;
                    mag += fabs(xv * wv);
                }
        if (relu && acc < 0.0) acc = 0.0;
        y[i] = acc;
        if (absdot) absdot[i] = mag;
    }
}

/*
 * Bias of a convolution layer (not part of the paper's kernels, which stop at the products; the
 * affine term every layer they are taken from carries): y[n][k][.][.] += bias[k], applied to the plain
 * sums before the ReLU of Section 5.5.  y is a convolution computed WITHOUT ReLU; relu != 0 applies
 * max(y, 0) afterwards.  absdot (optional) grows by |bias[k]|: the bias is one more term of the sum
 * the rounding-error bound is scaled by.  count = OH*OW (or however many results each (n, k) has).
 */
void oracle_add_bias(int32_t N, int32_t K, int64_t count, const float* bias, int relu, double* y, double* absdot)
{
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int64_t i = 0; i < count; ++i) {
                size_t o = ((size_t)n * K + k) * (size_t)count + (size_t)i;
                double v = y[o] + (double)bias[k];
                if (relu && v < 0.0) v = 0.0;
                y[o] = v;
                if (absdot) absdot[o] += fabs((double)bias[k]);
            }
}

/*
 * Max pooling p_h x p_w with stride p_s, no padding, floor sizes, over an [N][K][OH][OW]
 * tensor: z[N][K][PH][PW] = max over the window.  scale_in/scale_out (optional) carry the
 * error scale: the window maximum of it (max is 1-Lipschitz in every argument).
 */
void oracle_maxpool(const oracle_shape_t* s, const double* y, const double* scale_in, double* z,
                    double* scale_out)
{
    int32_t OH, OW, PH, PW;
    oracle_output_dims(s, &OH, &OW, &PH, &PW);
    for (int n = 0; n < s->N; ++n)
        for (int k = 0; k < s->K; ++k)
            for (int ph = 0; ph < PH; ++ph)
                for (int pw = 0; pw < PW; ++pw) {
                    double m = -INFINITY, sc = 0.0;
                    for (int py = 0; py < s->pool_h; ++py)
                        for (int px = 0; px < s->pool_w; ++px) {
                            size_t i = (((size_t)n * s->K + k) * OH + ph * s->pool_stride + py) * OW +
                                       pw * s->pool_stride + px;
                            if (y[i] > m) m = y[i];
                            if (scale_in && scale_in[i] > sc) sc = scale_in[i];
                        }
                    size_t o = (((size_t)n * s->K + k) * PH + ph) * PW + pw;
                    z[o] = m;
                    if (scale_out) scale_out[o] = sc;
                }
}

/*
 * Fused path, Section 6.4: convolution, ReLU, then max over each pooling window.
 * conv_tmp/abs_tmp: caller-provided [N][K][OH][OW] work arrays; z/scale: [N][K][PH][PW].
 */
void oracle_conv_pool(const oracle_shape_t* s, const float* x, const float* w, double* conv_tmp,
                      double* abs_tmp, double* z, double* scale)
{
    oracle_conv(s, x, w, 1, conv_tmp, abs_tmp);
    oracle_maxpool(s, conv_tmp, abs_tmp, z, scale);
}

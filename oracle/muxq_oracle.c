/*
 * MUXQ CPU oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, step-by-step implementation of the MUXQ quantized linear
 * layer Y = X.W (paper Sec. II-A Eq. 1-3 and Sec. III-C Eq. 4-7), used only
 * to check the GPU library and to give a host-CPU timing beside it.  Only the
 * tests, the smoke check and the bench's cpu_baseline leg may call it.  It
 * shares no code, header, table or helper with the HIP path.
 *
 * Every function is one step of the method, written as the plain definition:
 * no blocking, no fusion, no intrinsics, no BLAS.  OpenMP only splits
 * independent output rows across threads; each output element is still
 * produced by the same serial loop.  Inputs are fp32 arrays holding fp16
 * values widened exactly (the Python wrapper does the widening and the final
 * fp16 rounding with numpy's conversions).
 *
 * All floating-point work is IEEE binary32 with round-to-nearest-even and no
 * contraction (build with -ffp-contract=off, no -ffast-math).
 *
 * Pins (tests marked "not gpu"): exact-rational brute force on tiny inputs,
 * a hand-worked example, numpy int64 matmul for the accumulators, the
 * zero-outlier special case against plain Eq. 1-3, the Eq. 6 reconstruction
 * identity, closed-form quantisation error bounds.  The per-token (per-row)
 * activation scales of the per-vector setting and the narrower code widths
 * of Tables 1-2 are pinned the same way: exact brute force, equality with
 * the per-tensor result when all rows share their abs-max, independence of
 * a row's codes from the other rows, the half-step bound per row, the step
 * ratio per bit removed.  The switches for the two readings the paper leaves
 * open (Aux on a scale of its own with the sum of Eq. 7 taken after
 * dequantisation; "X / s" as a division per element) and the per-channel
 * scaling of the SmoothQuant-style combination are pinned by the same exact
 * brute force, by equality with the default reading where the two must agree,
 * and by exactness for power-of-two factors.  No function here is "parity
 * unpinned".
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

#define QMAX_DEFAULT 127 /* 2^7 - 1, Eq. 1-2 */

/* Sec. III-C, outlier criterion: the per-channel (column) maximum magnitude
 * of the activation matrix X (M x K, row stride ldx). */
void muxq_oracle_col_absmax(const float *X, int64_t M, int64_t K, int64_t ldx,
                            float *colmax)
{
    for (int64_t k = 0; k < K; ++k)
        colmax[k] = 0.0f;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k) {
            float a = fabsf(X[m * ldx + k]);
            if (a > colmax[k])
                colmax[k] = a;
        }
}

/* Sec. III-C: a channel is an outlier channel when at least one of its
 * elements has magnitude strictly greater than the threshold (6 in the
 * paper).  Channels are listed in ascending order; when more than r_cap
 * qualify only the r_cap lowest-indexed ones are kept (capacity rule of the
 * library boundary) and *n_total still reports how many qualified.
 * Unused idx entries are set to -1.  Returns the number kept. */
int32_t muxq_oracle_select_outliers(const float *colmax, int64_t K,
                                    float threshold, int32_t r_cap,
                                    int32_t *idx, int32_t *n_total)
{
    int32_t kept = 0, total = 0;
    for (int64_t k = 0; k < K; ++k) {
        if (colmax[k] > threshold) {
            if (kept < r_cap)
                idx[kept++] = (int32_t)k;
            ++total;
        }
    }
    for (int32_t j = kept; j < r_cap; ++j)
        idx[j] = -1;
    *n_total = total;
    return kept;
}

/* Eq. 4-5: Body equals X except that the outlier columns are shifted down by
 * `e` binary exponent steps (multiplied by 2^-e, exact in fp32 for every fp16
 * input); Aux (M x r, compact) is a copy of those shrunk columns. */
void muxq_oracle_decompose(const float *X, int64_t M, int64_t K, int64_t ldx,
                           const int32_t *idx, int32_t r, int32_t e,
                           float *body, float *aux)
{
    const float shrink = ldexpf(1.0f, -e);
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t k = 0; k < K; ++k)
            body[m * K + k] = X[m * ldx + k];
        for (int32_t j = 0; j < r; ++j) {
            float v = X[m * ldx + idx[j]] * shrink;
            body[m * K + idx[j]] = v;
            aux[m * (int64_t)r + j] = v;
        }
    }
}

/* Eq. 6: X_outlier = Body_outlier + (2^e - 1) Aux, evaluated in fp32 (exact
 * for fp16 inputs).  Writes the reconstructed M x r outlier submatrix. */
void muxq_oracle_reconstruct(const float *body, const float *aux, int64_t M,
                             int64_t K, const int32_t *idx, int32_t r,
                             int32_t e, float *x_outlier)
{
    const float c = (float)((1 << e) - 1);
    for (int64_t m = 0; m < M; ++m)
        for (int32_t j = 0; j < r; ++j)
            x_outlier[m * (int64_t)r + j] =
                body[m * K + idx[j]] + c * aux[m * (int64_t)r + j];
}

/* max |v| over a flat array (the abs-max of Eq. 1-2 for one quantisation
 * unit). */
float muxq_oracle_absmax(const float *V, int64_t n)
{
    float amax = 0.0f;
    for (int64_t i = 0; i < n; ++i) {
        float a = fabsf(V[i]);
        if (a > amax)
            amax = a;
    }
    return amax;
}

/* Eq. 1-2: scale s = amax / qmax and its reciprocal form inv = qmax / amax,
 * each one correctly rounded fp32 division.  An all-zero unit gives s = 0 and
 * inv = 0 (every code 0). */
void muxq_oracle_scale(float amax, int32_t qmax, float *s, float *inv)
{
    if (amax > 0.0f) {
        *s = amax / (float)qmax;
        *inv = (float)qmax / amax;
    } else {
        *s = 0.0f;
        *inv = 0.0f;
    }
}

/* Eq. 1-2, one element: round-to-nearest-even of v*inv, clamped to the
 * symmetric range [-qmax, qmax]. */
static int8_t quantize_one(float v, float inv, int32_t qmax)
{
    float t = nearbyintf(v * inv); /* default rounding mode: nearest even */
    if (t > (float)qmax)
        t = (float)qmax;
    if (t < -(float)qmax)
        t = -(float)qmax;
    return (int8_t)t;
}

/* Eq. 1 (and Eq. 2 per-tensor): quantise a flat array with one scale. */
void muxq_oracle_quantize(const float *V, int64_t n, float inv, int32_t qmax,
                          int8_t *q)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        q[i] = quantize_one(V[i], inv, qmax);
}

/* Per-vector quantisation, one scale per ROW of a rows x cols matrix
 * (per-token activations, Fig. 2(a)). */
void muxq_oracle_quantize_rows(const float *V, int64_t rows, int64_t cols,
                               const float *inv_row, int32_t qmax, int8_t *q)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t j = 0; j < cols; ++j)
            q[i * cols + j] = quantize_one(V[i * cols + j], inv_row[i], qmax);
}

/* Per-vector quantisation, one scale per COLUMN of a rows x cols matrix
 * (per-channel weights, Fig. 2(a)). */
void muxq_oracle_quantize_cols(const float *V, int64_t rows, int64_t cols,
                               const float *inv_col, int32_t qmax, int8_t *q)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t j = 0; j < cols; ++j)
            q[i * cols + j] = quantize_one(V[i * cols + j], inv_col[j], qmax);
}

/* max |v| per row of a rows x cols matrix. */
void muxq_oracle_row_absmax(const float *V, int64_t rows, int64_t cols,
                            float *rowmax)
{
    for (int64_t i = 0; i < rows; ++i)
        rowmax[i] = muxq_oracle_absmax(V + i * cols, cols);
}

/* Rows idx[0..r) of the quantised weight (K x N): the part of W that meets
 * the non-zero columns of Aux in Y_Aux = Aux.W of Eq. 7. */
void muxq_oracle_gather_rows(const int8_t *wq, int64_t N, const int32_t *idx,
                             int32_t r, int8_t *w_rows)
{
    for (int32_t j = 0; j < r; ++j)
        for (int64_t n = 0; n < N; ++n)
            w_rows[(int64_t)j * N + n] = wq[(int64_t)idx[j] * N + n];
}

/* Eq. 3 / Eq. 7 integer product: acc[m][n] = sum_k A[m][k] * B[k][n] in
 * int32, A is M x K, B is K x N, both row-major int8.  The classic triple
 * loop; rows of the output are independent and split across threads. */
void muxq_oracle_gemm_i8(const int8_t *A, const int8_t *B, int64_t M,
                         int64_t N, int64_t K, int32_t *acc)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        int32_t *row = acc + m * N;
        for (int64_t n = 0; n < N; ++n)
            row[n] = 0;
        for (int64_t k = 0; k < K; ++k) {
            const int32_t a = A[m * K + k];
            const int8_t *b = B + k * N;
            for (int64_t n = 0; n < N; ++n)
                row[n] += a * (int32_t)b[n];
        }
    }
}

/* Eq. 7 recombination carried out on the integer accumulators (both
 * products share one activation scale and one weight scale):
 * acc = acc_body + (2^e - 1) * acc_aux. */
void muxq_oracle_recombine(const int32_t *acc_body, const int32_t *acc_aux,
                           int64_t n, int32_t e, int32_t *acc)
{
    const int32_t c = (1 << e) - 1;
    for (int64_t i = 0; i < n; ++i)
        acc[i] = acc_body[i] + c * acc_aux[i];
}

/* Eq. 3 dequantisation: y = (s_x * s_w) * acc (+ bias), fp32, in exactly
 * this order: one fp32 product of the two scales, one int->fp32 conversion
 * (nearest even), one fp32 product, one fp32 add when a bias is given.
 * s_x has one entry (per-tensor) or M entries (per-token); s_w has one entry
 * (per-tensor) or N entries (per-channel). */
void muxq_oracle_dequant(const int32_t *acc, int64_t M, int64_t N,
                         const float *s_x, int32_t sx_per_row,
                         const float *s_w, int32_t sw_per_col,
                         const float *bias, float *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            float sx = sx_per_row ? s_x[m] : s_x[0];
            float sw = sw_per_col ? s_w[n] : s_w[0];
            float scale = sx * sw;
            float v = scale * (float)acc[m * N + n];
            if (bias)
                v = v + bias[n];
            y[m * N + n] = v;
        }
}

/* Eq. 1-2 read literally: q = round(v / s), the division carried out per
 * element in fp32 (correctly rounded), instead of the multiplication by the
 * reciprocal form that the other quantisers here use.  One scale per matrix
 * (s_row_stride = s_col_stride = 0), per row (s_row_stride = 1) or per column
 * (s_col_stride = 1).  A zero scale gives code 0.  Only used to measure how
 * often the two readings of "X / s" disagree. */
void muxq_oracle_quantize_div(const float *V, int64_t rows, int64_t cols,
                              const float *s, int64_t s_row_stride,
                              int64_t s_col_stride, int32_t qmax, int8_t *q)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t j = 0; j < cols; ++j) {
            float sc = s[i * s_row_stride + j * s_col_stride];
            float t = 0.0f;
            if (sc > 0.0f)
                t = nearbyintf(V[i * cols + j] / sc);
            if (t > (float)qmax)
                t = (float)qmax;
            if (t < -(float)qmax)
                t = -(float)qmax;
            q[i * cols + j] = (int8_t)t;
        }
}

/* Eq. 7 with Aux quantised on a scale of its own (the other reading of Eq. 5:
 * Aux is a matrix like any other and gets the abs-max scale of Eq. 1).  The
 * two integer products then live on different scales and are recombined after
 * dequantisation, in fp32, in exactly this order:
 *   y_body = (s_x * s_w) * acc_body,   y_aux = (s_aux * s_w) * acc_aux,
 *   y = y_body + (2^e - 1) * y_aux  (+ bias).
 * s_x and s_aux have one entry (per-tensor) or M entries (per-token). */
void muxq_oracle_dequant_sum(const int32_t *acc_body, const int32_t *acc_aux,
                             int64_t M, int64_t N, const float *s_x,
                             const float *s_aux, int32_t sx_per_row,
                             const float *s_w, int32_t sw_per_col, int32_t e,
                             const float *bias, float *y)
{
    const float c = (float)((1 << e) - 1);
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            float sx = sx_per_row ? s_x[m] : s_x[0];
            float sa = sx_per_row ? s_aux[m] : s_aux[0];
            float sw = sw_per_col ? s_w[n] : s_w[0];
            float scale_b = sx * sw;
            float y_body = scale_b * (float)acc_body[m * N + n];
            float scale_a = sa * sw;
            float y_aux = scale_a * (float)acc_aux[m * N + n];
            float t = c * y_aux;
            float v = y_body + t;
            if (bias)
                v = v + bias[n];
            y[m * N + n] = v;
        }
}

/* Difficulty migration between activations and weights (the combination with
 * SmoothQuant-style scaling that Sec. V names): channel k of X is divided by a
 * positive factor f[k] and row k of W multiplied by it, which leaves X.W
 * unchanged in exact arithmetic.  Done in fp32 and rounded back to fp16 values
 * (the operands a layer receives are fp16): out = fp16(v / f[k]) or
 * fp16(v * f[k]).  The fp16 rounding is done by the caller (numpy); these two
 * loops only do the fp32 step. */
void muxq_oracle_scale_cols(const float *X, int64_t M, int64_t K, const float *f,
                            int32_t divide, float *out)
{
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k)
            out[m * K + k] = divide ? X[m * K + k] / f[k] : X[m * K + k] * f[k];
}

void muxq_oracle_scale_rows(const float *W, int64_t K, int64_t N, const float *f,
                            int32_t divide, float *out)
{
    for (int64_t k = 0; k < K; ++k)
        for (int64_t n = 0; n < N; ++n)
            out[k * N + n] = divide ? W[k * N + n] / f[k] : W[k * N + n] * f[k];
}

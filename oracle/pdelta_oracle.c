/*
 * pdelta_oracle.c - CPU reference ("oracle") for the 1-bit per-axis weight-delta path.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It exists so that the GPU library can be
 * checked against something slow, plain and obviously right.  Only the tests, the smoke check
 * and the bench's cpu_baseline leg may call it.  It shares no code, header, table or helper
 * with the HIP library and neither includes the other.
 *
 * What it computes (paper, Section 2 "Method"):
 *   Delta W = W_f - W_b,   B = sign(Delta W) in {-1,+1}^(d_out x d_in)      (definition of B)
 *   W_hat   = v (.) B + W_b, v in R^(1 x d_out) (row) or R^(d_in x 1) (col)  (Eq. 1)
 *   Y       = X * W_hat^T                                                    (layer forward)
 *   v_0     = mean |Delta W| taken per output row / per input column        (Alg. "Per-layer
 *             compression with Row/Col selection", initialisation of v_r and v_c)
 *   Pack    = one bit per entry, consecutive input indices share a word     (Implementation
 *             remarks: the masks are kept bit-packed along the input axis)
 *
 * Everything floating point is done in fp64 on values decoded exactly from their 16-bit
 * storage format.  Nothing is blocked, fused or reordered: W_hat is rebuilt densely and the
 * product is the textbook triple loop.  OpenMP only spreads independent output rows over
 * threads; every individual sum runs in index order.
 *
 * Readings taken where the paper is silent (listed with their reasons in the design notes):
 *   - sign(0) = +1 (B has no zero entries).  Implemented as bit = !(W_f < W_b) on the decoded
 *     values, so +0, -0 and equal operands all give +1.
 *   - storage is [d_out, d_in] row-major; "row" mode has one scale per output feature
 *     (length d_out), "col" mode one per input feature (length d_in).
 *   - words are uint32, LSB first: entry (o, i) is bit (i % 32) of word [o][i / 32];
 *     bit 1 <-> +1, bit 0 <-> -1.  A ragged last word is padded with 0 bits that unpack ignores.
 *   - v is stored as fp16: v = RNE_fp16( fp64(sum |Delta W|) / count ).
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py (hand-written words,
 * exact rational arithmetic, closed forms, library matmul in the v = 0 case, brute force on
 * 4 x 8; the blockwise-scale functions also by their reductions to row mode, column mode and a
 * constant scale).  Nothing in this file is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { REF_F16 = 0, REF_BF16 = 1 };
enum { REF_OK = 0, REF_EINVAL = -1 };

/* ---- exact decode of a 16-bit pattern to fp64 ------------------------------------------- */

/* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits. */
static double decode_f16(uint16_t h)
{
    int s = (h >> 15) & 1, e = (h >> 10) & 0x1f, f = h & 0x3ff;
    double mag;
    if (e == 0)
        mag = ldexp((double)f, -24);                 /* zero and subnormals: f * 2^-24 */
    else if (e == 31)
        mag = f ? NAN : INFINITY;
    else
        mag = ldexp((double)(1024 + f), e - 25);     /* (1 + f/1024) * 2^(e-15) */
    return s ? -mag : mag;
}

/* bfloat16: 1 sign, 8 exponent (bias 127), 7 fraction bits (the top half of an fp32). */
static double decode_bf16(uint16_t h)
{
    int s = (h >> 15) & 1, e = (h >> 7) & 0xff, f = h & 0x7f;
    double mag;
    if (e == 0)
        mag = ldexp((double)f, -133);                /* f/128 * 2^-126 */
    else if (e == 255)
        mag = f ? NAN : INFINITY;
    else
        mag = ldexp((double)(128 + f), e - 134);     /* (1 + f/128) * 2^(e-127) */
    return s ? -mag : mag;
}

double pdelta_ref_decode(uint16_t bits, int dtype)
{
    return dtype == REF_BF16 ? decode_bf16(bits) : decode_f16(bits);
}

/* ---- round-to-nearest-even from fp64 to a 16-bit format ---------------------------------- */

/* p = number of stored fraction bits, emin = exponent of the smallest normal, bias, emax =
 * exponent of the largest finite.  rint() rounds to nearest even in the default FP environment. */
static uint16_t rne_generic(double x, int p, int emin, int bias, int emax)
{
    uint16_t sign = signbit(x) ? 0x8000 : 0;
    uint16_t inf = (uint16_t)((((emax + bias + 1) << p)));
    if (isnan(x)) return (uint16_t)(sign | inf | (1u << (p - 1)));
    double a = fabs(x);
    if (isinf(a)) return (uint16_t)(sign | inf);
    if (a < ldexp(1.0, emin)) {
        /* subnormal range: spacing is 2^(emin-p); a carry into 2^p lands on the first normal */
        double q = rint(ldexp(a, p - emin));
        return (uint16_t)(sign | (uint16_t)q);
    }
    int ex;
    (void)frexp(a, &ex);                 /* a = f * 2^ex, f in [0.5, 1)  =>  2^(ex-1) <= a */
    int e = ex - 1;
    double q = rint(ldexp(a, p - e));    /* in [2^p, 2^(p+1)] */
    if (q >= ldexp(1.0, p + 1)) { q = ldexp(1.0, p); e += 1; }
    if (e > emax) return (uint16_t)(sign | inf);
    return (uint16_t)(sign | (uint16_t)((e + bias) << p) | (uint16_t)((long)q - (1L << p)));
}

uint16_t pdelta_ref_rne_f16(double x)  { return rne_generic(x, 10, -14, 15, 15); }
uint16_t pdelta_ref_rne_bf16(double x) { return rne_generic(x, 7, -126, 127, 127); }

/* Array forms of the two conversions above (same arithmetic, one call per array). */
void pdelta_ref_decode_array(const uint16_t* bits, int64_t n, int dtype, double* out)
{
    for (int64_t j = 0; j < n; ++j) out[j] = pdelta_ref_decode(bits[j], dtype);
}

void pdelta_ref_rne_array(const double* x, int64_t n, int dtype, uint16_t* out)
{
    for (int64_t j = 0; j < n; ++j)
        out[j] = dtype == REF_BF16 ? pdelta_ref_rne_bf16(x[j]) : pdelta_ref_rne_f16(x[j]);
}

static int64_t words_per_row(int64_t d_in) { return (d_in + 31) / 32; }

/* ---- sign + pack + per-axis mean |Delta W| ------------------------------------------------
 * B = sign(W_f - W_b) (Section 2), packed one bit per entry along the input axis
 * (Implementation remarks); v_row[o] = mean_i |Delta W[o,i]|, v_col[i] = mean_o |Delta W[o,i]|
 * (initial values of v_r / v_c in the per-layer compression algorithm), stored as fp16.
 * v_row / v_col may be NULL.  B_packed is [d_out, ceil(d_in/32)].                           */
int pdelta_pack_ref(const uint16_t* W_f, const uint16_t* W_b, int64_t d_out, int64_t d_in,
                    int w_dtype, uint32_t* B_packed, uint16_t* v_row, uint16_t* v_col)
{
    if (!W_f || !W_b || !B_packed || d_out <= 0 || d_in <= 0) return REF_EINVAL;
    if (w_dtype != REF_F16 && w_dtype != REF_BF16) return REF_EINVAL;
    int64_t wpr = words_per_row(d_in);
    memset(B_packed, 0, (size_t)(d_out * wpr) * sizeof(uint32_t));

    for (int64_t o = 0; o < d_out; ++o) {
        double s_row = 0.0;
        for (int64_t i = 0; i < d_in; ++i) {
            double wf = pdelta_ref_decode(W_f[o * d_in + i], w_dtype);
            double wb = pdelta_ref_decode(W_b[o * d_in + i], w_dtype);
            if (!(wf < wb)) B_packed[o * wpr + i / 32] |= (uint32_t)1 << (i % 32);
            s_row += fabs(wf - wb);
        }
        if (v_row) v_row[o] = pdelta_ref_rne_f16(s_row / (double)d_in);
    }
    if (v_col) {
        for (int64_t i = 0; i < d_in; ++i) {
            double s_col = 0.0;
            for (int64_t o = 0; o < d_out; ++o) {
                double wf = pdelta_ref_decode(W_f[o * d_in + i], w_dtype);
                double wb = pdelta_ref_decode(W_b[o * d_in + i], w_dtype);
                s_col += fabs(wf - wb);
            }
            v_col[i] = pdelta_ref_rne_f16(s_col / (double)d_out);
        }
    }
    return REF_OK;
}

/* ---- unpack: B[o,i] = +1.0 if the bit is set, else -1.0 (B in {-1,+1}, Section 2) -------- */
int pdelta_unpack_ref(const uint32_t* B_packed, int64_t d_out, int64_t d_in, double* B)
{
    if (!B_packed || !B || d_out <= 0 || d_in <= 0) return REF_EINVAL;
    int64_t wpr = words_per_row(d_in);
    for (int64_t o = 0; o < d_out; ++o)
        for (int64_t i = 0; i < d_in; ++i)
            B[o * d_in + i] = ((B_packed[o * wpr + i / 32] >> (i % 32)) & 1u) ? 1.0 : -1.0;
    return REF_OK;
}

/* ---- patch: W_hat = v (.) B + W_b (Eq. 1), exact in fp64 ------------------------------------
 * axis 0 (row): v has d_out entries and W_hat[o,i] = W_b[o,i] + v[o] * B[o,i].
 * axis 1 (col): v has d_in  entries and W_hat[o,i] = W_b[o,i] + v[i] * B[o,i].               */
int pdelta_patch_ref(const uint16_t* W_b, const uint32_t* B_packed, const uint16_t* v, int axis,
                     int64_t d_out, int64_t d_in, int w_dtype, double* W_hat)
{
    if (!W_b || !B_packed || !v || !W_hat || d_out <= 0 || d_in <= 0) return REF_EINVAL;
    if (axis != 0 && axis != 1) return REF_EINVAL;
    int64_t wpr = words_per_row(d_in);
    for (int64_t o = 0; o < d_out; ++o)
        for (int64_t i = 0; i < d_in; ++i) {
            double b = ((B_packed[o * wpr + i / 32] >> (i % 32)) & 1u) ? 1.0 : -1.0;
            double scale = decode_f16(axis == 0 ? v[o] : v[i]);
            W_hat[o * d_in + i] = pdelta_ref_decode(W_b[o * d_in + i], w_dtype) + scale * b;
        }
    return REF_OK;
}

/* The merged weights as they would be stored: one RNE rounding of the exact fp64 sum to the
 * weight dtype (the one-time merge of every residual term, Limitations section).             */
int pdelta_patch_round_ref(const uint16_t* W_b, const uint32_t* B_packed, const uint16_t* v,
                           int axis, int64_t d_out, int64_t d_in, int w_dtype, uint16_t* W_out)
{
    if (!W_out) return REF_EINVAL;
    double* W_hat = (double*)malloc((size_t)(d_out * d_in) * sizeof(double));
    if (!W_hat) return REF_EINVAL;
    int rc = pdelta_patch_ref(W_b, B_packed, v, axis, d_out, d_in, w_dtype, W_hat);
    if (rc == REF_OK)
        for (int64_t j = 0; j < d_out * d_in; ++j)
            W_out[j] = w_dtype == REF_BF16 ? pdelta_ref_rne_bf16(W_hat[j])
                                           : pdelta_ref_rne_f16(W_hat[j]);
    free(W_hat);
    return rc;
}

/* ---- delta linear: Y = X * W_hat^T with W_hat rebuilt densely (Eq. 1 + layer forward) ------
 * X is [M, d_in] in x_dtype, W_b is [d_out, d_in] in the same dtype, Y is [M, d_out] fp64.   */
int pdelta_linear_ref(const uint16_t* X, const uint16_t* W_b, const uint32_t* B_packed,
                      const uint16_t* v, int axis, int64_t M, int64_t d_out, int64_t d_in,
                      int x_dtype, double* Y)
{
    if (!X || !Y || M <= 0) return REF_EINVAL;
    double* W_hat = (double*)malloc((size_t)(d_out * d_in) * sizeof(double));
    double* Xd = (double*)malloc((size_t)(M * d_in) * sizeof(double));
    if (!W_hat || !Xd) { free(W_hat); free(Xd); return REF_EINVAL; }
    int rc = pdelta_patch_ref(W_b, B_packed, v, axis, d_out, d_in, x_dtype, W_hat);
    if (rc == REF_OK) {
        for (int64_t j = 0; j < M * d_in; ++j) Xd[j] = pdelta_ref_decode(X[j], x_dtype);
#pragma omp parallel for schedule(static)
        for (int64_t o = 0; o < d_out; ++o)
            for (int64_t m = 0; m < M; ++m) {
                double acc = 0.0;
                for (int64_t i = 0; i < d_in; ++i) acc += Xd[m * d_in + i] * W_hat[o * d_in + i];
                Y[m * d_out + o] = acc;
            }
    }
    free(W_hat);
    free(Xd);
    return rc;
}

/* The same definition evaluated at chosen outputs only, for layers too large to multiply whole:
 * y[s] = sum_i X[m_s, i] * (W_b[o_s, i] + scale * B[o_s, i]).                                 */
int pdelta_linear_ref_at(const uint16_t* X, const uint16_t* W_b, const uint32_t* B_packed,
                         const uint16_t* v, int axis, int64_t M, int64_t d_out, int64_t d_in,
                         int x_dtype, int64_t n, const int64_t* m_idx, const int64_t* o_idx,
                         double* y)
{
    if (!X || !W_b || !B_packed || !v || !y || !m_idx || !o_idx) return REF_EINVAL;
    if (M <= 0 || d_out <= 0 || d_in <= 0 || n < 0 || (axis != 0 && axis != 1)) return REF_EINVAL;
    int64_t wpr = words_per_row(d_in);
    for (int64_t s = 0; s < n; ++s)
        if (m_idx[s] < 0 || m_idx[s] >= M || o_idx[s] < 0 || o_idx[s] >= d_out) return REF_EINVAL;
#pragma omp parallel for schedule(static)
    for (int64_t s = 0; s < n; ++s) {
        int64_t m = m_idx[s], o = o_idx[s];
        double acc = 0.0;
        for (int64_t i = 0; i < d_in; ++i) {
            double b = ((B_packed[o * wpr + i / 32] >> (i % 32)) & 1u) ? 1.0 : -1.0;
            double scale = decode_f16(axis == 0 ? v[o] : v[i]);
            double w_hat = pdelta_ref_decode(W_b[o * d_in + i], x_dtype) + scale * b;
            acc += pdelta_ref_decode(X[m * d_in + i], x_dtype) * w_hat;
        }
        y[s] = acc;
    }
    return REF_OK;
}

/*
 * Gradient of a loss with respect to the scale vector, given dY = dL/dY (algorithm "Train
 * per-row/column scaling vectors via activation matching": the loss is backpropagated through
 * v only).  From Eq. 1 inside the layer forward, Y[m,o] = sum_i X[m,i] (W_b[o,i] + v. B[o,i]):
 *   row:  dL/dv[o] = sum_m dY[m,o] * sum_i X[m,i] B[o,i]
 *   col:  dL/dv[i] = sum_m X[m,i] * sum_o dY[m,o] B[o,i]
 * Plain loops in fp64, sums in index order.  grad has d_out (row) or d_in (col) entries.
 */
int pdelta_grad_v_ref(const uint16_t* X, const uint16_t* dY, const uint32_t* B_packed, int axis,
                      int64_t M, int64_t d_out, int64_t d_in, int dtype, double* grad)
{
    if (!X || !dY || !B_packed || !grad || M < 0 || d_out <= 0 || d_in <= 0) return -1;
    if (axis != 0 && axis != 1) return -1;
    const int64_t wpr = words_per_row(d_in);
    const int64_t n = axis == 0 ? d_out : d_in;
#pragma omp parallel for schedule(static)
    for (int64_t a = 0; a < n; ++a) {
        double g = 0.0;
        for (int64_t m = 0; m < M; ++m) {
            if (axis == 0) {
                double s = 0.0;
                for (int64_t i = 0; i < d_in; ++i) {
                    const double b = ((B_packed[a * wpr + i / 32] >> (i % 32)) & 1u) ? 1.0 : -1.0;
                    s += pdelta_ref_decode(X[m * d_in + i], dtype) * b;
                }
                g += pdelta_ref_decode(dY[m * d_out + a], dtype) * s;
            } else {
                double t = 0.0;
                for (int64_t o = 0; o < d_out; ++o) {
                    const double b = ((B_packed[o * wpr + a / 32] >> (a % 32)) & 1u) ? 1.0 : -1.0;
                    t += pdelta_ref_decode(dY[m * d_out + o], dtype) * b;
                }
                g += pdelta_ref_decode(X[m * d_in + a], dtype) * t;
            }
        }
        grad[a] = g;
    }
    return 0;
}

/* ---- blockwise ("per-group") and scalar scales -------------------------------------------------
 * The paper names blockwise per-group scales as the first extension of the per-axis vectors
 * (Conclusion) and compares against a single learned scalar per matrix (the BitDelta baseline
 * of the Experiments section).  Both are the same Eq. 1, W_hat = v (.) B + W_b, with v constant
 * over blocks of the matrix instead of along one whole axis:
 *     scale(o, i) = v[ (v_rows == 1 ? 0 : o) * (d_in / group) + i / group ]
 * v has v_rows x (d_in / group) entries; v_rows is d_out (one scale per output row and group of
 * `group` consecutive inputs) or 1 (the rows share the scales).  Special cases:
 *     v_rows = d_out, group = d_in   row mode            (one scale per output row)
 *     v_rows = 1,     group = 1      column mode         (one scale per input)
 *     v_rows = 1,     group = d_in   one scalar for the whole matrix
 * group must divide d_in.  The initial value of each scale is the mean of |Delta W| over the
 * entries it covers (the per-layer compression algorithm's initialisation, applied per block),
 * rounded once to fp16.                                                                       */
static int group_args_ok(int64_t d_out, int64_t d_in, int64_t group, int64_t v_rows)
{
    return d_out > 0 && d_in > 0 && group > 0 && d_in % group == 0 && (v_rows == 1 || v_rows == d_out);
}

static double group_scale(const uint16_t* v, int64_t o, int64_t i, int64_t d_in, int64_t group,
                          int64_t v_rows)
{
    int64_t n_groups = d_in / group;
    return decode_f16(v[(v_rows == 1 ? 0 : o) * n_groups + i / group]);
}

/* Signs as in pdelta_pack_ref, scales per block: v[r, g] = RNE_fp16(mean |W_f - W_b|) over the
 * rows r covers (one row, or all of them when v_rows == 1) and inputs g*group .. g*group+group-1. */
int pdelta_pack_group_ref(const uint16_t* W_f, const uint16_t* W_b, int64_t d_out, int64_t d_in,
                          int w_dtype, int64_t group, int64_t v_rows, uint32_t* B_packed, uint16_t* v)
{
    if (!W_f || !W_b || !B_packed || !v || !group_args_ok(d_out, d_in, group, v_rows)) return REF_EINVAL;
    int rc = pdelta_pack_ref(W_f, W_b, d_out, d_in, w_dtype, B_packed, NULL, NULL);
    if (rc != REF_OK) return rc;
    int64_t n_groups = d_in / group;
    for (int64_t r = 0; r < v_rows; ++r)
        for (int64_t g = 0; g < n_groups; ++g) {
            int64_t o_first = v_rows == 1 ? 0 : r, o_last = v_rows == 1 ? d_out - 1 : r;
            double sum = 0.0;
            for (int64_t o = o_first; o <= o_last; ++o)
                for (int64_t i = g * group; i < (g + 1) * group; ++i)
                    sum += fabs(pdelta_ref_decode(W_f[o * d_in + i], w_dtype) -
                                pdelta_ref_decode(W_b[o * d_in + i], w_dtype));
            double count = (double)(o_last - o_first + 1) * (double)group;
            v[r * n_groups + g] = pdelta_ref_rne_f16(sum / count);
        }
    return REF_OK;
}

/* W_hat = W_b + scale(o, i) * B (Eq. 1 with blockwise scales), exact in fp64. */
int pdelta_patch_group_ref(const uint16_t* W_b, const uint32_t* B_packed, const uint16_t* v,
                           int64_t group, int64_t v_rows, int64_t d_out, int64_t d_in, int w_dtype,
                           double* W_hat)
{
    if (!W_b || !B_packed || !v || !W_hat || !group_args_ok(d_out, d_in, group, v_rows)) return REF_EINVAL;
    int64_t wpr = words_per_row(d_in);
    for (int64_t o = 0; o < d_out; ++o)
        for (int64_t i = 0; i < d_in; ++i) {
            double b = ((B_packed[o * wpr + i / 32] >> (i % 32)) & 1u) ? 1.0 : -1.0;
            W_hat[o * d_in + i] = pdelta_ref_decode(W_b[o * d_in + i], w_dtype) +
                                  group_scale(v, o, i, d_in, group, v_rows) * b;
        }
    return REF_OK;
}

/* The merged weights as stored: one RNE rounding of the exact sum to the weight dtype. */
int pdelta_patch_group_round_ref(const uint16_t* W_b, const uint32_t* B_packed, const uint16_t* v,
                                 int64_t group, int64_t v_rows, int64_t d_out, int64_t d_in,
                                 int w_dtype, uint16_t* W_out)
{
    if (!W_out || d_out <= 0 || d_in <= 0) return REF_EINVAL;
    double* W_hat = (double*)malloc((size_t)(d_out * d_in) * sizeof(double));
    if (!W_hat) return REF_EINVAL;
    int rc = pdelta_patch_group_ref(W_b, B_packed, v, group, v_rows, d_out, d_in, w_dtype, W_hat);
    if (rc == REF_OK)
        for (int64_t j = 0; j < d_out * d_in; ++j)
            W_out[j] = w_dtype == REF_BF16 ? pdelta_ref_rne_bf16(W_hat[j]) : pdelta_ref_rne_f16(W_hat[j]);
    free(W_hat);
    return rc;
}

/* Y = X * W_hat^T with W_hat rebuilt densely from blockwise scales; Y is [M, d_out] fp64. */
int pdelta_linear_group_ref(const uint16_t* X, const uint16_t* W_b, const uint32_t* B_packed,
                            const uint16_t* v, int64_t group, int64_t v_rows, int64_t M,
                            int64_t d_out, int64_t d_in, int x_dtype, double* Y)
{
    if (!X || !Y || M <= 0 || d_out <= 0 || d_in <= 0) return REF_EINVAL;
    double* W_hat = (double*)malloc((size_t)(d_out * d_in) * sizeof(double));
    double* Xd = (double*)malloc((size_t)(M * d_in) * sizeof(double));
    if (!W_hat || !Xd) { free(W_hat); free(Xd); return REF_EINVAL; }
    int rc = pdelta_patch_group_ref(W_b, B_packed, v, group, v_rows, d_out, d_in, x_dtype, W_hat);
    if (rc == REF_OK) {
        for (int64_t j = 0; j < M * d_in; ++j) Xd[j] = pdelta_ref_decode(X[j], x_dtype);
#pragma omp parallel for schedule(static)
        for (int64_t o = 0; o < d_out; ++o)
            for (int64_t m = 0; m < M; ++m) {
                double acc = 0.0;
                for (int64_t i = 0; i < d_in; ++i) acc += Xd[m * d_in + i] * W_hat[o * d_in + i];
                Y[m * d_out + o] = acc;
            }
    }
    free(W_hat);
    free(Xd);
    return rc;
}

/* The same definition at chosen outputs only (layers too large to multiply whole). */
int pdelta_linear_group_ref_at(const uint16_t* X, const uint16_t* W_b, const uint32_t* B_packed,
                               const uint16_t* v, int64_t group, int64_t v_rows, int64_t M,
                               int64_t d_out, int64_t d_in, int x_dtype, int64_t n,
                               const int64_t* m_idx, const int64_t* o_idx, double* y)
{
    if (!X || !W_b || !B_packed || !v || !y || !m_idx || !o_idx) return REF_EINVAL;
    if (M <= 0 || n < 0 || !group_args_ok(d_out, d_in, group, v_rows)) return REF_EINVAL;
    int64_t wpr = words_per_row(d_in);
    for (int64_t s = 0; s < n; ++s)
        if (m_idx[s] < 0 || m_idx[s] >= M || o_idx[s] < 0 || o_idx[s] >= d_out) return REF_EINVAL;
#pragma omp parallel for schedule(static)
    for (int64_t s = 0; s < n; ++s) {
        int64_t m = m_idx[s], o = o_idx[s];
        double acc = 0.0;
        for (int64_t i = 0; i < d_in; ++i) {
            double b = ((B_packed[o * wpr + i / 32] >> (i % 32)) & 1u) ? 1.0 : -1.0;
            double w_hat = pdelta_ref_decode(W_b[o * d_in + i], x_dtype) +
                           group_scale(v, o, i, d_in, group, v_rows) * b;
            acc += pdelta_ref_decode(X[m * d_in + i], x_dtype) * w_hat;
        }
        y[s] = acc;
    }
    return REF_OK;
}

/* Number of threads the parallel loops above will use (for the bench's "cores" field). */
int pdelta_ref_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

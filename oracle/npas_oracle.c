/*
 * CPU oracle for inference through layers pruned with NPAS's fine-grained
 * structured schemes (paper section 3: block-based pruning for FC layers,
 * block-punched pruning for CONV layers; section 2.1: pattern-based pruning
 * with kernel removal).
 *
 * THIS IS TEST INFRASTRUCTURE.  It exists to check the HIP library, and only
 * the test-suite, the smoke check and the benchmark's CPU-baseline leg may call
 * it.  It shares no code with the HIP library and is never a fallback for it.
 *
 * Pruning sets weights to zero (section 2.1), so a pruned layer computes exactly
 * the masked-dense result.  Every function below is therefore the plain
 * definition: apply the mask, then a direct nested-loop convolution / matrix
 * product in double precision.  No blocking, no reordering, no fusion.
 *
 * Layouts: activations NHWC (n, y, x, c), weights W[F][C][KH][KW] as in the
 * 4-D tensor of Fig. 1, masks uint8 of the same shape with 1 = kept.
 * Cross-correlation (no kernel flip), zero padding.
 *
 * Pins (tests marked "not gpu"): against a float64 library convolution, a
 * separately written im2col product on tiny shapes, closed forms (all-ones,
 * unit impulse, rate 1, everything pruned), and scheme invariants.  The paper
 * prints no worked numeric example, so no golden values from the paper exist.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_OK = 0, ORACLE_E_ARG = -1, ORACLE_E_MASK = -2 };
enum { ACT_NONE = 0, ACT_RELU = 1, ACT_RELU6 = 2, ACT_HARDSWISH = 3 };

/* Activations of the paper's networks: ReLU / ReLU6, and hard-swish, which Phase 1 of the
 * framework puts in place of swish (section 5.1):  hswish(v) = v * min(max(v + 3, 0), 6) / 6. */
static double activate(double v, int act)
{
    if (act == ACT_RELU)  return v > 0.0 ? v : 0.0;
    if (act == ACT_RELU6) return v < 0.0 ? 0.0 : (v > 6.0 ? 6.0 : v);
    if (act == ACT_HARDSWISH) {
        double t = v + 3.0;
        t = t < 0.0 ? 0.0 : (t > 6.0 ? 6.0 : t);
        return v * t / 6.0;
    }
    return v;
}

/* ---------------------------------------------------------------------------
 * Rounding of a real number to a binary floating-point storage format with
 * `mant` significand bits (implicit one included), minimum normal exponent
 * `emin` and largest finite value `maxfinite`: round to nearest, ties to even,
 * gradual underflow.  bf16: mant 8, emin -126; fp16: mant 11, emin -14;
 * fp32: mant 24, emin -126.
 * ------------------------------------------------------------------------- */
static double round_to_format(double x, int mant, int emin, double maxfinite)
{
    if (x == 0.0 || isnan(x) || isinf(x)) return x;
    int e;
    (void)frexp(x, &e);                 /* |x| = m * 2^e, m in [0.5, 1) */
    int q = e - mant;                   /* exponent of the last kept bit */
    if (q < emin + 1 - mant) q = emin + 1 - mant;   /* subnormal quantum */
    double r = ldexp(nearbyint(ldexp(x, -q)), q);   /* nearbyint: ties to even */
    if (fabs(r) > maxfinite) r = x > 0 ? INFINITY : -INFINITY;
    return r;
}

double oracle_round_bf16(double x) { return round_to_format(x, 8, -126, 3.3895313892515355e38); }
double oracle_round_f16(double x)  { return round_to_format(x, 11, -14, 65504.0); }
double oracle_round_f32(double x)  { return (double)(float)x; }

/* dtype: 0 = fp32, 1 = bf16, 2 = fp16 */
void oracle_round_array(const double *in, double *out, size_t n, int dtype)
{
    for (size_t i = 0; i < n; ++i)
        out[i] = dtype == 1 ? oracle_round_bf16(in[i]) : dtype == 2 ? oracle_round_f16(in[i])
                                                                    : oracle_round_f32(in[i]);
}

/* ---------------------------------------------------------------------------
 * Scheme validators (what a legal mask is).
 * ------------------------------------------------------------------------- */

/* Block-punched (section 3): the tensor is cut into blocks of Bf consecutive
 * filters x Bc consecutive channels; a punched (channel, kh, kw) location is
 * punched in every filter of its block.  Equivalently the mask does not depend
 * on the filter inside a filter group.  Returns 0 if legal. */
int oracle_validate_block_punched(const uint8_t *mask, int F, int C, int KH, int KW, int Bf, int Bc)
{
    if (!mask || F <= 0 || C <= 0 || KH <= 0 || KW <= 0 || Bf <= 0 || Bc <= 0) return ORACLE_E_ARG;
    size_t per_filter = (size_t)C * KH * KW;
    for (int f = 0; f < F; ++f) {
        int lead = (f / Bf) * Bf;       /* first filter of this filter's group */
        for (size_t p = 0; p < per_filter; ++p) {
            uint8_t a = mask[(size_t)f * per_filter + p], b = mask[(size_t)lead * per_filter + p];
            if (a > 1) return ORACLE_E_MASK;
            if (a != b) return ORACLE_E_MASK;
        }
    }
    return ORACLE_OK;
}

/* Block-based (section 3): the OUT x IN matrix is cut into Br x Bcol blocks and
 * whole columns and/or whole rows are pruned inside each block, i.e. inside a
 * block mask[r][c] = rowkeep[r] AND colkeep[c].  Returns 0 if legal. */
int oracle_validate_fc_block(const uint8_t *mask, int OUT, int IN, int Br, int Bcol)
{
    if (!mask || OUT <= 0 || IN <= 0 || Br <= 0 || Bcol <= 0) return ORACLE_E_ARG;
    for (int r0 = 0; r0 < OUT; r0 += Br)
        for (int c0 = 0; c0 < IN; c0 += Bcol) {
            int r1 = r0 + Br < OUT ? r0 + Br : OUT, c1 = c0 + Bcol < IN ? c0 + Bcol : IN;
            for (int r = r0; r < r1; ++r)
                for (int c = c0; c < c1; ++c) {
                    if (mask[(size_t)r * IN + c] > 1) return ORACLE_E_MASK;
                    int rowkeep = 0, colkeep = 0;
                    for (int cc = c0; cc < c1; ++cc) rowkeep |= mask[(size_t)r * IN + cc];
                    for (int rr = r0; rr < r1; ++rr) colkeep |= mask[(size_t)rr * IN + c];
                    if (mask[(size_t)r * IN + c] != (rowkeep & colkeep)) return ORACLE_E_MASK;
                }
        }
    return ORACLE_OK;
}

/* Pattern-based + connectivity (section 2.1): every 3x3 kernel (f, c) either
 * equals one pattern of the library (uint8 [n_pat][9], tap order kh*3+kw) or is
 * removed entirely.  Writes pat_id[f][c] = smallest matching library index, or
 * 255 for a removed kernel.  Returns 0 if legal. */
int oracle_validate_pattern(const uint8_t *mask, int F, int C, const uint8_t *library, int n_pat,
                            uint8_t *pat_id)
{
    if (!mask || !library || F <= 0 || C <= 0 || n_pat <= 0 || n_pat > 255) return ORACLE_E_ARG;
    for (int f = 0; f < F; ++f)
        for (int c = 0; c < C; ++c) {
            const uint8_t *k = mask + ((size_t)f * C + c) * 9;
            int nz = 0, found = 255;
            for (int t = 0; t < 9; ++t) { if (k[t] > 1) return ORACLE_E_MASK; nz += k[t]; }
            if (nz != 0) {
                for (int p = n_pat - 1; p >= 0; --p)
                    if (memcmp(k, library + (size_t)p * 9, 9) == 0) found = p;
                if (found == 255) return ORACLE_E_MASK;
            }
            if (pat_id) pat_id[(size_t)f * C + c] = (uint8_t)found;
        }
    return ORACLE_OK;
}

/* ---------------------------------------------------------------------------
 * Canonical compact form of a block-punched / block-based layer, written from
 * the format's prose definition (independently of the library's packer):
 *   filter group g = filters [g*Bf, (g+1)*Bf);
 *   k_pos lists, per group, the kept positions as (kh*KW + kw)*C + c in
 *   ascending order; grp_ptr[g] is the prefix sum of the list lengths;
 *   w_compact[(grp_ptr[g] + k)*Bf + j] = W[g*Bf + j] at position k, multiplied by
 *   the mask (a row-pruned FC weight becomes +0), +0 for j past the last filter.
 * A position is listed if ANY filter of the group keeps it.
 * Call with k_pos == NULL to get the total list length in *total.
 * ------------------------------------------------------------------------- */
int oracle_pack_block_punched(const double *W, const uint8_t *mask, int F, int C, int KH, int KW,
                              int Bf, int32_t *grp_ptr, int32_t *k_pos, double *w_compact,
                              int64_t *total)
{
    if (!W || !mask || F <= 0 || C <= 0 || KH <= 0 || KW <= 0 || Bf <= 0) return ORACLE_E_ARG;
    int G = (F + Bf - 1) / Bf;
    int64_t n = 0;
    for (int g = 0; g < G; ++g) {
        if (grp_ptr) grp_ptr[g] = (int32_t)n;
        for (int kh = 0; kh < KH; ++kh)
            for (int kw = 0; kw < KW; ++kw)
                for (int c = 0; c < C; ++c) {
                    int any = 0;
                    for (int j = 0; j < Bf && g * Bf + j < F; ++j)
                        any |= mask[(((size_t)(g * Bf + j) * C + c) * KH + kh) * KW + kw];
                    if (!any) continue;
                    if (k_pos) {
                        k_pos[n] = (kh * KW + kw) * C + c;
                        for (int j = 0; j < Bf; ++j) {
                            int f = g * Bf + j;
                            double v = 0.0;
                            if (f < F) {
                                size_t idx = (((size_t)f * C + c) * KH + kh) * KW + kw;
                                v = mask[idx] ? W[idx] : 0.0;
                            }
                            w_compact[(size_t)n * Bf + j] = v;
                        }
                    }
                    ++n;
                }
    }
    if (grp_ptr) grp_ptr[G] = (int32_t)n;
    if (total) *total = n;
    return ORACLE_OK;
}

/* Canonical compact form of a pattern-pruned layer: pat_id as written by
 * oracle_validate_pattern, and w4[f][c][j] = the j-th kept weight of kernel
 * (f, c) in ascending tap order (+0 for a removed kernel). */
int oracle_pack_pattern(const double *W, const uint8_t *mask, int F, int C, double *w4)
{
    if (!W || !mask || !w4) return ORACLE_E_ARG;
    for (size_t k = 0; k < (size_t)F * C; ++k) {
        int j = 0;
        for (int s = 0; s < 4; ++s) w4[k * 4 + s] = 0.0;
        for (int t = 0; t < 9; ++t)
            if (mask[k * 9 + t]) {
                if (j >= 4) return ORACLE_E_MASK;
                w4[k * 4 + j++] = W[k * 9 + t];
            }
    }
    return ORACLE_OK;
}

/* ---------------------------------------------------------------------------
 * Masked dense convolution, the definition:
 *   Y[n,y,x,f] = act( bias[f] + sum_{c,kh,kw} (W*mask)[f,c,kh,kw] * X[n, y*s+kh-p, x*s+kw-p, c]
 *                     + residual[n,y,x,f] )
 * with out-of-range input taken as 0.  Ho = (H + 2p - KH)/s + 1 (floor).
 * bias and residual may be NULL.  The only shortcut is skipping a term whose
 * masked weight is exactly zero, which cannot change the sum.
 * ------------------------------------------------------------------------- */
int oracle_conv2d_masked(const double *X, const double *W, const uint8_t *mask, const double *bias,
                         const double *residual, int N, int H, int Wd, int C, int F, int KH, int KW,
                         int stride, int pad, int act, double *Y)
{
    if (!X || !W || !mask || !Y || N <= 0 || H <= 0 || Wd <= 0 || C <= 0 || F <= 0 || KH <= 0 ||
        KW <= 0 || stride <= 0 || pad < 0)
        return ORACLE_E_ARG;
    int Ho = (H + 2 * pad - KH) / stride + 1, Wo = (Wd + 2 * pad - KW) / stride + 1;
    if (Ho <= 0 || Wo <= 0) return ORACLE_E_ARG;
    size_t nw = (size_t)F * C * KH * KW;
    double *Wm = (double *)malloc(nw * sizeof(double));
    if (!Wm) return ORACLE_E_ARG;
    for (size_t i = 0; i < nw; ++i) Wm[i] = mask[i] ? W[i] : 0.0;   /* W (.) mask */
    long rows = (long)N * Ho;
#pragma omp parallel for schedule(dynamic, 1)
    for (long r = 0; r < rows; ++r) {
        int n = (int)(r / Ho), y = (int)(r % Ho);
        for (int x = 0; x < Wo; ++x)
            for (int f = 0; f < F; ++f) {
                double acc = bias ? bias[f] : 0.0;
                for (int c = 0; c < C; ++c)
                    for (int kh = 0; kh < KH; ++kh) {
                        int iy = y * stride + kh - pad;
                        if (iy < 0 || iy >= H) continue;
                        for (int kw = 0; kw < KW; ++kw) {
                            int ix = x * stride + kw - pad;
                            if (ix < 0 || ix >= Wd) continue;
                            double w = Wm[(((size_t)f * C + c) * KH + kh) * KW + kw];
                            if (w == 0.0) continue;
                            acc += w * X[(((size_t)n * H + iy) * Wd + ix) * C + c];
                        }
                    }
                size_t o = (((size_t)n * Ho + y) * Wo + x) * F + f;
                if (residual) acc += residual[o];
                Y[o] = activate(acc, act);
            }
    }
    free(Wm);
    return ORACLE_OK;
}

/* Masked dense fully-connected layer: Y[b,o] = act(bias[o] + sum_i (W*mask)[o,i] X[b,i]). */
int oracle_fc_masked(const double *X, const double *W, const uint8_t *mask, const double *bias,
                     int B, int IN, int OUT, int act, double *Y)
{
    if (!X || !W || !mask || !Y || B <= 0 || IN <= 0 || OUT <= 0) return ORACLE_E_ARG;
#pragma omp parallel for schedule(static)
    for (int b = 0; b < B; ++b)
        for (int o = 0; o < OUT; ++o) {
            double acc = bias ? bias[o] : 0.0;
            for (int i = 0; i < IN; ++i) {
                double w = mask[(size_t)o * IN + i] ? W[(size_t)o * IN + i] : 0.0;
                if (w == 0.0) continue;
                acc += w * X[(size_t)b * IN + i];
            }
            Y[(size_t)b * OUT + o] = activate(acc, act);
        }
    return ORACLE_OK;
}

/* Pattern + connectivity 3x3 convolution computed from the compact form, the
 * way the scheme describes the layer: for every kept kernel (f, c), its four
 * weights sit on the taps of its library pattern.
 *   Y[n,y,x,f] = act(bias[f] + sum_{c alive} sum_{j<4} w4[f,c,j] * X[n, y*s+kh_j-p, x*s+kw_j-p, c]) */
int oracle_conv2d_pattern(const double *X, const double *w4, const uint8_t *pat_id,
                          const uint8_t *library, int n_pat, const double *bias, int N, int H, int Wd,
                          int C, int F, int stride, int pad, int act, double *Y)
{
    if (!X || !w4 || !pat_id || !library || !Y || stride <= 0 || pad < 0) return ORACLE_E_ARG;
    int Ho = (H + 2 * pad - 3) / stride + 1, Wo = (Wd + 2 * pad - 3) / stride + 1;
    if (Ho <= 0 || Wo <= 0) return ORACLE_E_ARG;
    long rows = (long)N * Ho;
#pragma omp parallel for schedule(dynamic, 1)
    for (long r = 0; r < rows; ++r) {
        int n = (int)(r / Ho), y = (int)(r % Ho);
        for (int x = 0; x < Wo; ++x)
            for (int f = 0; f < F; ++f) {
                double acc = bias ? bias[f] : 0.0;
                for (int c = 0; c < C; ++c) {
                    int p = pat_id[(size_t)f * C + c];
                    if (p == 255) continue;             /* kernel removed */
                    if (p >= n_pat) continue;
                    int j = 0;
                    for (int t = 0; t < 9; ++t) {
                        if (!library[(size_t)p * 9 + t]) continue;
                        double w = w4[((size_t)f * C + c) * 4 + j];
                        ++j;
                        int iy = y * stride + t / 3 - pad, ix = x * stride + t % 3 - pad;
                        if (iy < 0 || iy >= H || ix < 0 || ix >= Wd) continue;
                        acc += w * X[(((size_t)n * H + iy) * Wd + ix) * C + c];
                    }
                }
                Y[(((size_t)n * Ho + y) * Wo + x) * F + f] = activate(acc, act);
            }
    }
    return ORACLE_OK;
}

/* ---------------------------------------------------------------------------
 * Depthwise 3x3 convolution (the "3x3 DW" of the search space's cascades,
 * section 5.1.1): every channel is filtered by its own 3x3 kernel, padding 1,
 *   Y[n,y,x,c] = act( bias[c] + sum_{kh,kw} W[c,kh,kw] * X[n, y*s+kh-1, x*s+kw-1, c]
 *                     + residual[n,y,x,c] )
 * out-of-range input taken as 0, Ho = (H + 2 - 3)/s + 1 (floor).  bias and
 * residual may be NULL.
 * ------------------------------------------------------------------------- */
int oracle_dwconv3x3(const double *X, const double *W, const double *bias, const double *residual,
                     int N, int H, int Wd, int C, int stride, int act, double *Y)
{
    if (!X || !W || !Y || N <= 0 || H <= 0 || Wd <= 0 || C <= 0 || stride <= 0) return ORACLE_E_ARG;
    int Ho = (H + 2 - 3) / stride + 1, Wo = (Wd + 2 - 3) / stride + 1;
    if (Ho <= 0 || Wo <= 0) return ORACLE_E_ARG;
    for (int n = 0; n < N; ++n)
        for (int y = 0; y < Ho; ++y)
            for (int x = 0; x < Wo; ++x)
                for (int c = 0; c < C; ++c) {
                    double acc = bias ? bias[c] : 0.0;
                    for (int kh = 0; kh < 3; ++kh)
                        for (int kw = 0; kw < 3; ++kw) {
                            int iy = y * stride + kh - 1, ix = x * stride + kw - 1;
                            if (iy < 0 || iy >= H || ix < 0 || ix >= Wd) continue;
                            acc += W[((size_t)c * 3 + kh) * 3 + kw] * X[(((size_t)n * H + iy) * Wd + ix) * C + c];
                        }
                    size_t o = (((size_t)n * Ho + y) * Wo + x) * C + c;
                    if (residual) acc += residual[o];
                    Y[o] = activate(acc, act);
                }
    return ORACLE_OK;
}

/* 3x3 stride-2 max pooling with padding 1 (padded cells never win). */
int oracle_maxpool3x3s2(const double *X, int N, int H, int Wd, int C, double *Y)
{
    if (!X || !Y) return ORACLE_E_ARG;
    int Ho = (H + 2 - 3) / 2 + 1, Wo = (Wd + 2 - 3) / 2 + 1;
    for (int n = 0; n < N; ++n)
        for (int y = 0; y < Ho; ++y)
            for (int x = 0; x < Wo; ++x)
                for (int c = 0; c < C; ++c) {
                    double m = -INFINITY;
                    for (int kh = 0; kh < 3; ++kh)
                        for (int kw = 0; kw < 3; ++kw) {
                            int iy = 2 * y + kh - 1, ix = 2 * x + kw - 1;
                            if (iy < 0 || iy >= H || ix < 0 || ix >= Wd) continue;
                            double v = X[(((size_t)n * H + iy) * Wd + ix) * C + c];
                            if (v > m) m = v;
                        }
                    Y[(((size_t)n * Ho + y) * Wo + x) * C + c] = m;
                }
    return ORACLE_OK;
}

/* Global average pooling: Y[n,c] = mean over (y,x) of X[n,y,x,c]. */
int oracle_global_avgpool(const double *X, int N, int H, int Wd, int C, double *Y)
{
    if (!X || !Y) return ORACLE_E_ARG;
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c) {
            double s = 0.0;
            for (int p = 0; p < H * Wd; ++p) s += X[((size_t)n * H * Wd + p) * C + c];
            Y[(size_t)n * C + c] = s / (double)(H * Wd);
        }
    return ORACLE_OK;
}

int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}

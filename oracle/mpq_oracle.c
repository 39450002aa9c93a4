/*
 * mpq_oracle.c -- plain CPU definition of the mixed-precision layers.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement of what the
 * quantized (int8 / int16) and fp16 convolution, fully-connected, max-pool, quantize /
 * dequantize and expert-routing steps compute.  Only tests, the smoke check and the
 * cpu_baseline leg of the benchmark may call it; the GPU library shares no code with it.
 *
 * Conventions
 *   - logical layouts follow the paper's framework (Caffe): activations N,C,H,W; weights
 *     K,C/groups,R,S; FC weights N_out,K_in (row = one output feature);
 *   - quantized values travel as int32 arrays whose entries lie in the storage type's range,
 *     so one routine serves int8 and int16; accumulators are int64 (the paper's Acctype for
 *     16-bit storage, section "Caffe Device Abstracted Host Code"; for 8-bit storage every
 *     value provably fits int32, so int64 holds the same number);
 *   - floating point is fp64 throughout; fp16 enters only through orc_round_fp16().
 *   - OpenMP pragmas spread the outermost independent loop over host cores; there is no
 *     blocking, packing, or reordering of the inner sums.
 *
 * Parity pins: see tests/test_oracle_*.py (closed forms, identity kernels, big-integer
 * re-evaluation, bracket against exact rational arithmetic, numpy library routines).
 * The requantization rounding itself has no worked number printed in the paper; the quantized
 * ReLU listing (section "Emitted OpenCL Runtime Code") is the only statement of it: that choice
 * is "parity unpinned" by printed values and pinned only by that listing's text.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int orc_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void orc_set_threads(int n) {
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ------------------------------------------------------------------------------------------
 * Parameter estimation (section "Parameter Estimation", its three equations):
 *   s  = (fmax - fmin) / (imax - imin)
 *   i0 = min(max(round(imin - fmin / s), imin), imax)
 *   i1 = 1 / s + i0
 * Evaluated in full (double) precision; the caller casts.
 * ---------------------------------------------------------------------------------------- */
void orc_estimate_params(double fmin, double fmax, int64_t imin, int64_t imax,
                         double *s, int64_t *i0, double *i1) {
    double scale = (fmax - fmin) / (double)(imax - imin);
    double z = nearbyint((double)imin - fmin / scale);
    if (z < (double)imin) z = (double)imin;
    if (z > (double)imax) z = (double)imax;
    *s = scale;
    *i0 = (int64_t)z;
    *i1 = 1.0 / scale + z;
}

/* ------------------------------------------------------------------------------------------
 * Float -> quantized: q = clamp(rne(r / s) + z, qmin, qmax).  The quotient is an IEEE double
 * division of the widened fp32 operands, rounded to nearest with ties to even.  NaN maps to
 * the zero-point, infinities saturate.  (Section "Quantization Integration to Caffe": the
 * quantizer converts between types; the affine map r = s (q - z) is the one implied by the
 * quantized multiplication rule in section "Quantized Operations".)
 * ---------------------------------------------------------------------------------------- */
void orc_quantize(const float *r, size_t count, float scale, int32_t zero,
                  int32_t qmin, int32_t qmax, int32_t *q) {
    for (size_t i = 0; i < count; ++i) {
        double v = (double)r[i];
        int64_t out;
        if (isnan(v)) {
            out = zero;
        } else {
            double t = nearbyint(v / (double)scale); /* default rounding mode: ties-to-even */
            if (t > 4.0e9) t = 4.0e9;                 /* keeps the int64 cast defined for +-inf */
            if (t < -4.0e9) t = -4.0e9;
            out = (int64_t)t + (int64_t)zero;
        }
        if (out < qmin) out = qmin;
        if (out > qmax) out = qmax;
        q[i] = (int32_t)out;
    }
}

/* Quantized -> float: r = (float)(q - z) * s, one fp32 multiplication. */
void orc_dequantize(const int32_t *q, size_t count, float scale, int32_t zero, float *r) {
    for (size_t i = 0; i < count; ++i) {
        float d = (float)(q[i] - zero);
        r[i] = d * scale;
    }
}

/* ------------------------------------------------------------------------------------------
 * Integer rescale constants (section "Quantized Operations", the (x * m) >> h equation, and the
 * shift_bits expression in the listing "Caffe device abstracted launch code"):
 *   M = s_a s_b / s_c = M0 * 2^e with M0 in [0.5, 1);
 *   mult = round(M0 * 2^sb)  (sb = 31 for 8-bit storage, 15 for 16-bit storage);
 *   shift = -e, so that (t * mult / 2^sb) >> shift ~= t * M.
 * If rounding pushes mult to 2^sb it is halved and e grows by one.
 * Returns 0 on success, 1 if M is not a positive finite number.
 * ---------------------------------------------------------------------------------------- */
int orc_scale_quant_vals(float s_a, float s_b, float s_c, int sb, int64_t *mult, int *shift) {
    double M = (double)s_a * (double)s_b / (double)s_c;
    if (!(M > 0.0) || isinf(M)) return 1;
    int e;
    double M0 = frexp(M, &e);
    int64_t m = llrint(ldexp(M0, sb));
    if (m == ((int64_t)1 << sb)) {
        m >>= 1;
        e += 1;
    }
    *mult = m;
    *shift = -e;
    return 0;
}

/* ------------------------------------------------------------------------------------------
 * Requantize one accumulator (the integer branch of the quantized ReLU listing, applied to
 * every operator):
 *   y = (t * mult) / 2^sb        C integer division: truncates toward zero
 *   y = y >> shift  (shift >= 0, arithmetic: floor)   or   y * 2^(-shift)  (shift < 0)
 *   q = min(max(y + z_out, lo), hi)
 * ReLU is the raised lower clamp lo = max(qmin, z_out): both rescale stages are monotone and
 * send 0 to 0, so clamping after is the same as max(t, 0) before.
 * ---------------------------------------------------------------------------------------- */
static int64_t floor_div_pow2(int64_t v, int sh) {
    int64_t d = (int64_t)1 << sh;
    int64_t q = v / d;
    if ((v % d) != 0 && v < 0) q -= 1;
    return q;
}

int64_t orc_requant_one(int64_t t, int64_t mult, int sb, int shift,
                        int64_t z_out, int64_t lo, int64_t hi) {
    int64_t y = (t * mult) / ((int64_t)1 << sb);
    if (shift >= 0) {
        y = floor_div_pow2(y, shift);
    } else {
        y = y * ((int64_t)1 << (-shift));
    }
    y += z_out;
    if (y < lo) y = lo;
    if (y > hi) y = hi;
    return y;
}

/* Round-to-nearest variant of the rescale (the paper leaves the rounding of the rescale to the
 * operator, section "Quantized Operations"; this is the single-rounding alternative to the
 * listing's truncate-then-floor): with s = sb + shift,
 *   y = floor((t * mult + 2^(s-1)) / 2^s)     (nearest integer to t * mult / 2^s, halves upward)
 *   y = t * mult * 2^(-s)                     for s <= 0 (exact)
 * then + z_out and the clamp as above. */
int64_t orc_requant_nearest_one(int64_t t, int64_t mult, int sb, int shift,
                                int64_t z_out, int64_t lo, int64_t hi) {
    __int128 p = (__int128)t * (__int128)mult;
    int s = sb + shift;
    __int128 y;
    if (s <= 0) {
        y = p * ((__int128)1 << (-s));
    } else {
        __int128 d = (__int128)1 << s;
        __int128 v = p + (d >> 1);
        y = v / d;
        if ((v % d) != 0 && v < 0) y -= 1;
    }
    y += z_out;
    if (y < lo) y = lo;
    if (y > hi) y = hi;
    return (int64_t)y;
}

void orc_requant_nearest(const int64_t *t, size_t count, int64_t mult, int sb, int shift,
                         int32_t z_out, int32_t qmin, int32_t qmax, int relu, int32_t *q) {
    int64_t lo = qmin;
    if (relu && z_out > qmin) lo = z_out;
    for (size_t i = 0; i < count; ++i) {
        q[i] = (int32_t)orc_requant_nearest_one(t[i], mult, sb, shift, z_out, lo, qmax);
    }
}

void orc_requant(const int64_t *t, size_t count, int64_t mult, int sb, int shift,
                 int32_t z_out, int32_t qmin, int32_t qmax, int relu, int32_t *q) {
    int64_t lo = qmin;
    if (relu && z_out > qmin) lo = z_out;
    for (size_t i = 0; i < count; ++i) {
        q[i] = (int32_t)orc_requant_one(t[i], mult, sb, shift, z_out, lo, qmax);
    }
}

/* ------------------------------------------------------------------------------------------
 * Quantized convolution accumulator, differences first (first quantized-multiply equation of
 * section "Quantized Operations"):
 *   t[n,k,p,q] = bias[k] + sum_{c,r,s} (x[n, g Cg + c, p st - pad + r, q st - pad + s] - z_x)
 *                                     * (w[k, c, r, s] - z_w)
 * Cross-correlation (no kernel flip).  Taps outside the image contribute nothing.  Output
 * channel k belongs to group g = k / (K / groups) and sees input channels [g Cg, (g+1) Cg).
 * bias may be NULL.
 * ---------------------------------------------------------------------------------------- */
void orc_conv2d_acc(const int32_t *x, int N, int C, int H, int W, int32_t z_x,
                    const int32_t *w, int K, int R, int S, int32_t z_w,
                    const int64_t *bias,
                    int stride_h, int stride_w, int pad_h, int pad_w, int groups,
                    int64_t *t) {
    int Cg = C / groups, Kg = K / groups;
    int P = (H + 2 * pad_h - R) / stride_h + 1;
    int Q = (W + 2 * pad_w - S) / stride_w + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int k = 0; k < K; ++k) {
            int g = k / Kg;
            for (int p = 0; p < P; ++p) {
                for (int q = 0; q < Q; ++q) {
                    int64_t acc = bias ? bias[k] : 0;
                    for (int c = 0; c < Cg; ++c) {
                        for (int r = 0; r < R; ++r) {
                            int h = p * stride_h - pad_h + r;
                            if (h < 0 || h >= H) continue;
                            for (int s = 0; s < S; ++s) {
                                int ww = q * stride_w - pad_w + s;
                                if (ww < 0 || ww >= W) continue;
                                int64_t a = (int64_t)x[(((size_t)n * C + g * Cg + c) * H + h) * W + ww] - z_x;
                                int64_t b = (int64_t)w[(((size_t)k * Cg + c) * R + r) * S + s] - z_w;
                                acc += a * b;
                            }
                        }
                    }
                    t[(((size_t)n * K + k) * P + p) * Q + q] = acc;
                }
            }
        }
    }
}

/* ------------------------------------------------------------------------------------------
 * The same accumulator through the expanded form (second quantized-multiply equation of
 * section "Quantized Operations"): products of the raw codes, then the three zero-point
 * corrections  - z_x sum(w) - z_w sum(x) + count z_x z_w, all sums over the in-image taps.
 * A separate routine on purpose: it must agree with orc_conv2d_acc bit for bit.
 * ---------------------------------------------------------------------------------------- */
void orc_conv2d_acc_expanded(const int32_t *x, int N, int C, int H, int W, int32_t z_x,
                             const int32_t *w, int K, int R, int S, int32_t z_w,
                             const int64_t *bias,
                             int stride_h, int stride_w, int pad_h, int pad_w, int groups,
                             int64_t *t) {
    int Cg = C / groups, Kg = K / groups;
    int P = (H + 2 * pad_h - R) / stride_h + 1;
    int Q = (W + 2 * pad_w - S) / stride_w + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int k = 0; k < K; ++k) {
            int g = k / Kg;
            for (int p = 0; p < P; ++p) {
                for (int q = 0; q < Q; ++q) {
                    int64_t sum_ab = 0, sum_a = 0, sum_b = 0, taps = 0;
                    for (int c = 0; c < Cg; ++c) {
                        for (int r = 0; r < R; ++r) {
                            int h = p * stride_h - pad_h + r;
                            if (h < 0 || h >= H) continue;
                            for (int s = 0; s < S; ++s) {
                                int ww = q * stride_w - pad_w + s;
                                if (ww < 0 || ww >= W) continue;
                                int64_t a = x[(((size_t)n * C + g * Cg + c) * H + h) * W + ww];
                                int64_t b = w[(((size_t)k * Cg + c) * R + r) * S + s];
                                sum_ab += a * b;
                                sum_a += a;
                                sum_b += b;
                                taps += 1;
                            }
                        }
                    }
                    int64_t acc = sum_ab - (int64_t)z_x * sum_b - (int64_t)z_w * sum_a
                                  + taps * (int64_t)z_x * (int64_t)z_w;
                    t[(((size_t)n * K + k) * P + p) * Q + q] = acc + (bias ? bias[k] : 0);
                }
            }
        }
    }
}

/* ------------------------------------------------------------------------------------------
 * im2col: col[n, p, q, (c, r, s)] = x[n, g Cg + c, p st - pad + r, q st - pad + s], with the
 * zero-point z_x written where the tap leaves the image (so that (col - z_x) is 0 there).
 * One group at a time (g selects it).  Used with orc_gemm_acc as the second convolution path
 * the paper names (section "Library Multiplexer": im2col + GEMM next to direct convolution).
 * ---------------------------------------------------------------------------------------- */
void orc_im2col(const int32_t *x, int N, int C, int H, int W, int32_t z_x,
                int R, int S, int stride_h, int stride_w, int pad_h, int pad_w,
                int groups, int g, int32_t *col) {
    int Cg = C / groups;
    int P = (H + 2 * pad_h - R) / stride_h + 1;
    int Q = (W + 2 * pad_w - S) / stride_w + 1;
    size_t Kc = (size_t)Cg * R * S;
    for (int n = 0; n < N; ++n)
        for (int p = 0; p < P; ++p)
            for (int q = 0; q < Q; ++q) {
                int32_t *row = col + (((size_t)n * P + p) * Q + q) * Kc;
                for (int c = 0; c < Cg; ++c)
                    for (int r = 0; r < R; ++r)
                        for (int s = 0; s < S; ++s) {
                            int h = p * stride_h - pad_h + r;
                            int ww = q * stride_w - pad_w + s;
                            int32_t v = z_x;
                            if (h >= 0 && h < H && ww >= 0 && ww < W)
                                v = x[(((size_t)n * C + g * Cg + c) * H + h) * W + ww];
                            row[((size_t)c * R + r) * S + s] = v;
                        }
            }
}

/* ------------------------------------------------------------------------------------------
 * Fully-connected accumulator: t[m, n] = bias[n] + sum_k (x[m,k] - z_x)(w[n,k] - z_w).
 * ---------------------------------------------------------------------------------------- */
void orc_gemm_acc(const int32_t *x, int M, int K, int32_t z_x,
                  const int32_t *w, int N, int32_t z_w,
                  const int64_t *bias, int64_t *t) {
#pragma omp parallel for collapse(2) schedule(static)
    for (int m = 0; m < M; ++m) {
        for (int n = 0; n < N; ++n) {
            int64_t acc = bias ? bias[n] : 0;
            for (int k = 0; k < K; ++k) {
                int64_t a = (int64_t)x[(size_t)m * K + k] - z_x;
                int64_t b = (int64_t)w[(size_t)n * K + k] - z_w;
                acc += a * b;
            }
            t[(size_t)m * N + n] = acc;
        }
    }
}

/* Max-pool, square window k, stride st, no padding, floor output size.  Integer max. */
void orc_maxpool_i32(const int32_t *x, int N, int C, int H, int W, int k, int st, int32_t *y) {
    int P = (H - k) / st + 1, Q = (W - k) / st + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    const int32_t *plane = x + ((size_t)n * C + c) * H * W;
                    int32_t m = plane[(size_t)(p * st) * W + q * st];
                    for (int r = 0; r < k; ++r)
                        for (int s = 0; s < k; ++s) {
                            int32_t v = plane[(size_t)(p * st + r) * W + q * st + s];
                            if (v > m) m = v;
                        }
                    y[(((size_t)n * C + c) * P + p) * Q + q] = m;
                }
}

/* ------------------------------------------------------------------------------------------
 * Floating-point reference layers in fp64: the value the fp16 path approximates.
 * Products and sums in double, in index order; bias added last; optional ReLU.
 * ---------------------------------------------------------------------------------------- */
void orc_conv2d_f64(const double *x, int N, int C, int H, int W,
                    const double *w, int K, int R, int S, const double *bias,
                    int stride_h, int stride_w, int pad_h, int pad_w, int groups, int relu,
                    double *y) {
    int Cg = C / groups, Kg = K / groups;
    int P = (H + 2 * pad_h - R) / stride_h + 1;
    int Q = (W + 2 * pad_w - S) / stride_w + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int k = 0; k < K; ++k) {
            int g = k / Kg;
            for (int p = 0; p < P; ++p) {
                for (int q = 0; q < Q; ++q) {
                    double acc = 0.0;
                    for (int c = 0; c < Cg; ++c) {
                        for (int r = 0; r < R; ++r) {
                            int h = p * stride_h - pad_h + r;
                            if (h < 0 || h >= H) continue;
                            for (int s = 0; s < S; ++s) {
                                int ww = q * stride_w - pad_w + s;
                                if (ww < 0 || ww >= W) continue;
                                acc += x[(((size_t)n * C + g * Cg + c) * H + h) * W + ww]
                                     * w[(((size_t)k * Cg + c) * R + r) * S + s];
                            }
                        }
                    }
                    if (bias) acc += bias[k];
                    if (relu && acc < 0.0) acc = 0.0;
                    y[(((size_t)n * K + k) * P + p) * Q + q] = acc;
                }
            }
        }
    }
}

void orc_gemm_f64(const double *x, int M, int K, const double *w, int N, const double *bias,
                  int relu, double *y) {
#pragma omp parallel for collapse(2) schedule(static)
    for (int m = 0; m < M; ++m) {
        for (int n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int k = 0; k < K; ++k) acc += x[(size_t)m * K + k] * w[(size_t)n * K + k];
            if (bias) acc += bias[n];
            if (relu && acc < 0.0) acc = 0.0;
            y[(size_t)m * N + n] = acc;
        }
    }
}

void orc_maxpool_f64(const double *x, int N, int C, int H, int W, int k, int st, double *y) {
    int P = (H - k) / st + 1, Q = (W - k) / st + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    const double *plane = x + ((size_t)n * C + c) * H * W;
                    double m = plane[(size_t)(p * st) * W + q * st];
                    for (int r = 0; r < k; ++r)
                        for (int s = 0; s < k; ++s) {
                            double v = plane[(size_t)(p * st + r) * W + q * st + s];
                            if (v > m) m = v;
                        }
                    y[(((size_t)n * C + c) * P + p) * Q + q] = m;
                }
}

/* ------------------------------------------------------------------------------------------
 * Round a double to the nearest IEEE binary16 value (ties to even), returned as a double.
 * binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits; normal range 2^-14 .. 65504,
 * subnormal spacing 2^-24; values that round above 65504 become infinity.
 * ---------------------------------------------------------------------------------------- */
double orc_round_fp16_one(double v) {
    if (isnan(v) || isinf(v) || v == 0.0) return v;
    double a = fabs(v);
    int e;
    (void)frexp(a, &e);            /* a = f * 2^e, f in [0.5, 1)  =>  a in [2^(e-1), 2^e) */
    int ulp_exp = (e - 1) - 10;    /* spacing of binary16 in that binade */
    if (ulp_exp < -24) ulp_exp = -24;
    double scaled = ldexp(a, -ulp_exp);        /* exact: power-of-two scaling */
    double r = ldexp(nearbyint(scaled), ulp_exp);
    if (r > 65504.0) r = INFINITY;
    return v < 0.0 ? -r : r;
}

void orc_round_fp16(const double *x, size_t count, double *y) {
    for (size_t i = 0; i < count; ++i) y[i] = orc_round_fp16_one(x[i]);
}

/* ------------------------------------------------------------------------------------------
 * Top-1 routing (section "Mixture of Experts": the gating selection picks, per sample, the
 * experts with the largest gating outputs; with one expert per sample its normalised
 * probability is 1).  Ties go to the lowest expert index.  counts[i] is the paper's c_i.
 * ---------------------------------------------------------------------------------------- */
void orc_route_top1(const double *logits, int B, int E, int32_t *expert, int32_t *counts) {
    for (int i = 0; i < E; ++i) counts[i] = 0;
    for (int b = 0; b < B; ++b) {
        int best = 0;
        for (int i = 1; i < E; ++i)
            if (logits[(size_t)b * E + i] > logits[(size_t)b * E + best]) best = i;
        expert[b] = best;
        counts[best] += 1;
    }
}

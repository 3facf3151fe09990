/*
 * CPU oracle for the T-MAN low-bit-weight x fp16-activation matmul (arxiv 2511.11248).
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing on the product path may call into this file; it exists so the
 * tests, the smoke check and the benchmark's cpu_baseline leg have an independent statement of what
 * the HIP kernels must compute.  It shares no code, header, table or helper with the HIP library.
 *
 * What it computes.  The method (bit-serial table lookup for decoding, table-based dequantization
 * feeding a matrix unit for prefill) reaches, up to rounding, exactly the result of dequantizing
 * the weights and multiplying.  So the main oracle is that definition written out in double
 * precision:
 *     Wd[m][k] = (q[m][k] - zero[m][k/group]) * scale[m][k/group]        Sec. 2.2, "Dequantization-
 *                                                                         based low-bit inference"
 *     Y[n][m]  = sum_{k ascending} x[n][k] * Wd[m][k]                    Sec. 4.1: weights (M,K),
 *                                                                         activations (N,K)
 * A second routine evaluates the bit-serial table-lookup form of Sec. 2.2 ("Bit-serial table
 * lookup") step by step in the paper's order -- one-bit decomposition, per-group-of-g activation
 * tables, lookup by weight bit pattern, shift and accumulate -- so tests can check the identity
 * between the two forms and bound the effect of 16-bit table entries (Sec. 5, VLUT16).
 *
 * Every function here is pinned by tests/test_oracle_pins.py against something other than itself
 * (brute force, closed forms, special cases, the paper's printed repack example).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* IEEE 754 binary16 -> double, exact (1 sign, 5 exponent bits with bias 15, 10 fraction bits). */
double tman_oracle_half_to_double(uint16_t h) {
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int f = h & 0x3ff;
    double v;
    if (e == 0) {
        v = ldexp((double)f, -24); /* zero and subnormals: f * 2^-24 */
    } else if (e == 31) {
        v = f ? NAN : INFINITY;
    } else {
        v = ldexp((double)(1024 + f), e - 25); /* (1 + f/1024) * 2^(e-15) */
    }
    return sign ? -v : v;
}

/* double -> binary16 with round-to-nearest-even, one rounding (used to model 16-bit table entries
 * and fp16 dequantized weights).  Overflow goes to infinity. */
uint16_t tman_oracle_double_to_half(double d) {
    uint16_t sign = signbit(d) ? 0x8000u : 0u;
    double a = fabs(d);
    if (isnan(d)) return 0x7e00u;
    if (a == 0.0) return sign;
    if (isinf(a)) return sign | 0x7c00u;
    int ex;
    (void)frexp(a, &ex); /* a = m * 2^ex, m in [0.5,1) -> a in [2^(ex-1), 2^ex) */
    int e = ex - 1;      /* unbiased exponent of the leading bit */
    if (e < -14) e = -14; /* subnormal range shares the exponent of the smallest normal */
    /* spacing of representable values near a is 2^(e-10) */
    double scaled = ldexp(a, 10 - e); /* in [0, 2048] */
    double r = nearbyint(scaled);     /* default rounding mode is to-nearest-even */
    if (r >= 2048.0) { r = 1024.0; e += 1; }
    if (e > 15) return sign | 0x7c00u;
    uint32_t ri = (uint32_t)r;
    if (ri < 1024) return sign | (uint16_t)ri; /* subnormal (e == -14, no implicit bit) */
    return sign | (uint16_t)(((uint32_t)(e + 15) << 10) | (ri - 1024));
}

/* Sec. 2.2 dequantization of one weight row.  mode 0: (q - zero) * scale.  mode 1 (1-bit sign
 * plane, no zero array): (2q - 1) * scale, i.e. zero = 1/2 and a doubled scale. */
void tman_oracle_dequant_row(const uint8_t *q, const uint16_t *scale, const uint16_t *zero, int K, int group,
                             int sign_mode, double *out) {
    for (int k = 0; k < K; ++k) {
        double s = tman_oracle_half_to_double(scale[k / group]);
        if (sign_mode) {
            out[k] = (2.0 * (double)q[k] - 1.0) * s;
        } else {
            double z = tman_oracle_half_to_double(zero[k / group]);
            out[k] = ((double)q[k] - z) * s;
        }
    }
}

/* The definition: Y[n][m] = sum_k x[n][k] * Wd[m][k], double precision, ascending k, no blocking.
 * q is one code per byte, [M][K]; scale/zero fp16 bit patterns [M][K/group]; x fp16 bits [N][K];
 * Y double [N][M].  Parallel over rows m only (each output is still one sequential sum).
 * Returns the number of threads used. */
int tman_oracle_matmul(const uint8_t *q, const uint16_t *scale, const uint16_t *zero, const uint16_t *x, int N, int M,
                       int K, int group, int sign_mode, double *Y, int threads) {
    int G = K / group;
    double *xd = (double *)malloc((size_t)N * K * sizeof(double));
    if (!xd) return -1;
    for (size_t i = 0; i < (size_t)N * K; ++i) xd[i] = tman_oracle_half_to_double(x[i]);
    int used = 1;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#pragma omp parallel
    {
#pragma omp single
        used = omp_get_num_threads();
    }
#endif
#pragma omp parallel
    {
        double *wd = (double *)malloc((size_t)K * sizeof(double));
#pragma omp for schedule(static)
        for (int m = 0; m < M; ++m) {
            tman_oracle_dequant_row(q + (size_t)m * K, scale + (size_t)m * G, zero ? zero + (size_t)m * G : NULL, K,
                                    group, sign_mode, wd);
            for (int n = 0; n < N; ++n) {
                const double *xr = xd + (size_t)n * K;
                double acc = 0.0;
                for (int k = 0; k < K; ++k) acc += xr[k] * wd[k];
                Y[(size_t)n * M + m] = acc;
            }
        }
        free(wd);
    }
    free(xd);
    return used;
}

/* Sec. 2.2 "Bit-serial table lookup", precompute step: for every group j of g consecutive
 * activations and every g-bit pattern p, T[n][j][p] = sum_{t<g} bit_t(p) * x[n][g*j+t] (exact in
 * double for fp16 inputs).  T is double [N][K/g][2^g]. */
void tman_oracle_build_tables(const uint16_t *x, int N, int K, int g, double *T) {
    int J = K / g, P = 1 << g;
    for (int n = 0; n < N; ++n)
        for (int j = 0; j < J; ++j)
            for (int p = 0; p < P; ++p) {
                double acc = 0.0;
                for (int t = 0; t < g; ++t)
                    if ((p >> t) & 1) acc += tman_oracle_half_to_double(x[(size_t)n * K + (size_t)g * j + t]);
                T[((size_t)n * J + j) * P + p] = acc;
            }
}

/* Index generation of the bit-serial form: idx_i[m][j] = sum_{t<g} bit_i(q[m][g*j+t]) << t,
 * i.e. the g-bit pattern that plane i of g consecutive weights presents to table j.
 * idx is uint8 [bits][M][K/g] (g <= 8). */
void tman_oracle_lut_indices(const uint8_t *q, int M, int K, int bits, int g, uint8_t *idx) {
    int J = K / g;
    for (int i = 0; i < bits; ++i)
        for (int m = 0; m < M; ++m)
            for (int j = 0; j < J; ++j) {
                unsigned p = 0;
                for (int t = 0; t < g; ++t) p |= ((unsigned)(q[(size_t)m * K + (size_t)g * j + t] >> i) & 1u) << t;
                idx[((size_t)i * M + m) * J + j] = (uint8_t)p;
            }
}

/* The table-lookup form of the whole product, in the paper's order: decompose the codes into one-bit
 * planes, look every g-bit pattern up in the activation tables, shift by the plane's weight and
 * accumulate inside one quantization group; then apply the group's scale, and its zero through the
 * group's activation sum S[n][G] = sum_{k in G} x[n][k]:
 *     Y[n][m] = sum_G scale[m][G] * ( sum_i 2^i sum_{j in G} T[n][j][idx_i[m][j]] - zero[m][G] * S[n][G] )
 * (sign mode: scale * (2 * sum_j T - S)).  With round_tables != 0 every table entry is first
 * rounded to binary16 (16-bit entries, Sec. 5 "Efficient table look-up by VLUT"), which models the
 * precision the lookup kernel really works at; S stays exact.  If group_sums is non-NULL it receives
 * A[n][m][G] = sum_i 2^i sum_{j in G} T[..], the pre-scale integer-weighted sums, for the identity
 * test against sum_{k in G} q*x. */
void tman_oracle_lut_matmul(const uint8_t *q, const uint16_t *scale, const uint16_t *zero, const uint16_t *x, int N,
                            int M, int K, int bits, int group, int g, int sign_mode, int round_tables, double *Y,
                            double *group_sums) {
    int J = K / g, P = 1 << g, G = K / group, jpg = group / g;
    double *T = (double *)malloc((size_t)N * J * P * sizeof(double));
    uint8_t *idx = (uint8_t *)malloc((size_t)bits * M * J);
    double *S = (double *)malloc((size_t)N * G * sizeof(double));
    tman_oracle_build_tables(x, N, K, g, T);
    if (round_tables)
        for (size_t e = 0; e < (size_t)N * J * P; ++e)
            T[e] = tman_oracle_half_to_double(tman_oracle_double_to_half(T[e]));
    tman_oracle_lut_indices(q, M, K, bits, g, idx);
    for (int n = 0; n < N; ++n)
        for (int gq = 0; gq < G; ++gq) {
            double acc = 0.0;
            for (int k = gq * group; k < (gq + 1) * group; ++k) acc += tman_oracle_half_to_double(x[(size_t)n * K + k]);
            S[(size_t)n * G + gq] = acc;
        }
    for (int n = 0; n < N; ++n)
        for (int m = 0; m < M; ++m) {
            double y = 0.0;
            for (int gq = 0; gq < G; ++gq) {
                double a = 0.0;
                for (int i = 0; i < bits; ++i) {
                    double plane = 0.0;
                    for (int j = gq * jpg; j < (gq + 1) * jpg; ++j)
                        plane += T[((size_t)n * J + j) * P + idx[((size_t)i * M + m) * J + j]];
                    a += ldexp(plane, i); /* shift by the plane's bit position, then accumulate */
                }
                if (group_sums) group_sums[((size_t)n * M + m) * G + gq] = a;
                double s = tman_oracle_half_to_double(scale[(size_t)m * G + gq]);
                if (sign_mode) {
                    y += s * (2.0 * a - S[(size_t)n * G + gq]);
                } else {
                    double z = tman_oracle_half_to_double(zero[(size_t)m * G + gq]);
                    y += s * (a - z * S[(size_t)n * G + gq]);
                }
            }
            Y[(size_t)n * M + m] = y;
        }
    free(T);
    free(idx);
    free(S);
}

/* Sec. 4.1 "Bit repacking": entry p of the repacking table for bit position i maps the i-th bits of
 * four weights (pattern p, weight t in bit t) to a 16-bit word holding four 4-bit fields, field t
 * receiving that bit at position i:  R_i[p] = sum_t bit_t(p) << (4t + i). */
uint16_t tman_oracle_repack_entry(int i, int p) {
    uint16_t r = 0;
    for (int t = 0; t < 4; ++t)
        if ((p >> t) & 1) r |= (uint16_t)(1u << (4 * t + i));
    return r;
}

/* Sec. 4.1 "Integer-to-float conversion" + "Applying scales and zero-points": the per-quantization-
 * block table with the affine transform baked in, D[c] = fp16((c - zero) * scale), c in [0, 2^bits)
 * (sign mode: fp16((2c - 1) * scale)).  One rounding to binary16 from the exact double product of
 * fp16 inputs (the product of two 11-bit significands and the difference c - zero are exact in
 * double).  D is fp16 bit patterns [2^bits]. */
void tman_oracle_dequant_table(uint16_t scale, uint16_t zero, int bits, int sign_mode, uint16_t *D) {
    double s = tman_oracle_half_to_double(scale);
    double z = tman_oracle_half_to_double(zero);
    for (int c = 0; c < (1 << bits); ++c) {
        double v = sign_mode ? (2.0 * c - 1.0) * s : ((double)c - z) * s;
        D[c] = tman_oracle_double_to_half(v);
    }
}

/* Prefill as the method really computes it: the two-level table dequantization (Sec. 4.1) turns every
 * code into an fp16 weight through its block's table D, and the matrix unit multiplies fp16 by fp16
 * with wide accumulation -- modelled here as exact products summed in double.  Used to separate the
 * method's own fp16 weight rounding from kernel error when deriving the tolerance. */
void tman_oracle_table_dequant_matmul(const uint8_t *q, const uint16_t *scale, const uint16_t *zero, const uint16_t *x,
                                      int N, int M, int K, int bits, int group, int sign_mode, double *Y) {
    int G = K / group;
    uint16_t D[16];
    double *wd = (double *)malloc((size_t)K * sizeof(double));
    for (int m = 0; m < M; ++m) {
        for (int gq = 0; gq < G; ++gq) {
            tman_oracle_dequant_table(scale[(size_t)m * G + gq], zero ? zero[(size_t)m * G + gq] : 0, bits, sign_mode, D);
            for (int k = gq * group; k < (gq + 1) * group; ++k)
                wd[k] = tman_oracle_half_to_double(D[q[(size_t)m * K + k]]);
        }
        for (int n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int k = 0; k < K; ++k) acc += tman_oracle_half_to_double(x[(size_t)n * K + k]) * wd[k];
            Y[(size_t)n * M + m] = acc;
        }
    }
    free(wd);
}

/* ------------------------------------------------------------------------------------------------
 * Integer activations and integer tables (Sec. 6.1 "A_INT16"; Sec. 4.3 two-level tiling: table entries are
 * aggregated at low precision inside a quantization block, in floating point only across blocks; Sec. 5:
 * 16-bit table entries).
 *
 * Reading used here (the paper gives no quantizer): every token n gets a power-of-two step 2^e[n], the
 * smallest for which all |x[n][k]| / 2^e[n] <= 8191, and integer activations
 *     xq[n][k] = round_to_nearest_even( x[n][k] / 2^e[n] ),   |xq| <= 8191
 * so that the sum of any four of them fits a 16-bit table entry exactly.  Dividing an fp16 number by a power
 * of two is exact, so the integer is the same in any precision.  With max|x| = m * 2^E (0.5 <= m < 1) the
 * exponent is e = E - 13 (m <= 1 - 2^-11 for an fp16 number, hence m * 2^13 <= 8191); a token of zeros gets
 * e = 0.  The activations the method then works with are xhat = xq * 2^e.
 */
void tman_oracle_quantize_activations(const uint16_t *x, int N, int K, int16_t *xq, int32_t *e) {
    for (int n = 0; n < N; ++n) {
        double mx = 0.0;
        for (int k = 0; k < K; ++k) {
            double a = fabs(tman_oracle_half_to_double(x[(size_t)n * K + k]));
            if (a > mx) mx = a;
        }
        int ex = 0;
        if (mx > 0.0) {
            int E;
            (void)frexp(mx, &E);
            ex = E - 13;
        }
        e[n] = ex;
        for (int k = 0; k < K; ++k) {
            double t = ldexp(tman_oracle_half_to_double(x[(size_t)n * K + k]), -ex); /* exact */
            xq[(size_t)n * K + k] = (int16_t)nearbyint(t);                            /* ties to even */
        }
    }
}

/* The definition with real-valued (double) activations: Y[n][m] = sum_k xd[n][k] * Wd[m][k], as
 * tman_oracle_matmul but for activations that are not fp16 numbers (the dequantized integer activations). */
void tman_oracle_matmul_real_x(const uint8_t *q, const uint16_t *scale, const uint16_t *zero, const double *xd, int N,
                               int M, int K, int group, int sign_mode, double *Y) {
    int G = K / group;
#pragma omp parallel
    {
        double *wd = (double *)malloc((size_t)K * sizeof(double));
#pragma omp for schedule(static)
        for (int m = 0; m < M; ++m) {
            tman_oracle_dequant_row(q + (size_t)m * K, scale + (size_t)m * G, zero ? zero + (size_t)m * G : NULL, K,
                                    group, sign_mode, wd);
            for (int n = 0; n < N; ++n) {
                double acc = 0.0;
                for (int k = 0; k < K; ++k) acc += xd[(size_t)n * K + k] * wd[k];
                Y[(size_t)n * M + m] = acc;
            }
        }
        free(wd);
    }
}

/* The table-lookup form on integer activations, step by step: 16-bit integer tables
 *     Tq[n][j][p] = sum_{t<4} bit_t(p) * xq[n][4j+t]          (fits int16 by construction)
 * looked up by the 4-bit weight patterns of every bit plane, shifted by the plane's position and accumulated
 * as integers inside one quantization block,
 *     A[n][m][G] = sum_i 2^i sum_{j in G} Tq[n][j][idx_i[m][j]],   Sq[n][G] = sum_{k in G} xq[n][k]
 * and only then scaled in floating point:
 *     Y[n][m] = 2^e[n] * sum_G scale[m][G] * ( A[n][m][G] - zero[m][G] * Sq[n][G] )
 * (sign mode: scale * (2 A - Sq)).  block_sums, if non-NULL, receives A as 64-bit integers [N][M][K/group].
 * Returns 0, or 1 if a table entry would not fit 16 bits (it cannot, for quantizer output). */
int tman_oracle_lut_matmul_i16(const uint8_t *q, const uint16_t *scale, const uint16_t *zero, const int16_t *xq,
                               const int32_t *e, int N, int M, int K, int bits, int group, int sign_mode, double *Y,
                               int64_t *block_sums) {
    const int g = 4;
    int J = K / g, G = K / group, jpg = group / g, overflow = 0;
    int16_t *T = (int16_t *)malloc((size_t)N * J * 16 * sizeof(int16_t));
    uint8_t *idx = (uint8_t *)malloc((size_t)bits * M * J);
    for (int n = 0; n < N; ++n)
        for (int j = 0; j < J; ++j)
            for (int p = 0; p < 16; ++p) {
                int32_t acc = 0;
                for (int t = 0; t < g; ++t)
                    if ((p >> t) & 1) acc += xq[(size_t)n * K + (size_t)g * j + t];
                if (acc < -32768 || acc > 32767) overflow = 1;
                T[((size_t)n * J + j) * 16 + p] = (int16_t)acc;
            }
    tman_oracle_lut_indices(q, M, K, bits, g, idx);
    for (int n = 0; n < N; ++n)
        for (int m = 0; m < M; ++m) {
            double y = 0.0;
            for (int gq = 0; gq < G; ++gq) {
                int64_t a = 0, sq = 0;
                for (int i = 0; i < bits; ++i) {
                    int64_t plane = 0;
                    for (int j = gq * jpg; j < (gq + 1) * jpg; ++j)
                        plane += T[((size_t)n * J + j) * 16 + idx[((size_t)i * M + m) * J + j]];
                    a += plane * ((int64_t)1 << i); /* shift by the plane's bit position, then accumulate */
                }
                for (int k = gq * group; k < (gq + 1) * group; ++k) sq += xq[(size_t)n * K + k];
                if (block_sums) block_sums[((size_t)n * M + m) * G + gq] = a;
                double s = tman_oracle_half_to_double(scale[(size_t)m * G + gq]);
                if (sign_mode) {
                    y += s * (2.0 * (double)a - (double)sq);
                } else {
                    double z = tman_oracle_half_to_double(zero[(size_t)m * G + gq]);
                    y += s * ((double)a - z * (double)sq);
                }
            }
            Y[(size_t)n * M + m] = ldexp(y, e[n]);
        }
    free(T);
    free(idx);
    return overflow;
}

/* ------------------------------------------------------------------------------------------------
 * Per-channel / per-tensor formats on an integer matrix unit (Sec. 6.1: BitNet's ternary weights with one
 * scale per tensor, treated as 2-bit; Sec. 6.2 mpGEMM: such models are dequantized to INT8 and computed as
 * W_INT8 x A_INT8).
 *
 * Reading used here (the paper gives no activation quantizer; this is the per-token absmax quantizer of the
 * BitNet family): token n has the step delta[n] = max_k |x[n][k]| / 127 and integer activations
 *     xq[n][k] = round_to_nearest_even( x[n][k] * (127 / max) ),   |xq| <= 127,
 * the decision taken in binary32 arithmetic as the kernel takes it: inv = 127.0f / max (one correctly rounded
 * division), t = x * inv (one correctly rounded product), xq = rint(t).  A token of zeros has delta = 0.
 */
void tman_oracle_quantize_activations_i8(const uint16_t *x, int N, int K, int8_t *xq, float *absmax) {
    for (int n = 0; n < N; ++n) {
        float mx = 0.0f;
        for (int k = 0; k < K; ++k) {
            float a = fabsf((float)tman_oracle_half_to_double(x[(size_t)n * K + k]));
            if (a > mx) mx = a;
        }
        absmax[n] = mx;
        volatile float inv = mx > 0.0f ? 127.0f / mx : 0.0f; /* volatile: no excess precision, no reassociation */
        for (int k = 0; k < K; ++k) {
            volatile float t = (float)tman_oracle_half_to_double(x[(size_t)n * K + k]) * inv;
            xq[(size_t)n * K + k] = (int8_t)nearbyintf(t);
        }
    }
}

/* Integer product and its scaling: with the weights' codes c[m][k] (unsigned, below 2^bits), ONE scale s[m] and
 * zero z[m] per row (a per-tensor format repeats the same pair for every row):
 *     acc[n][m] = sum_k c[m][k] * xq[n][k]                      exact integer
 *     Y[n][m]   = s[m] * (absmax[n] / 127) * ( acc[n][m] - z[m] * sum_k xq[n][k] )
 * (sign form: s * delta * (2 acc - sum xq)).  acc is int64 [N][M]; Y double [N][M]. */
void tman_oracle_matmul_i8(const uint8_t *q, const uint16_t *row_scale, const uint16_t *row_zero, const int8_t *xq,
                           const float *absmax, int N, int M, int K, int sign_mode, int64_t *acc, double *Y) {
    for (int n = 0; n < N; ++n) {
        int64_t sx = 0;
        for (int k = 0; k < K; ++k) sx += xq[(size_t)n * K + k];
        double delta = (double)absmax[n] / 127.0;
        for (int m = 0; m < M; ++m) {
            int64_t a = 0;
            for (int k = 0; k < K; ++k) a += (int64_t)q[(size_t)m * K + k] * (int64_t)xq[(size_t)n * K + k];
            acc[(size_t)n * M + m] = a;
            double s = tman_oracle_half_to_double(row_scale[m]);
            if (sign_mode) {
                Y[(size_t)n * M + m] = s * delta * (2.0 * (double)a - (double)sx);
            } else {
                double z = tman_oracle_half_to_double(row_zero[m]);
                Y[(size_t)n * M + m] = s * delta * ((double)a - z * (double)sx);
            }
        }
    }
}

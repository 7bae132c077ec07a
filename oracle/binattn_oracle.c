/*
 * CPU oracle for the BinaryAttention forward pass.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, literal reference that the
 * HIP library is checked against.  Only the tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it; the product never does, and it
 * shares no code, header, table or constant with the HIP sources.
 *
 * Every function below is one step of the method, written the way the paper
 * states it (scalar loops, fp64 unless noted), for ONE attention head:
 * Q, K, V are row-major [N, d] arrays of bf16 bit patterns (uint16).
 * OpenMP is used over independent query rows only; there is no blocking,
 * fusion or reordering.
 *
 * Readings taken where the paper is silent or inconsistent:
 *  - sign(x) = +1 iff x >= 0 by IEEE comparison (so -0.0 -> +1, NaN -> -1);
 *    Sec. 3 defines sign as +1 on the non-negative reals and -1 elsewhere.
 *  - mu_q, mu_k = mean of ABSOLUTE values over tokens and channels of one head
 *    (the only non-negative "mean" that is also the optimal scale of Sec. 3).
 *  - The logit follows Eq. 6 (with 1/sqrt(d), passed in as `scale`), not
 *    Alg. 1's line that omits it.
 *  - P is quantised as in Alg. 1: round(255 * exp(S - max)), i.e. relative to
 *    the row maximum, not the normalised probability of Eq. 7 (which would
 *    round to zero for long flat rows).  The row sum l uses the unquantised
 *    exp values (Alg. 1).
 *  - Alg. 1's accumulator update multiplies the old accumulator by
 *    exp(m_old - m_new) (the printed inverse is a notation slip).
 *  - Rounding is to nearest, ties to even; V codes are clamped to [-127, 127],
 *    P codes to [0, 255].
 *  - V quantisation runs in fp32 (delta = absmax / 127 with IEEE division,
 *    code = rne(v / delta) with IEEE division) so that the integer codes are
 *    a bit-exact checkpoint; V is assumed finite.
 *
 * Parity status: sign bits, integer logits, V codes and the unquantised
 * output O1 are pinned by the CPU tests (brute force, the Hamming identity,
 * Theorem 1, closed forms, a library softmax).  The quantised output O2 is
 * pinned by special cases and by its error bound against O1; the paper prints
 * no worked numerical example, so end values against the paper itself are
 * "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* Exact value of a bf16 bit pattern (bf16 is the top half of an fp32). */
static float bf16_to_float(uint16_t h) {
    uint32_t u = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

int ba_oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------
 * Sec. 3 / Sec. 4.1 / Eq. 5: s = sign(x) in {-1,+1}.
 * ---------------------------------------------------------------------- */
void ba_oracle_sign_pm1(const uint16_t *x, int64_t count, int8_t *s) {
    for (int64_t i = 0; i < count; ++i) {
        double v = (double)bf16_to_float(x[i]);
        s[i] = (v >= 0.0) ? (int8_t)1 : (int8_t)-1;
    }
}

/* Bit-packed form of the same signs: bit (c & 31) of word (c >> 5) of token t
 * is 1 iff x[t][c] >= 0.  W = ceil(d/32) words per token, unused bits are 0. */
void ba_oracle_sign_pack(const uint16_t *x, int64_t n_tokens, int d, uint32_t *words) {
    int W = (d + 31) / 32;
    for (int64_t t = 0; t < n_tokens; ++t) {
        for (int w = 0; w < W; ++w) words[t * W + w] = 0u;
        for (int c = 0; c < d; ++c) {
            double v = (double)bf16_to_float(x[t * (int64_t)d + c]);
            if (v >= 0.0) words[t * W + (c >> 5)] |= (1u << (c & 31));
        }
    }
}

/* ------------------------------------------------------------------------
 * Eq. 5 text: mu = mean of |x| over the token and channel axes of one head.
 * ---------------------------------------------------------------------- */
double ba_oracle_abs_mean(const uint16_t *x, int64_t count) {
    double sum = 0.0;
    for (int64_t i = 0; i < count; ++i) sum += fabs((double)bf16_to_float(x[i]));
    return sum / (double)count;
}

/* ------------------------------------------------------------------------
 * Sec. 4.1: S_ij = s_i . t_j, the literal +-1 inner product.
 * rows[r] selects the query rows; I is [n_rows, N].
 * ---------------------------------------------------------------------- */
void ba_oracle_logits_literal(const uint16_t *Q, const uint16_t *K, int64_t N, int d,
                              const int64_t *rows, int64_t n_rows, int32_t *I) {
    int8_t *s = (int8_t *)malloc((size_t)N * d);
    int8_t *t = (int8_t *)malloc((size_t)N * d);
    ba_oracle_sign_pm1(Q, N * d, s);
    ba_oracle_sign_pm1(K, N * d, t);
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < n_rows; ++r) {
        int64_t i = rows[r];
        for (int64_t j = 0; j < N; ++j) {
            int32_t acc = 0;
            for (int c = 0; c < d; ++c) acc += (int32_t)s[i * d + c] * (int32_t)t[j * d + c];
            I[r * N + j] = acc;
        }
    }
    free(s);
    free(t);
}

/* Number of set bits, one bit at a time. */
static int popcount32_slow(uint32_t x) {
    int n = 0;
    for (int b = 0; b < 32; ++b) n += (int)((x >> b) & 1u);
    return n;
}

/* Sec. 4.1: the same inner product through the Hamming distance,
 * s.t = d - 2 * ||s - t||_H, with ||.||_H = popcount(bits_s XOR bits_t). */
void ba_oracle_logits_hamming(const uint32_t *qw, const uint32_t *kw, int64_t N, int d,
                              const int64_t *rows, int64_t n_rows, int32_t *I) {
    int W = (d + 31) / 32;
    for (int64_t r = 0; r < n_rows; ++r) {
        int64_t i = rows[r];
        for (int64_t j = 0; j < N; ++j) {
            int ham = 0;
            for (int w = 0; w < W; ++w) ham += popcount32_slow(qw[i * W + w] ^ kw[j * W + w]);
            I[r * N + j] = d - 2 * ham;
        }
    }
}

/* ------------------------------------------------------------------------
 * Eq. 7 / Sec. 4.2, signed 8-bit codes with one scale per channel:
 * delta[c] = max_n |v[n][c]| / 127, code = round(v / delta) in [-127, 127].
 * fp32 arithmetic with IEEE division (see header).
 * ---------------------------------------------------------------------- */
void ba_oracle_quant_v(const uint16_t *V, int64_t N, int d, int8_t *vq, float *delta) {
    for (int c = 0; c < d; ++c) {
        float a = 0.0f;
        for (int64_t n = 0; n < N; ++n) {
            float v = fabsf(bf16_to_float(V[n * d + c]));
            if (v > a) a = v;
        }
        volatile float dl = (a == 0.0f) ? 1.0f : a / 127.0f;
        delta[c] = dl;
    }
    for (int64_t n = 0; n < N; ++n) {
        for (int c = 0; c < d; ++c) {
            volatile float r = bf16_to_float(V[n * d + c]) / delta[c];
            float q = nearbyintf(r); /* default rounding mode: ties to even */
            if (q > 127.0f) q = 127.0f;
            if (q < -127.0f) q = -127.0f;
            vq[n * d + c] = (int8_t)q;
        }
    }
}

static double bias_at(const void *bias, int bias_dtype, int64_t idx) {
    if (bias_dtype == 1) return (double)bf16_to_float(((const uint16_t *)bias)[idx]);
    if (bias_dtype == 2) return (double)((const float *)bias)[idx];
    return 0.0;
}

/* ------------------------------------------------------------------------
 * The attention rows by their definition (Eq. 6 logits, softmax of Eq. 1,
 * Eq. 7 quantised aggregation with Alg. 1's choice of what is quantised),
 * using the row's true maximum.
 *
 * bias: [N, N] with row stride bias_row_stride elements, dtype 0 = none,
 *       1 = bf16 bits, 2 = fp32.
 * vq, delta: output of ba_oracle_quant_v for this head.
 * Outputs (each may be NULL): O2 [n_rows,d] quantised result, O1 [n_rows,d]
 * unquantised result, P_hat [n_rows,N] = exp(S - m), P_code [n_rows,N],
 * l_out [n_rows] = sum_j P_hat, m_out [n_rows], S_out [n_rows,N].
 * ---------------------------------------------------------------------- */
void ba_oracle_attention_rows(const uint16_t *Q, const uint16_t *K, const uint16_t *V,
                              int64_t N, int d, const void *bias, int bias_dtype,
                              int64_t bias_row_stride, double scale, double mu_q, double mu_k,
                              const int8_t *vq, const float *delta, const int64_t *rows,
                              int64_t n_rows, double *O2, double *O1, double *P_hat,
                              uint8_t *P_code, double *l_out, double *m_out, double *S_out) {
    int8_t *s = (int8_t *)malloc((size_t)N * d);
    int8_t *t = (int8_t *)malloc((size_t)N * d);
    ba_oracle_sign_pm1(Q, N * d, s);
    ba_oracle_sign_pm1(K, N * d, t);
#pragma omp parallel
    {
        double *S = (double *)malloc(sizeof(double) * (size_t)N);
        double *P = (double *)malloc(sizeof(double) * (size_t)N);
        int64_t *acc = (int64_t *)malloc(sizeof(int64_t) * (size_t)d);
#pragma omp for schedule(dynamic, 4)
        for (int64_t r = 0; r < n_rows; ++r) {
            int64_t i = rows[r];
            /* Eq. 6: S_ij = mu_q mu_k (s_i . t_j) * scale + b_ij */
            for (int64_t j = 0; j < N; ++j) {
                int32_t dot = 0;
                for (int c = 0; c < d; ++c) dot += (int32_t)s[i * d + c] * (int32_t)t[j * d + c];
                double b = bias_dtype ? bias_at(bias, bias_dtype, i * bias_row_stride + j) : 0.0;
                S[j] = mu_q * mu_k * (double)dot * scale + b;
            }
            /* softmax numerator relative to the row maximum, and its sum */
            double m = S[0];
            for (int64_t j = 1; j < N; ++j) if (S[j] > m) m = S[j];
            double l = 0.0;
            for (int64_t j = 0; j < N; ++j) { P[j] = exp(S[j] - m); l += P[j]; }
            /* Eq. 7 with Alg. 1's operand: code = round(255 * P_hat) */
            for (int c = 0; c < d; ++c) acc[c] = 0;
            for (int64_t j = 0; j < N; ++j) {
                double code = nearbyint(255.0 * P[j]);
                if (code > 255.0) code = 255.0;
                if (code < 0.0) code = 0.0;
                if (P_code) P_code[r * N + j] = (uint8_t)code;
                int64_t pc = (int64_t)code;
                for (int c = 0; c < d; ++c) acc[c] += pc * (int64_t)vq[j * d + c];
            }
            /* Alg. 1 last line: O = O / (255 l) * delta_v */
            if (O2)
                for (int c = 0; c < d; ++c)
                    O2[r * d + c] = (double)delta[c] * (double)acc[c] / (255.0 * l);
            /* Eq. 1 with the logits of Eq. 6, nothing quantised */
            if (O1)
                for (int c = 0; c < d; ++c) {
                    double o = 0.0;
                    for (int64_t j = 0; j < N; ++j)
                        o += (P[j] / l) * (double)bf16_to_float(V[j * d + c]);
                    O1[r * d + c] = o;
                }
            if (P_hat) for (int64_t j = 0; j < N; ++j) P_hat[r * N + j] = P[j];
            if (S_out) for (int64_t j = 0; j < N; ++j) S_out[r * N + j] = S[j];
            if (l_out) l_out[r] = l;
            if (m_out) m_out[r] = m;
        }
        free(S);
        free(P);
        free(acc);
    }
    free(s);
    free(t);
}

/* ------------------------------------------------------------------------
 * Alg. 1 taken step by step: key/value blocks of Bv rows, running maximum m,
 * running sum l, accumulator rescaled by exp(m_old - m_new) per block, P
 * quantised relative to the RUNNING maximum, final O / (255 l) * delta_v.
 * With quantise = 0 the codes are replaced by 255 * P_hat and V codes by
 * v / delta (nothing rounded), which must reproduce O1 for any Bv.
 * O is [n_rows, d].
 * ---------------------------------------------------------------------- */
void ba_oracle_algorithm1_rows(const uint16_t *Q, const uint16_t *K, const uint16_t *V,
                               int64_t N, int d, const void *bias, int bias_dtype,
                               int64_t bias_row_stride, double scale, double mu_q, double mu_k,
                               const int8_t *vq, const float *delta, int64_t Bv, int quantise,
                               const int64_t *rows, int64_t n_rows, double *O) {
    int8_t *s = (int8_t *)malloc((size_t)N * d);
    int8_t *t = (int8_t *)malloc((size_t)N * d);
    ba_oracle_sign_pm1(Q, N * d, s);
    ba_oracle_sign_pm1(K, N * d, t);
    double *Sblk = (double *)malloc(sizeof(double) * (size_t)Bv);
    double *Pblk = (double *)malloc(sizeof(double) * (size_t)Bv);
    double *acc = (double *)malloc(sizeof(double) * (size_t)d);
    double *blk = (double *)malloc(sizeof(double) * (size_t)d);
    for (int64_t r = 0; r < n_rows; ++r) {
        int64_t i = rows[r];
        double m = -INFINITY, l = 0.0;
        for (int c = 0; c < d; ++c) acc[c] = 0.0;
        for (int64_t j0 = 0; j0 < N; j0 += Bv) {
            int64_t nb = (N - j0 < Bv) ? (N - j0) : Bv;
            /* S_ij = BinaryMatmul(S_i, T_j) * mu_q * mu_k (* scale) + B_ij */
            for (int64_t jj = 0; jj < nb; ++jj) {
                int64_t j = j0 + jj;
                int32_t dot = 0;
                for (int c = 0; c < d; ++c) dot += (int32_t)s[i * d + c] * (int32_t)t[j * d + c];
                double b = bias_dtype ? bias_at(bias, bias_dtype, i * bias_row_stride + j) : 0.0;
                Sblk[jj] = mu_q * mu_k * (double)dot * scale + b;
            }
            /* m_ij = max(m_{i,j-1}, rowmax(S_ij)) */
            double m_new = m;
            for (int64_t jj = 0; jj < nb; ++jj) if (Sblk[jj] > m_new) m_new = Sblk[jj];
            /* P_hat = exp(S - m_ij); l_ij = e^{m_old - m_new} l + rowsum(P_hat) */
            double resc = exp(m - m_new); /* exp(-inf) = 0 on the first block */
            double rs = 0.0;
            if (m_new == -INFINITY) {
                /* every key seen so far carries a -inf bias (a mask): exp(-inf - (-inf)) is
                   undefined in Alg. 1 as printed; a masked key has weight 0 (the limit of
                   exp(s - m) for s -> -inf at any finite m), so the block adds nothing */
                resc = 1.0;
                for (int64_t jj = 0; jj < nb; ++jj) Pblk[jj] = 0.0;
            } else {
                for (int64_t jj = 0; jj < nb; ++jj) { Pblk[jj] = exp(Sblk[jj] - m_new); rs += Pblk[jj]; }
            }
            l = resc * l + rs;
            /* O_ij = IntMatmul(P_hat * 255, V~_j) */
            for (int c = 0; c < d; ++c) blk[c] = 0.0;
            for (int64_t jj = 0; jj < nb; ++jj) {
                int64_t j = j0 + jj;
                double pc = 255.0 * Pblk[jj];
                if (quantise) {
                    pc = nearbyint(pc);
                    if (pc > 255.0) pc = 255.0;
                    if (pc < 0.0) pc = 0.0;
                }
                for (int c = 0; c < d; ++c) {
                    double vv = quantise ? (double)vq[j * d + c]
                                         : (double)bf16_to_float(V[j * d + c]) / (double)delta[c];
                    blk[c] += pc * vv;
                }
            }
            /* O_ij = e^{m_old - m_new} O_{i,j-1} + O_ij */
            for (int c = 0; c < d; ++c) acc[c] = resc * acc[c] + blk[c];
            m = m_new;
        }
        /* O_i = O / l / 255 * delta_v */
        for (int c = 0; c < d; ++c) O[r * d + c] = acc[c] / l / 255.0 * (double)delta[c];
    }
    free(s); free(t); free(Sblk); free(Pblk); free(acc); free(blk);
}

/*
 * CPU oracle for the BitNet b1.58 BitLinear product (arXiv 2410.16144).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is the plain, slow, scalar definition of
 * what the GPU library computes.  Only the test-suite, the smoke check and
 * the benchmark's "cpu_baseline" leg may call it; the product path never
 * does.  It shares no code, headers, tables or helpers with the HIP path.
 *
 * Every function is a literal loop nest over the definition.  No blocking,
 * no SIMD intrinsics, no reordering.  The only concession to run time is an
 * OpenMP "parallel for" over independent output elements.
 *
 * Build:  gcc -O2 -std=c11 -ffp-contract=off -fno-fast-math -fopenmp
 *         -shared -fPIC bitlinear_oracle.c -o libbl_oracle.so -lm
 * (-ffp-contract=off matters: the activation quantizer is specified as a
 * sequence of individually rounded fp32 operations.)
 *
 * Notation (paper Section 2 and the BitNet b1.58 formulation it builds on):
 *   W  in {-1,0,+1}^{N x K}, row n = output feature n, out = x * W^T
 *   w_scale   one fp32 per matrix (the absmean scale)
 *   X  in R^{M x K}, one row per token
 *   q  in int8^{M x K}, a_scale in fp32^M (per-token absmax scale)
 *   acc in int32^{M x N}, out in fp32^{M x N}
 *
 * Pins (tests/test_oracle_pins.py): every function below is checked against
 * something other than itself -- the code tables the paper prints (Tables
 * 1-3), float64 brute force, closed forms, invariants.  Nothing here is
 * "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void orc_set_num_threads(int n) {
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ------------------------------------------------------------------ */
/* Weight side                                                         */
/* ------------------------------------------------------------------ */

/*
 * Absmean ternarization (the "per-tensor absmean scale" of BitNet b1.58,
 * which Section 2 calls transforming each full-precision weight offline).
 *   w_scale = mean(|Wf|)                      sum in double, result fp32
 *   Wt      = clip(round_half_even(Wf / (w_scale + 1e-5)), -1, +1)
 * The epsilon only guards the division; the dequant scale is w_scale itself.
 * Offline helper: no GPU kernel computes this.
 */
void orc_absmean_ternarize(const float *wf, int64_t count, int8_t *wt, float *w_scale) {
    double s = 0.0;
    for (int64_t i = 0; i < count; ++i) s += fabs((double)wf[i]);
    float gamma = count > 0 ? (float)(s / (double)count) : 0.0f;
    float denom = gamma + 1e-5f;
    for (int64_t i = 0; i < count; ++i) {
        float r = rintf(wf[i] / denom);
        if (r > 1.0f) r = 1.0f;
        if (r < -1.0f) r = -1.0f;
        wt[i] = (int8_t)r;
    }
    *w_scale = gamma;
}

/*
 * I2_S 2-bit code (Table 1): -1 -> 00, 0 -> 01, +1 -> 10.  Code 11 is unused.
 * encode returns -1 for a value that is not ternary; decode returns -2 for
 * the unused code.
 */
int orc_i2s_encode(int w) {
    if (w == -1) return 0;
    if (w == 0) return 1;
    if (w == 1) return 2;
    return -1;
}

int orc_i2s_decode(int code) {
    if (code == 0) return -1;
    if (code == 1) return 0;
    if (code == 2) return 1;
    return -2;
}

/*
 * Canonical (oracle-only) I2_S packing, used to exercise the code table on
 * whole matrices: row-major, weight k of a row goes to bits [2(k%4), 2(k%4)+1]
 * of byte k/4 of that row; each row occupies ceil(K/4) bytes, unused bit
 * positions of the last byte hold the code for 0.  The GPU library's own
 * tiled layout is different and is never seen by the oracle.
 * Returns the number of non-ternary inputs (each is stored as 0).
 */
int64_t orc_i2s_pack(const int8_t *w, int64_t N, int64_t K, uint8_t *packed) {
    int64_t row_bytes = (K + 3) / 4;
    int64_t bad = 0;
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t b = 0; b < row_bytes; ++b) {
            unsigned byte = 0;
            for (int j = 0; j < 4; ++j) {
                int64_t k = 4 * b + j;
                int code = 1; /* pad = weight 0 */
                if (k < K) {
                    code = orc_i2s_encode(w[n * K + k]);
                    if (code < 0) { code = 1; ++bad; }
                }
                byte |= (unsigned)code << (2 * j);
            }
            packed[n * row_bytes + b] = (uint8_t)byte;
        }
    }
    return bad;
}

/* Inverse of orc_i2s_pack.  Returns the number of invalid (11) codes met. */
int64_t orc_i2s_unpack(const uint8_t *packed, int64_t N, int64_t K, int8_t *w) {
    int64_t row_bytes = (K + 3) / 4;
    int64_t bad = 0;
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t k = 0; k < K; ++k) {
            unsigned byte = packed[n * row_bytes + k / 4];
            int v = orc_i2s_decode((int)((byte >> (2 * (k % 4))) & 3u));
            if (v == -2) { v = 0; ++bad; }
            w[n * K + k] = (int8_t)v;
        }
    }
    return bad;
}

/*
 * TL1 index (Table 2): two ternary weights -> 4-bit index, base-3 with the
 * first weight as the high digit: idx = 3*(w0+1) + (w1+1), range 0..8.
 */
int orc_tl1_index(int w0, int w1) { return 3 * (w0 + 1) + (w1 + 1); }

/*
 * TL2 code (Table 3): three ternary weights -> 1 sign bit + 4-bit index.
 * With v = 9*w0 + 3*w1 + w2 (range -13..13): sign = 1 iff v < 0, idx = |v|.
 * The table prints 9 of its 27 rows; all of them satisfy this form.
 */
void orc_tl2_code(int w0, int w1, int w2, int *sign, int *idx) {
    int v = 9 * w0 + 3 * w1 + w2;
    *sign = v < 0 ? 1 : 0;
    *idx = v < 0 ? -v : v;
}

/*
 * A whole matrix in TL2 codes (Table 3): row n, group g = weights 3g, 3g+1, 3g+2 of the row (zeros beyond K)
 * becomes one byte, sign << 4 | index.  codes is [N, ceil(K/3)].  A value outside {-1,0,+1} is encoded as 0 and
 * counted.
 */
int64_t orc_tl2_encode_rows(const int8_t *w, int64_t N, int64_t K, uint8_t *codes) {
    int64_t groups = (K + 2) / 3, bad = 0;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t g = 0; g < groups; ++g) {
            int t[3];
            for (int j = 0; j < 3; ++j) {
                t[j] = (3 * g + j < K) ? w[n * K + 3 * g + j] : 0;
                if (t[j] < -1 || t[j] > 1) { t[j] = 0; ++bad; }
            }
            int sign, idx;
            orc_tl2_code(t[0], t[1], t[2], &sign, &idx);
            codes[n * groups + g] = (uint8_t)(sign << 4 | idx);
        }
    return bad;
}

/*
 * The inverse, by search: the weights of a code are the one triple among the 27 that orc_tl2_code maps to it
 * (Table 3 is a bijection between the 27 triples and the 27 codes in use).  A code no triple maps to (index 14
 * or 15, or sign with index 0) decodes to zeros and is counted.
 */
int64_t orc_tl2_decode_rows(const uint8_t *codes, int64_t N, int64_t K, int8_t *w) {
    int64_t groups = (K + 2) / 3, bad = 0;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t g = 0; g < groups; ++g) {
            int code = codes[n * groups + g], found = 0, t[3] = {0, 0, 0};
            for (int a = -1; a <= 1 && !found; ++a)
                for (int b = -1; b <= 1 && !found; ++b)
                    for (int c = -1; c <= 1 && !found; ++c) {
                        int sign, idx;
                        orc_tl2_code(a, b, c, &sign, &idx);
                        if ((sign << 4 | idx) == code) { t[0] = a; t[1] = b; t[2] = c; found = 1; }
                    }
            if (!found) ++bad;
            for (int j = 0; j < 3; ++j)
                if (3 * g + j < K) w[n * K + 3 * g + j] = (int8_t)t[j];
        }
    return bad;
}

/* ------------------------------------------------------------------ */
/* Activation side                                                     */
/* ------------------------------------------------------------------ */

/* bf16 bit pattern -> fp32 (exact: bf16 is the top half of an fp32). */
float orc_bf16_to_f32(uint16_t h) {
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/*
 * Per-token absmax quantization to int8 (BitNet b1.58 activation quantizer;
 * the paper inherits it by citation).  For each row m, in fp32, each
 * operation rounded on its own (round-to-nearest-even, no fused mul-add):
 *   amax    = max_k |x[m,k]|
 *   inv     = 127 / amax                 one fp32 division
 *   q[m,k]  = clip(round_half_even(x[m,k] * inv), -128, 127)
 *   a_scale = amax / 127                 one fp32 division
 * A row whose inv is not finite (amax == 0, or so small that 127/amax
 * overflows) is an all-zero token: q = 0 and a_scale = 0.
 * x is fp32 (is_bf16 == 0) or bf16 bit patterns (is_bf16 != 0); ldx and ldq
 * are row strides in elements.  q_sum[m] = sum_k q[m,k] if q_sum != NULL.
 */
void orc_quant_act(const void *x, int is_bf16, int64_t M, int64_t K, int64_t ldx,
                   int8_t *q, int64_t ldq, float *a_scale, int32_t *q_sum) {
    for (int64_t m = 0; m < M; ++m) {
        const float *xf = (const float *)x + m * ldx;
        const uint16_t *xh = (const uint16_t *)x + m * ldx;
        float amax = 0.0f;
        for (int64_t k = 0; k < K; ++k) {
            float v = is_bf16 ? orc_bf16_to_f32(xh[k]) : xf[k];
            float a = fabsf(v);
            if (a > amax) amax = a;
        }
        float inv = 127.0f / amax;
        int32_t sum = 0;
        if (!isfinite(inv)) {
            for (int64_t k = 0; k < K; ++k) q[m * ldq + k] = 0;
            a_scale[m] = 0.0f;
        } else {
            for (int64_t k = 0; k < K; ++k) {
                float v = is_bf16 ? orc_bf16_to_f32(xh[k]) : xf[k];
                float p = v * inv;
                float r = rintf(p);
                if (r > 127.0f) r = 127.0f;
                if (r < -128.0f) r = -128.0f;
                int32_t qi = (int32_t)r;
                q[m * ldq + k] = (int8_t)qi;
                sum += qi;
            }
            a_scale[m] = amax / 127.0f;
        }
        if (q_sum) q_sum[m] = sum;
    }
}

/* ------------------------------------------------------------------ */
/* The product                                                         */
/* ------------------------------------------------------------------ */

/*
 * Exact integer product (Section 2, I2_S: weights are turned back into their
 * original values and a plain multiply-then-add GEMV is performed):
 *   acc[m,n] = sum_k q[m,k] * W[n,k]        in int32
 * q is [M, ldq] (ldq >= K), w is [N, K] row-major with values in {-1,0,1}.
 */
void orc_matmul_i32(const int8_t *q, int64_t M, int64_t K, int64_t ldq,
                    const int8_t *w, int64_t N, int32_t *acc) {
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            int32_t s = 0;
            for (int64_t k = 0; k < K; ++k)
                s += (int32_t)q[m * ldq + k] * (int32_t)w[n * K + k];
            acc[m * N + n] = s;
        }
    }
}

/* The same sum for a chosen list of output columns n_idx[0..n_count). */
void orc_matmul_i32_cols(const int8_t *q, int64_t M, int64_t K, int64_t ldq,
                         const int8_t *w, const int64_t *n_idx, int64_t n_count,
                         int32_t *acc /* [M, n_count] */) {
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t j = 0; j < n_count; ++j) {
            int64_t n = n_idx[j];
            int32_t s = 0;
            for (int64_t k = 0; k < K; ++k)
                s += (int32_t)q[m * ldq + k] * (int32_t)w[n * K + k];
            acc[m * n_count + j] = s;
        }
    }
}

/*
 * Dequantization: out[m,n] = (float)acc[m,n] * (w_scale * a_scale[m]),
 * two fp32 multiplies (scale product first).
 */
void orc_dequant(const int32_t *acc, int64_t M, int64_t N, float w_scale,
                 const float *a_scale, float *out) {
    for (int64_t m = 0; m < M; ++m) {
        float s = w_scale * a_scale[m];
        for (int64_t n = 0; n < N; ++n) out[m * N + n] = (float)acc[m * N + n] * s;
    }
}

/*
 * The whole BitLinear forward for fp32/bf16 activations: quantize, integer
 * product, dequantize.  Scratch (q, a_scale, acc) is supplied by the caller
 * so nothing is allocated here.
 */
void orc_bitlinear(const void *x, int is_bf16, int64_t M, int64_t K, int64_t ldx,
                   const int8_t *w, int64_t N, float w_scale,
                   int8_t *q /*[M,K]*/, float *a_scale /*[M]*/, int32_t *acc /*[M,N]*/,
                   float *out /*[M,N]*/) {
    orc_quant_act(x, is_bf16, M, K, ldx, q, K, a_scale, 0);
    orc_matmul_i32(q, M, K, K, w, N, acc);
    orc_dequant(acc, M, N, w_scale, a_scale, out);
}

/* ------------------------------------------------------------------ */
/* The paper's table-lookup kernels, as second derivations of acc      */
/* ------------------------------------------------------------------ */

/*
 * TL1 kernel (Section 2, Table 2).  For each pair of activations
 * (q[2p], q[2p+1]) the 3^2 = 9 possible partial sums are precomputed into an
 * int16 table addressed by the 4-bit index of the weight pair; the product
 * is then lookups and additions only.  Odd K is padded with one zero weight
 * and one zero activation.  Must equal orc_matmul_i32 exactly.
 * Single row of activations (a GEMV), as in the paper.
 */
void orc_tl1_gemv_i32(const int8_t *q, int64_t K, const int8_t *w, int64_t N, int32_t *acc) {
    int64_t pairs = (K + 1) / 2;
    for (int64_t n = 0; n < N; ++n) acc[n] = 0;
    for (int64_t p = 0; p < pairs; ++p) {
        int q0 = q[2 * p];
        int q1 = (2 * p + 1 < K) ? q[2 * p + 1] : 0;
        int16_t lut[9];
        for (int a = -1; a <= 1; ++a)
            for (int b = -1; b <= 1; ++b)
                lut[orc_tl1_index(a, b)] = (int16_t)(a * q0 + b * q1);
        for (int64_t n = 0; n < N; ++n) {
            int w0 = w[n * K + 2 * p];
            int w1 = (2 * p + 1 < K) ? w[n * K + 2 * p + 1] : 0;
            acc[n] += lut[orc_tl1_index(w0, w1)];
        }
    }
}

/*
 * TL2 kernel (Section 2, Table 3).  Groups of three weights; the table holds
 * the 14 partial sums for index 0..13 (the non-negative half of the 27
 * combinations) and the sign bit negates the looked-up value.  K is padded
 * with zeros to a multiple of 3.  Must equal orc_matmul_i32 exactly.
 */
void orc_tl2_gemv_i32(const int8_t *q, int64_t K, const int8_t *w, int64_t N, int32_t *acc) {
    int64_t groups = (K + 2) / 3;
    for (int64_t n = 0; n < N; ++n) acc[n] = 0;
    for (int64_t g = 0; g < groups; ++g) {
        int qv[3];
        for (int j = 0; j < 3; ++j) qv[j] = (3 * g + j < K) ? q[3 * g + j] : 0;
        int16_t lut[14];
        for (int a = -1; a <= 1; ++a)
            for (int b = -1; b <= 1; ++b)
                for (int c = -1; c <= 1; ++c) {
                    int sign, idx;
                    orc_tl2_code(a, b, c, &sign, &idx);
                    if (!sign) lut[idx] = (int16_t)(a * qv[0] + b * qv[1] + c * qv[2]);
                }
        for (int64_t n = 0; n < N; ++n) {
            int wv[3];
            for (int j = 0; j < 3; ++j) wv[j] = (3 * g + j < K) ? w[n * K + 3 * g + j] : 0;
            int sign, idx;
            orc_tl2_code(wv[0], wv[1], wv[2], &sign, &idx);
            acc[n] += sign ? -lut[idx] : lut[idx];
        }
    }
}

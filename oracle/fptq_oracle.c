/*
 * CPU oracle for the statically quantized INT4 x INT4 linear layer of FPTQuant.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the tests, the smoke check
 * and the benchmark's cpu_baseline leg may call it.  It shares no code with the
 * HIP library and is deliberately plain: straight loops, no blocking, no
 * intrinsics, no BLAS.  OpenMP only spreads independent token rows over cores.
 *
 * What it computes, and where the paper fixes it:
 *   row scale   S = 1 / ||x||_R, ||x||_R = sqrt(mean_k x_k^2)      Sec. 3.1.3, Step 1
 *   quantizer   q = clamp(round(x * S / s_a), -8, 7), static s_a    App. B "Static quantization"
 *   integer GEMM with a 32-bit accumulator on 4-bit operands        App. J "Setup"
 *   epilogue    y = acc * s_a * s_w[o], the float scale factors
 *               applied after the integer matmul                    App. B "Static quantization"
 *   storage     two 4-bit values per byte                           App. J "Setup"
 *
 * The paper is silent on the exact floating-point recipe; the reading taken here
 * (and by the HIP library, independently) is:
 *   - sum of squares accumulated in fp64, sequentially over k
 *   - S_t = (float)(1.0 / sqrt(ss / K + eps))
 *   - inv = 1.0f / s_a            (one fp32 division)
 *   - c_t = S_t * inv             (one fp32 multiply; for no row scale c_t = inv)
 *   - u   = (float)x * c_t        (one fp32 multiply, no contraction)
 *   - q   = clamp(rintf(u), -8, 7) with ties to even; NaN -> 0
 *   - cw  = s_a * s_w[o] (fp32);  yf = (float)acc * cw;  optional yf *= d_t;
 *     y = bf16 round-to-nearest-even of yf
 * Canonical packing: byte j of a row = (v[2j] & 15) | ((v[2j+1] & 15) << 4).
 *
 * Build: gcc -O3 -march=x86-64-v3 -ffp-contract=off -fopenmp -shared -fPIC
 */
#include <math.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_MODE_NONE 0
#define ORACLE_MODE_RMS 1
#define ORACLE_MODE_GIVEN 2

static inline float bf16_bits_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

static inline uint16_t f32_to_bf16_bits_rne(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7fffffffu) > 0x7f800000u) /* NaN: keep it a quiet NaN */
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    return (uint16_t)(u >> 16);
}

/* exported scalar helpers so the tests can pin the conversions one value at a time */
float oracle_bf16_to_f32(uint16_t h) { return bf16_bits_to_f32(h); }
uint16_t oracle_f32_to_bf16(float f) { return f32_to_bf16_bits_rne(f); }

/* Sec. 3.1.3 Step 1: S_t = 1 / RMS(x_t).  mode NONE -> 1, GIVEN -> copy. */
int oracle_row_scale(const uint16_t *x, int64_t M, int64_t K, int mode, float eps,
                     const float *row_scale_in, float *row_scale_out)
{
    if (mode == ORACLE_MODE_NONE) {
        for (int64_t t = 0; t < M; ++t) row_scale_out[t] = 1.0f;
        return 0;
    }
    if (mode == ORACLE_MODE_GIVEN) {
        for (int64_t t = 0; t < M; ++t) row_scale_out[t] = row_scale_in[t];
        return 0;
    }
    if (mode != ORACLE_MODE_RMS) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < M; ++t) {
        const uint16_t *row = x + t * K;
        double ss = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            double v = (double)bf16_bits_to_f32(row[k]);
            ss += v * v;
        }
        row_scale_out[t] = (float)(1.0 / sqrt(ss / (double)K + (double)eps));
    }
    return 0;
}

/* the scalar quantizer, also exported so that it can be brute-forced */
static inline int8_t quantize_one(float x, float c)
{
    float u = x * c;
    if (u != u) return 0;
    float r = rintf(u); /* default rounding mode: nearest, ties to even */
    if (r < -8.0f) r = -8.0f;
    if (r > 7.0f) r = 7.0f;
    return (int8_t)r;
}

int8_t oracle_quantize_scalar(uint16_t x_bf16, float c) { return quantize_one(bf16_bits_to_f32(x_bf16), c); }

/* combined per-row multiplier c_t = S_t * (1 / s_a); exported for the same reason */
float oracle_row_multiplier(float row_scale, float s_a, int has_row_scale)
{
    float inv = 1.0f / s_a;
    return has_row_scale ? row_scale * inv : inv;
}

/* App. B static quantization on the row-scaled input: one int8 per element, values in [-8, 7].
 * row_scale == NULL means no row scale. */
int oracle_quantize(const uint16_t *x, int64_t M, int64_t K, const float *row_scale, float s_a, int8_t *q)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < M; ++t) {
        float c = oracle_row_multiplier(row_scale ? row_scale[t] : 1.0f, s_a, row_scale != NULL);
        for (int64_t k = 0; k < K; ++k) q[t * K + k] = quantize_one(bf16_bits_to_f32(x[t * K + k]), c);
    }
    return 0;
}

/* App. J: two 4-bit values per byte; even index in the low nibble */
int oracle_pack(const int8_t *v, int64_t rows, int64_t K, uint8_t *packed)
{
    if (K % 2) return -1;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t j = 0; j < K / 2; ++j) {
            uint8_t lo = (uint8_t)v[r * K + 2 * j] & 15u;
            uint8_t hi = (uint8_t)v[r * K + 2 * j + 1] & 15u;
            packed[r * (K / 2) + j] = (uint8_t)(lo | (hi << 4));
        }
    return 0;
}

int oracle_unpack(const uint8_t *packed, int64_t rows, int64_t K, int8_t *v)
{
    if (K % 2) return -1;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t j = 0; j < K / 2; ++j) {
            uint8_t b = packed[r * (K / 2) + j];
            int lo = b & 15, hi = b >> 4;
            v[r * K + 2 * j] = (int8_t)(lo >= 8 ? lo - 16 : lo);
            v[r * K + 2 * j + 1] = (int8_t)(hi >= 8 ? hi - 16 : hi);
        }
    return 0;
}

/* App. J integer matmul, checked build: 64-bit accumulation, then the assertion that the
 * 32-bit accumulator the method assumes would have held it.  Returns the number of
 * accumulators that do not fit int32 (0 expected). q [M x K], w [N x K], acc [M x N]. */
int64_t oracle_gemm_i64(const int8_t *q, const int8_t *w, int64_t M, int64_t N, int64_t K, int64_t *acc)
{
    int64_t bad = 0;
#pragma omp parallel for schedule(static) reduction(+ : bad)
    for (int64_t t = 0; t < M; ++t)
        for (int64_t o = 0; o < N; ++o) {
            int64_t s = 0;
            for (int64_t k = 0; k < K; ++k) s += (int64_t)q[t * K + k] * (int64_t)w[o * K + k];
            acc[t * N + o] = s;
            if (s > INT32_MAX || s < INT32_MIN) ++bad;
        }
    return bad;
}

/* Same matmul with the 32-bit accumulator the paper names; this is the build that is timed. */
int oracle_gemm_i32(const int8_t *q, const int8_t *w, int64_t M, int64_t N, int64_t K, int32_t *acc)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < M; ++t)
        for (int64_t o = 0; o < N; ++o) {
            int32_t s = 0;
            for (int64_t k = 0; k < K; ++k) s += (int32_t)q[t * K + k] * (int32_t)w[o * K + k];
            acc[t * N + o] = s;
        }
    return 0;
}

/* Selected outputs only: acc[i] = <q[rows[i], :], w[cols[i], :]> in 64 bits.  Lets the tests
 * check sampled entries of a result too large to recompute whole. */
int oracle_gemm_i64_samples(const int8_t *q, const int8_t *w, int64_t K, const int64_t *rows, const int64_t *cols,
                            int64_t n_samples, int64_t *acc)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_samples; ++i) {
        const int8_t *a = q + rows[i] * K, *b = w + cols[i] * K;
        int64_t s = 0;
        for (int64_t k = 0; k < K; ++k) s += (int64_t)a[k] * (int64_t)b[k];
        acc[i] = s;
    }
    return 0;
}

/* App. B: float scale factors after the integer matmul.  row_out_scale may be NULL. */
int oracle_epilogue(const int32_t *acc, int64_t M, int64_t N, float s_a, const float *s_w, const float *row_out_scale,
                    uint16_t *y_bf16)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < M; ++t)
        for (int64_t o = 0; o < N; ++o) {
            float cw = s_a * s_w[o];
            float yf = (float)acc[t * N + o] * cw;
            if (row_out_scale) yf = yf * row_out_scale[t];
            y_bf16[t * N + o] = f32_to_bf16_bits_rne(yf);
        }
    return 0;
}

/* App. D "Hadamard non-powers of 2": the online transform in front of the down projection is a
 * block-wise Walsh-Hadamard transform, H_B = kron of [[1, 1], [1, -1]], applied to consecutive
 * blocks of B = 2^n channels and scaled by 1 / sqrt(B).  Evaluated here by the textbook in-place
 * butterfly network in fp32, strides h = B/2, B/4, ..., 1, each pair (a, b) -> (a + b, a - b).
 * The result is the unnormalised transform; the 1 / sqrt(B) goes into the quantizer's multiplier. */
static void fwht_block_f32(float *x, int64_t B)
{
    for (int64_t h = B / 2; h >= 1; h /= 2)
        for (int64_t i = 0; i < B; i += 2 * h)
            for (int64_t j = i; j < i + h; ++j) {
                float a = x[j], b = x[j + h];
                x[j] = a + b;
                x[j + h] = a - b;
            }
}

int oracle_hadamard_rows(const uint16_t *x, int64_t M, int64_t K, int64_t B, float *out)
{
    if (B < 1 || (B & (B - 1)) || K % B) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < M; ++t) {
        float *row = out + t * K;
        for (int64_t k = 0; k < K; ++k) row[k] = bf16_bits_to_f32(x[t * K + k]);
        for (int64_t k0 = 0; k0 < K; k0 += B) fwht_block_f32(row + k0, B);
    }
    return 0;
}

/* multiplier of the Hadamard path: c_t = (S_t * (1 / s_a)) * (float)(1 / sqrt(B)), two fp32 products */
float oracle_hadamard_multiplier(float row_scale, float s_a, int has_row_scale, int64_t B)
{
    float hn = (float)(1.0 / sqrt((double)B));
    return oracle_row_multiplier(row_scale, s_a, has_row_scale) * hn;
}

/* Hadamard, then the static quantizer: q = clamp(rne(h * c_t), -8, 7) on the transformed row.
 * h [M x K] fp32 is what oracle_hadamard_rows produced. */
int oracle_quantize_f32(const float *h, int64_t M, int64_t K, const float *row_scale, float s_a, int64_t B, int8_t *q)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < M; ++t) {
        float c = oracle_hadamard_multiplier(row_scale ? row_scale[t] : 1.0f, s_a, row_scale != NULL, B);
        for (int64_t k = 0; k < K; ++k) q[t * K + k] = quantize_one(h[t * K + k], c);
    }
    return 0;
}

/* Asymmetric static grid (App. D: scale and offset of every quantizer are parameters): the
 * integer code is shifted by a zero point z before clamping, v = clamp(rne(x * c) + z, -8, 7), and
 * represents s_a * (v - z).  NaN maps to the code of zero.  z = 0 is the symmetric quantizer. */
static inline int8_t quantize_one_zp(float x, float c, int zp)
{
    float u = x * c;
    if (u != u) return (int8_t)zp;
    float r = rintf(u) + (float)zp;
    if (r < -8.0f) r = -8.0f;
    if (r > 7.0f) r = 7.0f;
    return (int8_t)r;
}

int8_t oracle_quantize_scalar_zp(uint16_t x_bf16, float c, int zp) { return quantize_one_zp(bf16_bits_to_f32(x_bf16), c, zp); }

int oracle_quantize_zp(const uint16_t *x, int64_t M, int64_t K, const float *row_scale, float s_a, int zp, int8_t *q)
{
    if (zp < -8 || zp > 7) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < M; ++t) {
        float c = oracle_row_multiplier(row_scale ? row_scale[t] : 1.0f, s_a, row_scale != NULL);
        for (int64_t k = 0; k < K; ++k) q[t * K + k] = quantize_one_zp(bf16_bits_to_f32(x[t * K + k]), c, zp);
    }
    return 0;
}

/* sum_k w[o, k] per output channel: what the zero point multiplies in the epilogue */
int oracle_weight_row_sums(const int8_t *w, int64_t N, int64_t K, int32_t *sums)
{
    for (int64_t o = 0; o < N; ++o) {
        int64_t s = 0;
        for (int64_t k = 0; k < K; ++k) s += w[o * K + k];
        sums[o] = (int32_t)s;
    }
    return 0;
}

/* Epilogue with the zero point removed: sum_k (v - z) w = acc - z * wsum[o], then the float scales. */
int oracle_epilogue_zp(const int32_t *acc, int64_t M, int64_t N, float s_a, const float *s_w, const float *row_out_scale,
                       int zp, const int32_t *w_row_sum, uint16_t *y_bf16)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < M; ++t)
        for (int64_t o = 0; o < N; ++o) {
            int32_t a = acc[t * N + o] - (int32_t)zp * w_row_sum[o];
            float cw = s_a * s_w[o];
            float yf = (float)a * cw;
            if (row_out_scale) yf = yf * row_out_scale[t];
            y_bf16[t * N + o] = f32_to_bf16_bits_rne(yf);
        }
    return 0;
}

/* Sec. 3.1.3, Eq. (5)-(7): one step of the scaled residual stream, fused with the quantizer of
 * the next block's input.  Given the scaled residual X~_{n-1}, the scaled block output Y~_{n-1}
 * and S_{n-1}:  Z~ = X~ + Y~,  nrm = RMS(Z~),  S_n = S_{n-1} / nrm,  X~_n = Z~ / nrm (unit RMS:
 * at once the new residual and the gain-free RMSNorm output), q = quantizer(X~_n / s_a).
 * fp32 recipe: z = (float)x + (float)y; sum of z^2 in fp64; inv = (float)(1 / sqrt(ss / K + eps));
 * S_n = S_{n-1} * inv; X~_n = bf16(z * inv); c = inv * (1.0f / s_a); q = clamp(rne(z * c), -8, 7). */
int oracle_residual_norm_quantize(const uint16_t *x_res, const uint16_t *y_blk, int64_t M, int64_t K, const float *s_prev,
                                  float eps, float s_a, uint16_t *x_next, float *s_next, int8_t *q)
{
    float inv_sa = 1.0f / s_a;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < M; ++t) {
        double ss = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            float z = bf16_bits_to_f32(x_res[t * K + k]) + bf16_bits_to_f32(y_blk[t * K + k]);
            ss += (double)z * (double)z;
        }
        float inv = (float)(1.0 / sqrt(ss / (double)K + (double)eps));
        s_next[t] = (s_prev ? s_prev[t] : 1.0f) * inv;
        float c = inv * inv_sa;
        for (int64_t k = 0; k < K; ++k) {
            float z = bf16_bits_to_f32(x_res[t * K + k]) + bf16_bits_to_f32(y_blk[t * K + k]);
            x_next[t * K + k] = f32_to_bf16_bits_rne(z * inv);
            q[t * K + k] = quantize_one(z, c);
        }
    }
    return 0;
}

/* App. B "Dynamic quantization": the scale factor is computed at run time for each token
 * independently, from that token's range.  With the symmetric 4-bit grid: s_t = max_k |x_t,k| / 7,
 * q = clamp(rne(x * (1 / s_t)), -8, 7).  NaNs do not enter the maximum; an all-zero (or infinite)
 * row gets s_t = 1.  Arithmetic in fp32: one division for s_t, one for its reciprocal, one
 * multiply per element. */
int oracle_quantize_dynamic(const uint16_t *x, int64_t M, int64_t K, float *s_out, int8_t *q)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < M; ++t) {
        float amax = 0.0f;
        for (int64_t k = 0; k < K; ++k) {
            float v = fabsf(bf16_bits_to_f32(x[t * K + k]));
            if (v == v && v > amax) amax = v;
        }
        float s = (amax > 0.0f && amax < INFINITY) ? amax / 7.0f : 1.0f;
        float c = 1.0f / s;
        s_out[t] = s;
        for (int64_t k = 0; k < K; ++k) q[t * K + k] = quantize_one(bf16_bits_to_f32(x[t * K + k]), c);
    }
    return 0;
}

/* Whole path for the timed baseline: row scale -> quantize -> int32 GEMM -> epilogue.
 * Scratch (q [M x K] int8, acc [M x N] int32, r [M] float) is the caller's. */
int oracle_w4a4_linear(const uint16_t *x, const int8_t *w, int64_t M, int64_t N, int64_t K, int mode, float eps,
                       const float *row_scale_in, float s_a, const float *s_w, const float *row_out_scale, float *r,
                       int8_t *q, int32_t *acc, uint16_t *y_bf16)
{
    int rc = oracle_row_scale(x, M, K, mode, eps, row_scale_in, r);
    if (rc) return rc;
    oracle_quantize(x, M, K, mode == ORACLE_MODE_NONE ? NULL : r, s_a, q);
    oracle_gemm_i32(q, w, M, N, K, acc);
    return oracle_epilogue(acc, M, N, s_a, s_w, row_out_scale, y_bf16);
}

int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp single
        n = omp_get_num_threads();
    }
#endif
    return n;
}

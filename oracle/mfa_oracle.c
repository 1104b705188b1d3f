/*
 * CPU oracle for decode-step Multi-Matrix Factorization Attention (MFA).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, fp64
 * statement of what the GPU library must compute.  Only the tests, the smoke
 * check and the cpu_baseline leg of the benchmark may call it.  It shares no
 * code, header, table or constant with the HIP path.
 *
 * What is computed (paper, Section 2 "Model Card" and its model-card table):
 *   - 64 query heads of dimension 256 attend over ONE shared key head and ONE
 *     shared value head of the same dimension (multi-query softmax attention,
 *     one query token per sequence at decode time);
 *   - the query comes from a low-rank factorisation: the hidden state is
 *     down-projected 7168 -> 2048, normalised, and up-projected to 64*256.
 *   - each GPU serves a batch of independent sequences (Section 7.1, local
 *     data-parallel attention), so sequences never interact.
 *   - the cache holds one key row and one value row per token (Section 6:
 *     512 bytes per token at 8 bits = 256 key + 256 value elements).
 *
 * The paper fixes neither the softmax scale, the kind of normalisation, the
 * fp8 flavour nor the scale granularity; the readings taken here are
 *   scale: runtime float (1/16 for head dim 256);
 *   normalisation: RMSNorm, eps added to the mean square inside the root;
 *   fp8: OCP e4m3fn (bias 7, no infinity, 0x7F/0xFF are NaN, subnormals kept);
 *   one fp32 dequantisation scale per cached token per tensor;
 *   4-bit storage (Section 5.2 discusses keeping the cache in 4 bits and
 *   computing in 8; it names no format): OCP e2m1 elements (1 sign, 2 exponent
 *   bits with bias 1, 1 fraction bit, subnormal kept, no infinity or NaN),
 *   two per byte with the even element in the low four bits, and the same one
 *   fp32 scale per token per tensor as the 8-bit record.
 *
 * Every floating point sum is carried in double.  Nothing is tiled, fused or
 * reordered: scores, maximum, exponentials, normaliser and weighted sum are
 * separate passes over the tokens in index order.
 *
 * Parity pins (tests/test_oracle_*.py): brute force in numpy, weights sum to
 * one, context length one returns the value row, permuted page table equals
 * contiguous cache, zero query returns the mean value row, key-shift and
 * token-permutation invariance, split/merge identity through the returned
 * log-sum-exp, torch fp64 scaled_dot_product_attention / rms_norm / matmul,
 * exhaustive bf16 and e4m3fn code tables against torch's CPU casts.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_API __attribute__((visibility("default")))

enum { ORACLE_KV_BF16 = 0, ORACLE_KV_E4M3 = 1, ORACLE_KV_E2M1 = 2 };

/* ------------------------------------------------------------------ */
/* Storage formats, decoded field by field.                            */
/* ------------------------------------------------------------------ */

/* bfloat16: 1 sign, 8 exponent (bias 127), 7 fraction bits. */
static double decode_bf16(uint16_t bits)
{
    int sign = (bits >> 15) & 1;
    int expo = (bits >> 7) & 0xFF;
    int frac = bits & 0x7F;
    double mag;
    if (expo == 0xFF)
        mag = frac ? NAN : INFINITY;
    else if (expo == 0)
        mag = ldexp((double)frac, -126 - 7);             /* subnormal */
    else
        mag = ldexp((double)(128 + frac), expo - 127 - 7);
    return sign ? -mag : mag;
}

/* OCP e4m3fn: 1 sign, 4 exponent (bias 7), 3 fraction bits; no infinity;
 * exponent 15 with fraction 7 is NaN, every other code is finite (max 448). */
static double decode_e4m3fn(uint8_t bits)
{
    int sign = (bits >> 7) & 1;
    int expo = (bits >> 3) & 0xF;
    int frac = bits & 0x7;
    double mag;
    if (expo == 0xF && frac == 0x7)
        mag = NAN;
    else if (expo == 0)
        mag = ldexp((double)frac, -6 - 3);               /* subnormal */
    else
        mag = ldexp((double)(8 + frac), expo - 7 - 3);
    return sign ? -mag : mag;
}

/* double -> bfloat16, round to nearest, ties to even, done directly on the
 * double so that no intermediate float rounding happens. */
static uint16_t encode_bf16_rne(double x)
{
    uint16_t sign = signbit(x) ? 0x8000u : 0;
    if (isnan(x)) return (uint16_t)(sign | 0x7FC0u);
    double a = fabs(x);
    if (isinf(a)) return (uint16_t)(sign | 0x7F80u);
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);              /* a = f * 2^e, f in [0.5, 1)  */
    int expo = e - 1;                /* a = 1.xxx * 2^expo          */
    if (expo < -126) expo = -126;    /* subnormal range: fixed quantum */
    /* quantum of the target grid at this exponent is 2^(expo-7) */
    double scaled = ldexp(a, 7 - expo);          /* exact */
    double r = nearbyint(scaled);                /* default mode: ties-to-even */
    /* r in [0, 256]; value = r * 2^(expo-7) */
    long mant = (long)r;
    long biased;
    if (expo == -126 && mant < 128) {
        biased = 0;                              /* stays subnormal */
    } else {
        biased = expo + 127;
        if (mant == 256) { mant = 128; biased += 1; }
        mant -= 128;
    }
    if (biased >= 255) return (uint16_t)(sign | 0x7F80u);   /* overflow -> inf */
    return (uint16_t)(sign | (uint16_t)(biased << 7) | (uint16_t)mant);
}

ORACLE_API double mfa_oracle_decode_bf16(uint16_t bits)   { return decode_bf16(bits); }
/* e2m1 ("fp4"): 1 sign, 2 exponent bits (bias 1), 1 fraction bit.  Exponent field 0 is the
 * subnormal binade (0 and 0.5); every code is a finite number. */
static double decode_e2m1(uint8_t code)
{
    int sign = (code >> 3) & 1;
    int expo = (code >> 1) & 3;
    int frac = code & 1;
    double mag = expo == 0 ? 0.5 * (double)frac : ldexp(1.0 + 0.5 * (double)frac, expo - 1);
    return sign ? -mag : mag;
}

ORACLE_API double mfa_oracle_decode_e4m3fn(uint8_t bits)  { return decode_e4m3fn(bits); }
ORACLE_API double mfa_oracle_decode_e2m1(uint8_t code)    { return decode_e2m1(code & 15); }
ORACLE_API uint16_t mfa_oracle_encode_bf16(double x)      { return encode_bf16_rne(x); }

/* ------------------------------------------------------------------ */
/* Threads.                                                            */
/* ------------------------------------------------------------------ */
static int g_threads = 0;   /* 0 = OpenMP default */

ORACLE_API void mfa_oracle_set_threads(int n) { g_threads = n > 0 ? n : 0; }

ORACLE_API int mfa_oracle_get_threads(void)
{
#ifdef _OPENMP
    return g_threads > 0 ? g_threads : omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ */
/* One cached row (key or value) of one token, dequantised to double.  */
/* ------------------------------------------------------------------ */
typedef struct {
    const void  *k, *v;            /* cache or pool base                         */
    const float *k_scale, *v_scale;/* per-token scales (fp8 only)                */
    int          kv_dtype;
    int          D;
    /* contiguous: token j of sequence b is row b*seq_stride_tokens + j          */
    int64_t      seq_stride_tokens;
    /* paged: token j of sequence b is row block_table[b][j/page]*page + j%page  */
    const int32_t *block_table;
    int32_t      max_blocks_per_seq;
    int32_t      page_size;
} kv_view;

static int64_t token_row(const kv_view *kv, int b, int j)
{
    if (kv->block_table) {
        int32_t page = kv->block_table[(int64_t)b * kv->max_blocks_per_seq + j / kv->page_size];
        return (int64_t)page * kv->page_size + j % kv->page_size;
    }
    return (int64_t)b * kv->seq_stride_tokens + j;
}

static double kv_elem(const kv_view *kv, const void *base, const float *scale, int64_t row, int d)
{
    if (kv->kv_dtype == ORACLE_KV_BF16)
        return decode_bf16(((const uint16_t *)base)[row * kv->D + d]);
    if (kv->kv_dtype == ORACLE_KV_E2M1) {
        /* D/2 bytes per row; element d in byte d/2, low four bits when d is even */
        uint8_t byte = ((const uint8_t *)base)[row * (kv->D / 2) + d / 2];
        return (double)scale[row] * decode_e2m1((d & 1) ? (byte >> 4) : (byte & 15));
    }
    return (double)scale[row] * decode_e4m3fn(((const uint8_t *)base)[row * kv->D + d]);
}

/* ------------------------------------------------------------------ */
/* Softmax attention of one query row over the L cached tokens of its  */
/* sequence: the textbook definition in three passes.                  */
/*   s_j = scale * <q, k_j>;  p_j = exp(s_j - max s);  Z = sum p_j;     */
/*   out_d = sum_j p_j v_{j,d} / Z;  lse = max s + log Z.               */
/* weights (optional, length L) receives p_j / Z.                      */
/* ------------------------------------------------------------------ */
static void attend_one(const uint16_t *q_row, const kv_view *kv, int b, int L, double scale,
                       float *out_row, double *lse, double *weights)
{
    const int D = kv->D;
    if (L <= 0) {
        for (int d = 0; d < D; ++d) out_row[d] = 0.0f;
        if (lse) *lse = -INFINITY;
        return;
    }
    double *s = (double *)malloc(sizeof(double) * (size_t)L);
    double *qd = (double *)malloc(sizeof(double) * (size_t)D);
    double *acc = (double *)malloc(sizeof(double) * (size_t)D);
    for (int d = 0; d < D; ++d) qd[d] = decode_bf16(q_row[d]);

    for (int j = 0; j < L; ++j) {
        int64_t row = token_row(kv, b, j);
        double dot = 0.0;
        for (int d = 0; d < D; ++d) dot += qd[d] * kv_elem(kv, kv->k, kv->k_scale, row, d);
        s[j] = scale * dot;
    }
    double m = s[0];
    for (int j = 1; j < L; ++j) if (s[j] > m) m = s[j];
    double Z = 0.0;
    for (int j = 0; j < L; ++j) { s[j] = exp(s[j] - m); Z += s[j]; }

    for (int d = 0; d < D; ++d) acc[d] = 0.0;
    for (int j = 0; j < L; ++j) {
        int64_t row = token_row(kv, b, j);
        for (int d = 0; d < D; ++d) acc[d] += s[j] * kv_elem(kv, kv->v, kv->v_scale, row, d);
    }
    for (int d = 0; d < D; ++d) out_row[d] = (float)(acc[d] / Z);
    if (lse) *lse = m + log(Z);
    if (weights) for (int j = 0; j < L; ++j) weights[j] = s[j] / Z;
    free(s); free(qd); free(acc);
}

/* Rows to compute: either every (b,h) pair, or the n_rows pairs listed in
 * row_b/row_h (used to sample full-size workloads).  Output row r goes to
 * out + r*D (and lse[r]). */
static int run_rows(const uint16_t *q, const kv_view *kv, const int32_t *seq_lens,
                    int B, int H, double scale,
                    int64_t n_rows, const int32_t *row_b, const int32_t *row_h,
                    float *out, double *lse)
{
    const int D = kv->D;
    int64_t total = row_b ? n_rows : (int64_t)B * H;
    int nthreads = mfa_oracle_get_threads();
    (void)nthreads;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
    for (int64_t r = 0; r < total; ++r) {
        int b = row_b ? row_b[r] : (int)(r / H);
        int h = row_b ? row_h[r] : (int)(r % H);
        attend_one(q + ((int64_t)b * H + h) * D, kv, b, seq_lens[b], scale,
                   out + r * D, lse ? lse + r : NULL, NULL);
    }
    return 0;
}

/* Contiguous cache.  q: bf16 [B,H,D]; k,v: [B, seq_stride_tokens, D] in
 * kv_dtype; k_scale,v_scale: fp32 [B, seq_stride_tokens] (fp8 only);
 * out: fp32 [rows, D]; lse: double [rows] or NULL. */
ORACLE_API int mfa_oracle_decode_attn(const uint16_t *q, const void *k, const void *v,
                                      const float *k_scale, const float *v_scale, int kv_dtype,
                                      int64_t seq_stride_tokens, const int32_t *seq_lens,
                                      int B, int H, int D, double scale,
                                      int64_t n_rows, const int32_t *row_b, const int32_t *row_h,
                                      float *out, double *lse)
{
    if (kv_dtype != ORACLE_KV_BF16 && kv_dtype != ORACLE_KV_E4M3 && kv_dtype != ORACLE_KV_E2M1) return 1;
    if (kv_dtype != ORACLE_KV_BF16 && (!k_scale || !v_scale)) return 1;
    if (kv_dtype == ORACLE_KV_E2M1 && (D & 1)) return 1;
    kv_view kv = { k, v, k_scale, v_scale, kv_dtype, D, seq_stride_tokens, NULL, 0, 0 };
    return run_rows(q, &kv, seq_lens, B, H, scale, n_rows, row_b, row_h, out, lse);
}

/* Paged cache.  k_pool,v_pool: [n_pages, page_size, D]; scale pools fp32
 * [n_pages, page_size]; block_table: int32 [B, max_blocks_per_seq]. */
ORACLE_API int mfa_oracle_decode_attn_paged(const uint16_t *q, const void *k_pool, const void *v_pool,
                                            const float *k_scale_pool, const float *v_scale_pool,
                                            int kv_dtype, int32_t page_size,
                                            const int32_t *block_table, int32_t max_blocks_per_seq,
                                            const int32_t *seq_lens, int B, int H, int D, double scale,
                                            int64_t n_rows, const int32_t *row_b, const int32_t *row_h,
                                            float *out, double *lse)
{
    if (kv_dtype != ORACLE_KV_BF16 && kv_dtype != ORACLE_KV_E4M3 && kv_dtype != ORACLE_KV_E2M1) return 1;
    if (kv_dtype != ORACLE_KV_BF16 && (!k_scale_pool || !v_scale_pool)) return 1;
    if (kv_dtype == ORACLE_KV_E2M1 && (D & 1)) return 1;
    if (!block_table || page_size <= 0) return 1;
    kv_view kv = { k_pool, v_pool, k_scale_pool, v_scale_pool, kv_dtype, D, 0,
                   block_table, max_blocks_per_seq, page_size };
    return run_rows(q, &kv, seq_lens, B, H, scale, n_rows, row_b, row_h, out, lse);
}

/* Attention weights p_j / Z of one (b,h) row over a contiguous bf16/fp8 cache
 * (for the rows-sum-to-one pin). weights: double [seq_lens[b]]. */
ORACLE_API int mfa_oracle_attn_weights(const uint16_t *q, const void *k, const void *v,
                                       const float *k_scale, const float *v_scale, int kv_dtype,
                                       int64_t seq_stride_tokens, const int32_t *seq_lens,
                                       int H, int D, double scale, int b, int h,
                                       double *weights, float *out_row)
{
    kv_view kv = { k, v, k_scale, v_scale, kv_dtype, D, seq_stride_tokens, NULL, 0, 0 };
    attend_one(q + ((int64_t)b * H + h) * D, &kv, b, seq_lens[b], scale, out_row, NULL, weights);
    return 0;
}

/* ------------------------------------------------------------------ */
/* Low-rank query path (Section 2): c = x W_qa;                        */
/* c_hat = c / sqrt(mean(c^2) + eps) * gain;  q = c_hat W_qb.          */
/* x: bf16 [B, d_model]; w_qa: bf16 [d_model, r]; gain: fp32 [r] or     */
/* NULL (unit); w_qb: bf16 [r, n_out].  Everything between the inputs   */
/* and the stored query stays in double; the only rounding is the final */
/* one to the bf16 storage type.  q_bf16: [B, n_out] (may be NULL);     */
/* q_f64: [B, n_out] unrounded (may be NULL); c_hat_f64: [B, r] (may be */
/* NULL).                                                               */
/* ------------------------------------------------------------------ */
ORACLE_API int mfa_oracle_query_proj(const uint16_t *x, const uint16_t *w_qa, const float *gain,
                                     const uint16_t *w_qb, int B, int d_model, int r, int n_out,
                                     double eps, uint16_t *q_bf16, double *q_f64, double *c_hat_f64)
{
    int nthreads = mfa_oracle_get_threads();
    (void)nthreads;
    double *wa = (double *)malloc(sizeof(double) * (size_t)d_model * r);
    double *wb = (double *)malloc(sizeof(double) * (size_t)r * n_out);
    if (!wa || !wb) { free(wa); free(wb); return 2; }
    for (int64_t i = 0; i < (int64_t)d_model * r; ++i) wa[i] = decode_bf16(w_qa[i]);
    for (int64_t i = 0; i < (int64_t)r * n_out; ++i) wb[i] = decode_bf16(w_qb[i]);

#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
    for (int b = 0; b < B; ++b) {
        double *c = (double *)calloc((size_t)r, sizeof(double));
        double *qrow = (double *)calloc((size_t)n_out, sizeof(double));
        for (int i = 0; i < d_model; ++i) {
            double xi = decode_bf16(x[(int64_t)b * d_model + i]);
            const double *wrow = wa + (int64_t)i * r;
            for (int j = 0; j < r; ++j) c[j] += xi * wrow[j];
        }
        double ms = 0.0;
        for (int j = 0; j < r; ++j) ms += c[j] * c[j];
        ms /= (double)r;
        double inv = 1.0 / sqrt(ms + eps);
        for (int j = 0; j < r; ++j) {
            c[j] = c[j] * inv * (gain ? (double)gain[j] : 1.0);
            if (c_hat_f64) c_hat_f64[(int64_t)b * r + j] = c[j];
        }
        for (int j = 0; j < r; ++j) {
            const double *wrow = wb + (int64_t)j * n_out;
            double cj = c[j];
            for (int n = 0; n < n_out; ++n) qrow[n] += cj * wrow[n];
        }
        for (int n = 0; n < n_out; ++n) {
            if (q_f64) q_f64[(int64_t)b * n_out + n] = qrow[n];
            if (q_bf16) q_bf16[(int64_t)b * n_out + n] = encode_bf16_rne(qrow[n]);
        }
        free(c); free(qrow);
    }
    free(wa); free(wb);
    return 0;
}

/* ------------------------------------------------------------------ */
/* The linear maps around the attention core and the writing of a new   */
/* token into the cache (Section 6 counts them in the attention layer:  */
/* key and value projections 7168 -> 256 each, output projection        */
/* 64*256 -> 7168; the cache holds 8-bit keys and values).              */
/* ------------------------------------------------------------------ */

/* y = a . w in double.  a: [B, K], bf16 bit patterns (a_is_f32 = 0) or fp32 values (a_is_f32 = 1);
 * w: bf16 [K, N] (in x out); y: double [B, N]. */
ORACLE_API int mfa_oracle_linear(const void *a, int a_is_f32, const uint16_t *w, int B, int K, int N, double *y)
{
    int nthreads = mfa_oracle_get_threads();
    (void)nthreads;
    double *wd = (double *)malloc(sizeof(double) * (size_t)K * N);
    if (!wd) return 2;
    for (int64_t i = 0; i < (int64_t)K * N; ++i) wd[i] = decode_bf16(w[i]);
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
    for (int b = 0; b < B; ++b) {
        double *row = y + (int64_t)b * N;
        for (int n = 0; n < N; ++n) row[n] = 0.0;
        for (int k = 0; k < K; ++k) {
            double ak = a_is_f32 ? (double)((const float *)a)[(int64_t)b * K + k]
                                 : decode_bf16(((const uint16_t *)a)[(int64_t)b * K + k]);
            const double *wrow = wd + (int64_t)k * N;
            for (int n = 0; n < N; ++n) row[n] += ak * wrow[n];
        }
    }
    free(wd);
    return 0;
}

/* Nearest e4m3fn code of a finite float with |x| <= 448, ties to the even code.
 * Normal numbers 2^e (1 + m/8), e = -6..8; below 2^-6 the spacing is 2^-9. */
static uint8_t encode_e4m3fn_rne(float x)
{
    uint8_t sign = (uint8_t)(signbit(x) ? 0x80 : 0x00);
    double a = fabs((double)x);
    if (a >= 448.0) return (uint8_t)(sign | 0x7E);
    if (a < 0.015625) {                              /* subnormal range: code = a / 2^-9, 8 rolls over into 2^-6 */
        double q = nearbyint(a * 512.0);             /* default rounding mode: to nearest, ties to even */
        return (uint8_t)(sign | (uint8_t)q);
    }
    int e;
    double f = frexp(a, &e);                         /* a = f 2^e, f in [0.5, 1) */
    f *= 2.0; e -= 1;                                /* a = f 2^e, f in [1, 2) */
    double m = nearbyint((f - 1.0) * 8.0);           /* 0..8 */
    if (m == 8.0) { m = 0.0; e += 1; }
    if (e > 8 || (e == 8 && m > 6.0)) return (uint8_t)(sign | 0x7E);
    return (uint8_t)(sign | (uint8_t)((e + 7) << 3) | (uint8_t)m);
}

/* Per-token quantisation of cache rows, defined in single precision because floating point
 * decides integer codes here: scale = max(max_d |x_d|, 1e-12) / 448, code_d = e4m3fn(x_d / scale)
 * with the quotient clamped to [-448, 448].  x: fp32 [rows, D]. */
ORACLE_API int mfa_oracle_quantize_rows_e4m3(const float *x, int rows, int D, uint8_t *codes, float *scales)
{
    for (int r = 0; r < rows; ++r) {
        const float *row = x + (int64_t)r * D;
        float amax = 0.0f;
        for (int d = 0; d < D; ++d) amax = fmaxf(amax, fabsf(row[d]));
        volatile float scale = fmaxf(amax, 1e-12f) / 448.0f;
        scales[r] = scale;
        for (int d = 0; d < D; ++d) {
            volatile float y = row[d] / scale;
            float c = y > 448.0f ? 448.0f : (y < -448.0f ? -448.0f : y);
            codes[(int64_t)r * D + d] = encode_e4m3fn_rne(c);
        }
    }
    return 0;
}

/* Nearest e2m1 code of a finite float, ties to the code with an even fraction bit: the eight
 * magnitudes are tried one after the other. */
static uint8_t encode_e2m1_rne(float x)
{
    uint8_t sign = (uint8_t)(signbit(x) ? 8 : 0);
    double a = fabs((double)x);
    uint8_t best = 0;
    double best_err = a;                             /* distance to magnitude 0 */
    for (uint8_t c = 1; c < 8; ++c) {
        double err = fabs(a - decode_e2m1(c));
        if (err < best_err || (err == best_err && (c & 1) == 0)) { best = c; best_err = err; }
    }
    return (uint8_t)(sign | best);
}

/* 4-bit record of cache rows, the 8-bit record's recipe with e2m1's largest magnitude 6 in
 * place of 448: scale = max(max_d |x_d|, 1e-12) / 6, code_d = e2m1(clamp(x_d / scale, -6, 6)),
 * in single precision.  Packed two per byte, even d in the low four bits.  x: fp32 [rows, D],
 * D even; packed: [rows, D/2]. */
ORACLE_API int mfa_oracle_quantize_rows_e2m1(const float *x, int rows, int D, uint8_t *packed, float *scales)
{
    if (D & 1) return 1;
    for (int r = 0; r < rows; ++r) {
        const float *row = x + (int64_t)r * D;
        float amax = 0.0f;
        for (int d = 0; d < D; ++d) amax = fmaxf(amax, fabsf(row[d]));
        volatile float scale = fmaxf(amax, 1e-12f) / 6.0f;
        scales[r] = scale;
        for (int d = 0; d < D; d += 2) {
            uint8_t code[2];
            for (int i = 0; i < 2; ++i) {
                volatile float y = row[d + i] / scale;
                float c = y > 6.0f ? 6.0f : (y < -6.0f ? -6.0f : y);
                code[i] = encode_e2m1_rne(c);
            }
            packed[(int64_t)r * (D / 2) + d / 2] = (uint8_t)(code[0] | (code[1] << 4));
        }
    }
    return 0;
}

/* Round fp32 values to bf16 bit patterns (nearest, ties to even). */
ORACLE_API int mfa_oracle_round_bf16(const float *x, int64_t n, uint16_t *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = encode_bf16_rne((double)x[i]);
    return 0;
}


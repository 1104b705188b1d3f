/*
 * mfa.h - C boundary of the MI355X (gfx950) decode-step Multi-Matrix
 * Factorization Attention (MFA) library.
 *
 * The operation is the attention module of the Step-3 paper (Section 2,
 * "Model Card", and its model-card table): 64 query heads of dimension 256,
 * produced by a low-rank query factorisation (hidden 7168 -> rank 2048 ->
 * normalisation -> 64*256), all attend over ONE shared key head and ONE shared
 * value head of dimension 256.  At decode time every sequence contributes one
 * query token that attends over all tokens cached for that sequence; a GPU
 * serves a batch of independent sequences (Section 7.1, local data-parallel
 * attention).  The cache holds one key row and one value row per token
 * (Section 6: 512 bytes per token at 8 bits).
 *
 * Conventions for every entry point
 *   - Every data pointer is a DEVICE pointer (HIP global memory on the device
 *     given at init) unless marked "host".  All tensors are dense, row-major,
 *     last index fastest, and must be 16-byte aligned.
 *   - The caller owns every buffer, including the workspace handed to
 *     mfa_decode_init; the library allocates no device memory, frees nothing
 *     of the caller's, never synchronises the device or the stream and never
 *     reads device memory from the host.  All work is enqueued on `hip_stream`
 *     (a hipStream_t passed as void*; NULL = the default stream).
 *   - Inputs are only read.  Outputs and the workspace are the only writes.
 *   - Errors are returned as mfa_status; nothing aborts or throws.  Conditions
 *     the host can see (NULL or misaligned pointers, sizes out of range,
 *     unsupported shapes or types, fp8 without scales, workspace too small) are
 *     rejected before anything is launched.  Conditions only the device can see
 *     have defined results instead: seq_lens[b] <= 0 gives out[b,:,:] = 0;
 *     seq_lens[b] > max_seq_len_hint is treated as max_seq_len_hint; a page id
 *     outside [0, n_pages) that an attention call reads is clamped into that
 *     range, one that a cache-append call would write to is skipped (the result
 *     for that sequence is then meaningless, but no memory outside the pools is
 *     touched).
 *   - Memory of the cache past a sequence's length (padding, the rest of the
 *     last page, unused pages) may hold anything, NaN included; it never
 *     influences the result.
 *   - A context is not safe for concurrent calls (they share its workspace);
 *     calls on one context must be ordered on one stream or otherwise
 *     serialised by the caller.  Distinct contexts are independent.
 *   - bf16 is bfloat16 (1-8-7).  fp8 is OCP e4m3fn (1-4-3, bias 7, max 448, no
 *     infinity, 0x7F/0xFF NaN), the native 8-bit float of gfx950.
 */
#ifndef MFA_H
#define MFA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Exported from libmfa.so (the library is built with hidden default visibility). */
#define MFA_API __attribute__((visibility("default")))

typedef struct mfa_ctx mfa_ctx;          /* opaque; made by mfa_decode_init */

typedef enum {
    MFA_OK = 0,
    MFA_ERR_INVALID_ARG = 1,             /* NULL/misaligned pointer, size out of range      */
    MFA_ERR_UNSUPPORTED = 2,             /* shape or type this build has no kernel for      */
    MFA_ERR_WORKSPACE_TOO_SMALL = 3,
    MFA_ERR_HIP = 4,                     /* a HIP runtime call or kernel launch failed      */
    MFA_ERR_HOST_ALLOC = 5               /* host memory for the context could not be had    */
} mfa_status;

/* How the cached tokens of a call are shared out among workgroups (mfa_config.schedule). */
typedef enum {
    MFA_SCHEDULE_BALANCED = 0,           /* tiles of all sequences end to end, equal ranges */
    MFA_SCHEDULE_FIXED = 1               /* every sequence cut into the same number of equal chunks of the hint */
} mfa_schedule;

typedef enum {
    MFA_KV_BF16 = 0,
    MFA_KV_FP8_E4M3 = 1,                 /* one fp32 scale per token per tensor             */
    MFA_KV_FP4_E2M1 = 2                  /* 4-bit elements, two per byte; scales as for fp8 */
} mfa_kv_dtype;

/* Problem description fixed at init (Section 2, model-card table, gives the
 * Step-3 values in the comments). */
typedef struct {
    int32_t n_q_heads;      /* 64; this build supports exactly 64                          */
    int32_t head_dim;       /* 256; this build supports exactly 256                        */
    int32_t d_model;        /* 7168; multiple of 64                                        */
    int32_t q_rank;         /* 2048; multiple of 128                                       */
    float   softmax_scale;  /* multiplies q.k before the softmax; 1/16 for head_dim 256    */
    float   rms_eps;        /* added to the mean square inside the root; 1e-6              */
    int32_t page_size;      /* tokens per cache page; this build supports exactly 64       */
    int32_t max_batch;      /* largest B of any later call (attention and query path)      */
    int32_t max_seq_len;    /* largest max_seq_len_hint of any later call                  */
    int32_t device;         /* HIP device ordinal                                          */
    int32_t target_workgroups; /* workgroups an attention call aims for; 0 = the default, one per
                                  compute unit of MI355X (256); 1..4096                           */
    int32_t schedule;       /* mfa_schedule; MFA_SCHEDULE_BALANCED (0) is the default; batches
                               above 4096 sequences always take MFA_SCHEDULE_FIXED                 */
} mfa_config;
/* Test override: when target_workgroups is 0 / schedule is MFA_SCHEDULE_BALANCED, the environment
 * variables MFA_TARGET_ITEMS=<n> / MFA_SCHEDULE=fixed, read when a context is created, select the
 * same things. */

/* Bytes of device workspace a context for `cfg` needs.  Pure host function;
 * returns 0 if cfg is NULL or invalid. */
MFA_API size_t mfa_decode_workspace_bytes(const mfa_config* cfg);

/* Create a context.  `d_workspace` is device memory of at least
 * mfa_decode_workspace_bytes(cfg) bytes, 256-byte aligned, owned by the caller
 * and kept alive until mfa_decode_destroy.  Launches nothing. */
MFA_API mfa_status mfa_decode_init(const mfa_config* cfg, void* d_workspace, size_t workspace_bytes,
                           mfa_ctx** out_ctx);

/* Free the host-side context (not the workspace).  NULL is allowed. */
MFA_API void mfa_decode_destroy(mfa_ctx* ctx);

/* Static string for a status code. */
MFA_API const char* mfa_status_string(mfa_status s);

/*
 * Low-rank query path (Section 2: the query is down-projected from 7168 to a
 * rank of 2048, normalised, then up-projected to 64*256):
 *     c     = x . W_qa                          [B, q_rank]
 *     c_hat = c / sqrt(mean_j(c_j^2) + rms_eps) * gain
 *     q     = c_hat . W_qb                      [B, n_q_heads*head_dim]
 * The paper says only "a normalization"; RMSNorm is this library's reading.
 *   x        bf16 [B, d_model]
 *   w_qa     bf16 [d_model, q_rank]             (in x out: y = x.W)
 *   rms_gain fp32 [q_rank], or NULL for unit gain
 *   w_qb     bf16 [q_rank, n_q_heads*head_dim]; column h*head_dim + d feeds q[b,h,d]
 *   q_out    bf16 [B, n_q_heads, head_dim]      (written)
 * Products are accumulated in fp32; c_hat is rounded to bf16 before the second
 * product; q is rounded to bf16 once on store.  1 <= B <= max_batch.
 */
MFA_API mfa_status mfa_query_proj(mfa_ctx* ctx, const void* x, const void* w_qa, const float* rms_gain,
                          const void* w_qb, void* q_out, int32_t B, void* hip_stream);

/*
 * Key/value projection of the new token and its cache record (Section 6 counts both
 * 7168 -> 256 projections in the attention layer and has the cache hold one key
 * row and one value row per token, 8 bits per element in the deployed system):
 *     [k_new | v_new] = x . W_kv                     [B, 2*head_dim], fp32 accumulation
 *     bf16 cache: row seq_lens[b] of sequence b  <-  round-to-nearest-even(k_new), (v_new)
 *     fp8 cache:  per token and tensor  scale = max(max_d |x_d|, 1e-12) / 448,
 *                 code_d = e4m3(clamp(x_d / scale, -448, 448)),  scale stored beside the row;
 *                 single precision throughout, so the codes depend on the fp32 row alone
 *     fp4 cache:  the same with 6, e2m1's largest magnitude, in place of 448 and
 *                 code_d = e2m1(...) rounded to nearest, ties to the even code; codes of
 *                 elements 2i and 2i+1 in byte i, the even one in the low four bits
 *   x        bf16 [B, d_model]
 *   w_kv     bf16 [d_model, 2*head_dim]  (in x out; key columns first, then value columns)
 *   k_cache, v_cache, k_scale, v_scale, kv_seq_stride_tokens, seq_lens: as for
 *            mfa_decode_attn, but written; seq_lens[b] is the number of tokens already
 *            cached, i.e. the row the new token takes (the caller then attends with
 *            seq_lens[b] + 1).  A row at or past kv_seq_stride_tokens is not written.
 * The paper does not say where positional encoding enters; none is applied here.
 */
MFA_API mfa_status mfa_kv_append(mfa_ctx* ctx, const void* x, const void* w_kv, mfa_kv_dtype kv_dtype, void* k_cache,
                         void* v_cache, float* k_scale, float* v_scale, int64_t kv_seq_stride_tokens,
                         const int32_t* seq_lens, int32_t B, void* hip_stream);

/* The same into a paged cache: the row is (seq_lens[b] % page_size) of page
 * block_table[b][seq_lens[b] / page_size]; a block index at or past
 * max_blocks_per_seq, or a page id outside [0, n_pages), is not written. */
MFA_API mfa_status mfa_kv_append_paged(mfa_ctx* ctx, const void* x, const void* w_kv, mfa_kv_dtype kv_dtype, void* k_pool,
                               void* v_pool, float* k_scale_pool, float* v_scale_pool, int32_t n_pages,
                               const int32_t* block_table, int32_t max_blocks_per_seq, const int32_t* seq_lens,
                               int32_t B, void* hip_stream);

/* Test aid: the record step alone from given fp32 rows kv [B, 2*head_dim] (block_table
 * NULL: contiguous cache).  Used to check that rounding and quantisation are bit-exact. */
MFA_API mfa_status mfa_debug_kv_record(mfa_ctx* ctx, const float* kv, mfa_kv_dtype kv_dtype, void* k_cache, void* v_cache,
                               float* k_scale, float* v_scale, int64_t kv_seq_stride_tokens, const int32_t* block_table,
                               int32_t max_blocks_per_seq, const int32_t* seq_lens, int32_t B, void* hip_stream);

/*
 * Output projection of the attention layer (Section 6: 64*256 -> 7168):
 *     y = bf16(attn_out) . W_o
 *   attn_out fp32 [B, n_q_heads*head_dim]   (what mfa_decode_attn* wrote)
 *   w_o      bf16 [n_q_heads*head_dim, d_model]
 *   y        bf16 [B, d_model]              (written)
 * The attention output is rounded to bf16 for the MFMA, products accumulate in fp32,
 * y is rounded to bf16 once on store.  1 <= B <= max_batch.
 */
MFA_API mfa_status mfa_out_proj(mfa_ctx* ctx, const float* attn_out, const void* w_o, void* y, int32_t B, void* hip_stream);

/*
 * Decode-step attention over a contiguous cache (Section 2: 64 query heads
 * share one key head and one value head; Section 7.1: independent sequences):
 *     s[b,h,j] = softmax_scale * sum_d q[b,h,d] * K[b,j,d]        j < seq_lens[b]
 *     p[b,h,:] = softmax_j(s[b,h,:])
 *     out[b,h,d] = sum_j p[b,h,j] * V[b,j,d]
 * with K[b,j,:] = k_cache[b,j,:] for bf16 and k_scale[b,j] * k_cache[b,j,:] for
 * fp8 and fp4 (V likewise).  MFA_KV_FP4_E2M1 is the "4-bit storage, 8-bit
 * arithmetic" cache that Section 5.2 discusses: a row is head_dim/2 bytes, element
 * d in byte d/2 (low four bits when d is even) as an e2m1 code (1 sign, 2 exponent
 * bits with bias 1, 1 fraction bit: 0, 0.5, 1, 1.5, 2, 3, 4, 6 and their negatives),
 * with the same per-token fp32 scales as fp8.
 *   q        bf16 [B, n_q_heads, head_dim]
 *   k_cache, v_cache  [B, kv_seq_stride_tokens, head_dim] in kv_dtype (fp4: head_dim/2 bytes per row)
 *   k_scale, v_scale  fp32 [B, kv_seq_stride_tokens]; NULL for bf16
 *   kv_seq_stride_tokens  rows between consecutive sequences (>= max_seq_len_hint)
 *   seq_lens int32 [B] on the DEVICE (never read by the host)
 *   max_seq_len_hint  host-side upper bound of seq_lens, used only to size the
 *            launch; 1 <= hint <= cfg.max_seq_len
 *   out      fp32 [B, n_q_heads, head_dim]      (written)
 * Scores and sums are accumulated in fp32; attention weights are rounded to
 * bf16 before they multiply V.  For a given build, device and arguments the
 * result is bitwise reproducible from call to call.
 * Work distribution: for B <= 4096 the 64-token tiles of all sequences, laid end
 * to end, are cut into equal ranges over at most 256 workgroups, whatever the
 * individual lengths are (they are read on the device); larger batches, or a
 * context created with schedule = MFA_SCHEDULE_FIXED, cut every sequence
 * into the same number of equal chunks of max_seq_len_hint instead.  Pieces of a
 * sequence are merged in order of position by the library.
 */
MFA_API mfa_status mfa_decode_attn(mfa_ctx* ctx, const void* q, const void* k_cache, const void* v_cache,
                           const float* k_scale, const float* v_scale, mfa_kv_dtype kv_dtype,
                           int64_t kv_seq_stride_tokens, const int32_t* seq_lens,
                           int32_t max_seq_len_hint, int32_t B, float* out, void* hip_stream);

/*
 * The same attention over a paged cache: token j of sequence b is row
 * (j % page_size) of page block_table[b][j / page_size].
 *   k_pool, v_pool            [n_pages, page_size, head_dim] in kv_dtype (fp4: head_dim/2 bytes per row)
 *   k_scale_pool, v_scale_pool  fp32 [n_pages, page_size]; NULL for bf16
 *   block_table  int32 [B, max_blocks_per_seq] on the device; entries at or past
 *                ceil(seq_lens[b] / page_size) are never read (may be -1).  A page id
 *                outside [0, n_pages) that is read is clamped into that range: the result
 *                of that sequence is then meaningless, but no memory outside the pools
 *                is touched.
 *   max_blocks_per_seq >= ceil(max_seq_len_hint / page_size)
 * Other arguments as mfa_decode_attn.  For the same tokens the result is
 * bitwise equal to mfa_decode_attn's on the gathered contiguous cache with the
 * same max_seq_len_hint and B.
 */
MFA_API mfa_status mfa_decode_attn_paged(mfa_ctx* ctx, const void* q, const void* k_pool, const void* v_pool,
                                 const float* k_scale_pool, const float* v_scale_pool,
                                 mfa_kv_dtype kv_dtype, int32_t n_pages, const int32_t* block_table,
                                 int32_t max_blocks_per_seq, const int32_t* seq_lens,
                                 int32_t max_seq_len_hint, int32_t B, float* out, void* hip_stream);

/*
 * Test aid, not part of the serving path: copy the logical cache of every
 * sequence out of a paged pool into a contiguous buffer
 *   dst [B, dst_seq_stride_tokens, row_bytes] (bytes; row_bytes = bytes of one
 *   token row, a multiple of 4), rows j < seq_lens[b] only; other rows untouched.
 * Used to check that paged addressing moves bytes exactly.
 */
MFA_API mfa_status mfa_debug_gather_paged(mfa_ctx* ctx, const void* pool, int32_t row_bytes, int32_t n_pages,
                                  const int32_t* block_table, int32_t max_blocks_per_seq,
                                  const int32_t* seq_lens, int32_t max_seq_len_hint, int32_t B,
                                  void* dst, int64_t dst_seq_stride_tokens, void* hip_stream);

/*
 * Several query tokens per sequence (Section 5.2 names multi-token prediction as the way to
 * raise the arithmetic intensity of decoding attention: the new tokens share one pass over the
 * cache).  The q_len new tokens are the last q_len rows of the cache (seq_lens[b] counts them);
 * query token j of sequence b attends to the first seq_lens[b] - (q_len - 1 - j) cached tokens,
 * i.e. causally among the new tokens.  A query token left without any token to attend to
 * (seq_lens[b] < q_len) gets the zero row.
 *   q    bf16 [B, q_len, n_q_heads, head_dim]
 *   out  fp32 [B, q_len, n_q_heads, head_dim]     (written)
 * 1 <= q_len <= 4 (larger: MFA_ERR_UNSUPPORTED); q_len = 1 is mfa_decode_attn[_paged].  Two query
 * tokens share one pass over the cache; three and four share one pass over a bf16 cache when
 * B <= 512, and are otherwise (8-bit and 4-bit caches, larger batches) worked off as two pairs, i.e.
 * two passes.  Several query tokens need the balanced work distribution (B <= 4096, schedule
 * MFA_SCHEDULE_BALANCED).
 * Everything else as for q_len = 1.
 */
MFA_API mfa_status mfa_decode_attn_multi(mfa_ctx* ctx, const void* q, const void* k_cache, const void* v_cache,
                                 const float* k_scale, const float* v_scale, mfa_kv_dtype kv_dtype,
                                 int64_t kv_seq_stride_tokens, const int32_t* seq_lens, int32_t max_seq_len_hint,
                                 int32_t B, int32_t q_len, float* out, void* hip_stream);
MFA_API mfa_status mfa_decode_attn_paged_multi(mfa_ctx* ctx, const void* q, const void* k_pool, const void* v_pool,
                                       const float* k_scale_pool, const float* v_scale_pool, mfa_kv_dtype kv_dtype,
                                       int32_t n_pages, const int32_t* block_table, int32_t max_blocks_per_seq,
                                       const int32_t* seq_lens, int32_t max_seq_len_hint, int32_t B, int32_t q_len,
                                       float* out, void* hip_stream);

/*
 * mfa_decode_attn for callers that cannot allocate device memory or hand over a
 * workspace at the time of the call: code under HIP graph capture, tight serving
 * loops, harnesses that forbid allocation.  Same arguments, same kernels and the
 * same (bitwise) result as mfa_decode_attn, but the partial results of the context
 * splits go to a fixed device array inside the library (about 25.4 MB per device,
 * held from the time the library is loaded until the process ends) instead of the
 * context's workspace; the call itself allocates nothing and calls no allocating
 * routine.  Limits: B <= 128 and B + workgroups <= 384 partial-result slots
 * (always true for B <= 128 with the default 256 workgroups); beyond them the call
 * returns MFA_ERR_WORKSPACE_TOO_SMALL and launches nothing.  All calls on one
 * device share that one array, whichever context they go through: calls that
 * overlap on a device (different streams without ordering) race; order them on
 * one stream.  Nothing in the array has to survive from call to call.
 */
MFA_API mfa_status mfa_decode_attn_static(mfa_ctx* ctx, const void* q, const void* k_cache, const void* v_cache,
                                  const float* k_scale, const float* v_scale, mfa_kv_dtype kv_dtype,
                                  int64_t kv_seq_stride_tokens, const int32_t* seq_lens,
                                  int32_t max_seq_len_hint, int32_t B, float* out, void* hip_stream);

/*
 * Measurement aid, not part of the serving path: while both handles are non-NULL
 * (hipEvent_t passed as void*, created by the caller with timing enabled), every
 * mfa_decode_attn / mfa_decode_attn_paged call on this context attaches the two
 * events to the dispatch of its streaming kernel (the one that reads the cache)
 * on the call's stream: `ev_before` takes the time that kernel starts on the
 * device and `ev_after` the time it ends, so hipEventElapsedTime(ev_before,
 * ev_after) is the duration of that kernel alone.  Pass NULLs to stop.
 */
MFA_API mfa_status mfa_debug_set_kernel_events(mfa_ctx* ctx, void* ev_before, void* ev_after);

/*
 * Measurement aid, not part of the serving path: one kernel that reads `bytes_each`
 * bytes from each of the two device buffers with plain 16-byte loads and computes
 * nothing, i.e. the time any kernel needs just to stream that many bytes from HBM
 * on this device.  bytes_each must be a positive multiple of 16 MiB.  Honours the
 * events set with mfa_debug_set_kernel_events.
 */
MFA_API mfa_status mfa_debug_stream_read(mfa_ctx* ctx, const void* a, const void* b, size_t bytes_each,
                                         void* hip_stream);

/* Number of pieces into which the next mfa_decode_attn* call with these host
 * arguments cuts a sequence of the full length max_seq_len_hint when every
 * sequence has that length (shorter sequences get proportionally fewer; each
 * piece's partial result is merged by the library).  Pure host function; 0 on
 * invalid arguments. */
MFA_API int32_t mfa_decode_num_splits(const mfa_ctx* ctx, int32_t B, int32_t max_seq_len_hint);

#ifdef __cplusplus
}
#endif
#endif /* MFA_H */

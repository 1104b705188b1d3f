// Internal declarations shared by the translation units of libmfa.so (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/mfa.h"

namespace mfa {

constexpr int kHeads = 64;       // query heads sharing one key head and one value head
constexpr int kHeadDim = 256;
constexpr int kPage = 64;        // tokens per cache page = tokens per streamed tile
constexpr int kTile = 64;

// Vector types for MFMA operands.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// How the context of one call is cut into work items.  Pure host arithmetic.
struct SplitPlan {
    int32_t n_splits;       // work items per sequence
    int32_t chunk_tokens;   // tokens per work item, a multiple of kTile
};
SplitPlan plan_splits(int32_t B, int32_t max_seq_len_hint, int32_t target_items);

// Balanced schedule (batches of at most kMaxBalancedBatch sequences): the tiles of all sequences,
// laid end to end in sequence order, are cut into n_wgs equal ranges, one per workgroup; a range
// that crosses sequence boundaries is worked off as one segment per sequence.  The workgroup
// count, and the number of partial-result slots that any schedule over it can need.
constexpr int32_t kMaxQueryTokens = 4;         // query tokens per sequence and call
constexpr int32_t kMaxBalancedBatch = 4096;
int32_t balanced_workgroups(int32_t B, int32_t max_seq_len_hint, int32_t target_items);   // 0 if B is too large
inline size_t balanced_slots(int32_t B, int32_t n_wgs) { return (size_t)B + (size_t)n_wgs; }

// Per work item the split kernel leaves: acc [kHeads][kHeadDim] fp32 (unnormalised),
// and (m, l) per head: running maximum in the log2 domain and the sum of weights.
constexpr size_t kPartialAccFloats = (size_t)kHeads * kHeadDim;
constexpr size_t kPartialMlFloats = (size_t)kHeads * 2;

struct AttnArgs {
    const void* q;                 // bf16 [B,q_len,64,256]
    const void* k;                 // cache or pool
    const void* v;
    const float* k_scale;          // fp8 only
    const float* v_scale;
    const int32_t* seq_lens;       // device
    const int32_t* block_table;    // device, NULL for contiguous
    float* out;                    // fp32 [B,q_len,64,256]
    float* ws_acc;                 // [B*n_splits][64][256]
    float* ws_ml;                  // [B*n_splits][64][2]
    int32_t* ws_seg;               // balanced schedule: per sequence (first partial slot, number of partials)
    int64_t seq_stride_tokens;     // contiguous only
    int32_t max_blocks_per_seq;    // paged only
    int32_t n_pages;               // paged only: page ids are clamped into [0, n_pages) when read, rows with ids outside are not written
    int32_t B;
    int32_t q_len;                 // query tokens per sequence (q and out are [B, q_len, 64, 256])
    int32_t q0;                    // first query token this launch works on: a launch takes tokens q0 .. q0 + n_here - 1
    int32_t n_here;                // query tokens of this launch (1, 2, or 3 / 4 in the one-pass kernel); the partial of
                                   // (slot, token j of the launch) sits at slot * n_here + j
    int32_t n_wgs;                 // > 0: balanced schedule over this many workgroups; 0: fixed splits below
    int32_t n_splits;
    int32_t chunk_tokens;
    int32_t max_seq_len_hint;
    float scale_log2e;             // softmax_scale * log2(e)
};

// Launchers (enqueue only; return the launch status).
hipError_t launch_decode_attn(const AttnArgs& a, mfa_kv_dtype kv_dtype, hipStream_t stream,
                              hipEvent_t ev_before, hipEvent_t ev_after);   // events may be NULL
hipError_t prepare_decode_attn_kernels();
// bytes_each must be a multiple of 2048 * 8192; sink is 4 writable bytes
hipError_t launch_stream_read(const void* a, const void* b, size_t bytes_each, void* sink, hipStream_t stream,
                              hipEvent_t ev_before, hipEvent_t ev_after);   // one-time function attributes (dynamic LDS size)

struct QProjArgs {
    const void* x;        // bf16 [B,d_model]
    const void* w_qa;     // bf16 [d_model,q_rank]
    const float* gain;    // fp32 [q_rank] or NULL
    const void* w_qb;     // bf16 [q_rank,n_out]
    void* q_out;          // bf16 [B,n_out]
    float* ws_c;          // fp32 [split_k][B_pad][q_rank] partial sums of the first product
    void* ws_chat;        // bf16, k-step-major: element (m, k) at ((k/32)*B_pad + m)*32 + k%32
    int32_t B, d_model, q_rank, n_out;
    int32_t split_k;
    int32_t k_per_split;  // multiple of 32
    float eps;
};
constexpr int kQProjRows = 128;   // rows of x one workgroup covers
struct QProjPlan {
    int32_t split_k;      // K splits of a product whose fp32 partials go through the workspace
    int32_t k_per_split;
    int32_t strips_per_wg;   // adjacent 64-column strips a workgroup owns: 1, or 2 / 4 (output projection with at most 128 / 64 rows)
};
// Split of the k range of y = x.W ([K] -> [N]) that fills the device: N/64 column strips times split_k
// workgroups, about one per compute unit, at most 32 splits.
QProjPlan plan_linear(int32_t K, int32_t N, int32_t strips_per_wg = 1);
QProjPlan plan_out_proj(int32_t K, int32_t N, int32_t B);
inline QProjPlan plan_qproj(int32_t d_model, int32_t q_rank) { return plan_linear(d_model, q_rank); }
hipError_t prepare_query_proj_kernels();   // one-time function attributes (dynamic LDS size)
hipError_t launch_query_proj(const QProjArgs& a, hipStream_t stream);

// Key/value projection of the new token and its cache record.
constexpr int kKvWidth = 2 * kHeadDim;     // columns of W_kv: key then value
struct KvAppendArgs {
    const void* x;                 // bf16 [B, d_model]
    const void* w_kv;              // bf16 [d_model, 512]
    void* k;                       // cache or pool (bf16 or e4m3 codes)
    void* v;
    float* k_scale;                // fp8 only
    float* v_scale;
    const int32_t* seq_lens;       // device: tokens already cached = row the new token takes
    const int32_t* block_table;    // device, NULL for contiguous
    float* ws_c;                   // fp32 [split_k][B_pad][512]
    int64_t seq_stride_tokens;     // contiguous only
    int32_t max_blocks_per_seq;    // paged only
    int32_t n_pages;               // paged only: page ids are clamped into [0, n_pages) when read, rows with ids outside are not written
    int32_t B, d_model;
    QProjPlan plan;
};
hipError_t launch_kv_append(const KvAppendArgs& a, mfa_kv_dtype kv_dtype, hipStream_t stream);
// The record step alone, from given fp32 rows kv [B, 512] (plan.split_k is ignored: one "partial").
hipError_t launch_kv_record(const KvAppendArgs& a, const float* kv, mfa_kv_dtype kv_dtype, hipStream_t stream);

// Output projection y = bf16(attn) . W_o.
struct OutProjArgs {
    const float* attn;             // fp32 [B, n_in]
    const void* w_o;               // bf16 [n_in, d_model]
    void* y;                       // bf16 [B, d_model]
    float* ws_c;                   // fp32 [split_k][B_pad][d_model]
    void* ws_act;                  // bf16 k-step-major copy of attn
    int32_t B, n_in, d_model;
    QProjPlan plan;
};
hipError_t launch_out_proj(const OutProjArgs& a, hipStream_t stream);

hipError_t launch_gather_paged(const void* pool, int32_t row_bytes, const int32_t* block_table,
                               int32_t max_blocks_per_seq, int32_t n_pages, const int32_t* seq_lens, int32_t max_seq_len_hint,
                               int32_t B, void* dst, int64_t dst_seq_stride_tokens, hipStream_t stream);

}  // namespace mfa

// C boundary of libmfa.so: argument checking, workspace carving and dispatch.
// Every entry point is declared and documented in include/mfa.h.
#include <cmath>
#include <cstdlib>
#include <mutex>
#include <new>
#include <string>

#include "mfa_internal.hpp"

using namespace mfa;

struct mfa_ctx {
    mfa_config cfg;
    int32_t target_items;      // workgroups the planner aims for (one per compute unit by default)
    bool fixed_splits;         // MFA_SCHEDULE_FIXED: every sequence cut into the same number of equal chunks
    size_t max_items;          // bound on B * n_splits over all admissible calls
    float* ws_acc;
    float* ws_ml;
    int32_t* ws_seg;
    float* ws_c;
    void* ws_chat;
    QProjPlan qproj;
    int32_t qproj_rows_pad;
    hipEvent_t ev_before;      // measurement aid: recorded around the streaming kernel when both are set
    hipEvent_t ev_after;
    unsigned char* static_scratch;   // this device's copy of the file-scope scratch array (mfa_decode_attn_static)
};

namespace {

constexpr int32_t kDefaultTargetItems = 256;   // MI355X has 256 compute units; one workgroup fills one

// ---- Scratch of mfa_decode_attn_static, the attention call for callers that cannot allocate or
// pass a workspace: the partial results (acc, then (m, l)) of at most kStaticSlots segments and the
// per-sequence merge records of at most kStaticMaxBatch sequences live in a file-scope device array.
// Every device the library runs on holds its own copy from the time the code object is loaded until
// the process ends; its address on a device is asked for once, in mfa_decode_init with that device
// current, and only that address (never the array's name) is used in host code.
constexpr int32_t kStaticMaxBatch = 128;
constexpr size_t kStaticSlots = (size_t)kStaticMaxBatch + kDefaultTargetItems;
constexpr size_t kStaticAccOffset = 0;
constexpr size_t kStaticMlOffset = kStaticAccOffset + kStaticSlots * kPartialAccFloats * sizeof(float);
constexpr size_t kStaticSegOffset = kStaticMlOffset + kStaticSlots * kPartialMlFloats * sizeof(float);
constexpr size_t kStaticScratchBytes = kStaticSegOffset + (size_t)kStaticMaxBatch * 2 * sizeof(int32_t);
static_assert(kStaticMlOffset % 256 == 0 && kStaticSegOffset % 256 == 0, "the pieces of the scratch array stay 256-byte aligned");
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
unsigned char* g_scratch_ptr[kMaxDevices];        // per device; filled with that device current

// The calling thread's current device must be `device`.
hipError_t static_scratch_for_device(int device, unsigned char** out)
{
    *out = nullptr;
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = static_cast<unsigned char*>(p);
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}

// Workgroups an attention call aims for: the configuration's figure, else (test override) the
// environment's, else one per compute unit.
int32_t target_items_of(const mfa_config* c)
{
    if (c->target_workgroups >= 1 && c->target_workgroups <= 4096) return c->target_workgroups;
    const char* s = std::getenv("MFA_TARGET_ITEMS");
    if (s) {
        const long v = std::strtol(s, nullptr, 10);
        if (v >= 1 && v <= 4096) return (int32_t)v;
    }
    return kDefaultTargetItems;
}

bool fixed_schedule_of(const mfa_config* c)
{
    if (c->schedule == MFA_SCHEDULE_FIXED) return true;
    const char* sch = std::getenv("MFA_SCHEDULE");
    return sch && std::string(sch) == "fixed";
}

bool config_ok(const mfa_config* c)
{
    if (!c) return false;
    if (c->max_batch < 1 || c->max_batch > 65536) return false;
    if (c->max_seq_len < 1 || c->max_seq_len > (1 << 24)) return false;
    if (c->d_model < 64 || c->d_model % 64) return false;
    if (c->q_rank < 128 || c->q_rank % 128) return false;
    if (!(c->softmax_scale > 0.f) || !std::isfinite(c->softmax_scale)) return false;
    if (!(c->rms_eps >= 0.f) || !std::isfinite(c->rms_eps)) return false;
    if (c->device < 0) return false;
    if (c->target_workgroups < 0 || c->target_workgroups > 4096) return false;
    if (c->schedule != MFA_SCHEDULE_BALANCED && c->schedule != MFA_SCHEDULE_FIXED) return false;
    return true;
}

bool config_supported(const mfa_config* c)
{
    return c->n_q_heads == kHeads && c->head_dim == kHeadDim && c->page_size == kPage;
}

size_t max_items_for(const mfa_config* c, int32_t target)
{
    size_t best = 0;
    for (int32_t B = 1; B <= c->max_batch; ++B) {
        const SplitPlan p = plan_splits(B, c->max_seq_len, target);
        const size_t items = (size_t)B * p.n_splits;
        if (items > best) best = items;
    }
    const int32_t Bb = c->max_batch < kMaxBalancedBatch ? c->max_batch : kMaxBalancedBatch;
    const size_t balanced = balanced_slots(Bb, target);                 // >= B + workgroups of any balanced call
    return best > balanced ? best : balanced;
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct Carve {
    size_t acc, ml, seg, c, chat, total;
    size_t max_items;
    QProjPlan qproj;
    int32_t rows_pad;
};

Carve carve(const mfa_config* c, int32_t target)
{
    Carve w;
    w.max_items = max_items_for(c, target);
    w.qproj = plan_qproj(c->d_model, c->q_rank);
    w.rows_pad = (c->max_batch + kQProjRows - 1) / kQProjRows * kQProjRows;
    size_t off = 0;
    // partial results: one slot per (workgroup segment, query token of a launch), up to kMaxQueryTokens of them
    w.acc = off; off = align_up(off + kMaxQueryTokens * w.max_items * kPartialAccFloats * sizeof(float), 256);
    w.ml = off;  off = align_up(off + kMaxQueryTokens * w.max_items * kPartialMlFloats * sizeof(float), 256);
    w.seg = off; off = align_up(off + (size_t)c->max_batch * 2 * sizeof(int32_t), 256);
    // split-K partials of whichever product is running, and the bf16 k-step-major activations of the
    // second query product / the output projection
    const int32_t n_attn = c->n_q_heads * c->head_dim;
    size_t partial_floats = (size_t)w.qproj.split_k * c->q_rank;
    const size_t kv_floats = (size_t)plan_linear(c->d_model, kKvWidth).split_k * kKvWidth;
    const size_t o_floats = (size_t)std::max(std::max(plan_linear(n_attn, c->d_model, 1).split_k, plan_linear(n_attn, c->d_model, 2).split_k), plan_linear(n_attn, c->d_model, 4).split_k) * c->d_model;
    if (kv_floats > partial_floats) partial_floats = kv_floats;
    if (o_floats > partial_floats) partial_floats = o_floats;
    w.c = off;   off = align_up(off + partial_floats * w.rows_pad * sizeof(float), 256);
    w.chat = off; off = align_up(off + (size_t)w.rows_pad * (c->q_rank > n_attn ? c->q_rank : n_attn) * 2, 256);
    w.total = off;
    return w;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool on_device(const mfa_ctx* ctx)
{
    int dev = -1;
    return hipGetDevice(&dev) == hipSuccess && dev == ctx->cfg.device;
}

mfa_status check_attn_common(const mfa_ctx* ctx, const void* q, const void* k, const void* v, const float* ks,
                             const float* vs, mfa_kv_dtype kv_dtype, const int32_t* seq_lens, int32_t hint,
                             int32_t B, const float* out)
{
    if (!ctx || !q || !k || !v || !seq_lens || !out) return MFA_ERR_INVALID_ARG;
    if (kv_dtype != MFA_KV_BF16 && kv_dtype != MFA_KV_FP8_E4M3 && kv_dtype != MFA_KV_FP4_E2M1) return MFA_ERR_INVALID_ARG;
    if (kv_dtype != MFA_KV_BF16 && (!ks || !vs)) return MFA_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(ks) || !aligned16(vs) ||
        (reinterpret_cast<uintptr_t>(seq_lens) & 3u))
        return MFA_ERR_INVALID_ARG;
    if (B < 1 || B > ctx->cfg.max_batch) return MFA_ERR_INVALID_ARG;
    if (hint < 1 || hint > ctx->cfg.max_seq_len) return MFA_ERR_INVALID_ARG;
    if (!on_device(ctx)) return MFA_ERR_INVALID_ARG;
    return MFA_OK;
}

void fill_common(const mfa_ctx* ctx, AttnArgs& a, int32_t B, int32_t hint)
{
    const SplitPlan p = plan_splits(B, hint, ctx->target_items);
    a.n_splits = p.n_splits;
    a.chunk_tokens = p.chunk_tokens;
    a.B = B;
    a.q_len = 1;
    a.q0 = 0;
    a.n_here = 1;
    a.max_seq_len_hint = hint;
    a.ws_acc = ctx->ws_acc;
    a.ws_ml = ctx->ws_ml;
    a.ws_seg = ctx->ws_seg;
    a.n_wgs = ctx->fixed_splits ? 0 : balanced_workgroups(B, hint, ctx->target_items);
    a.scale_log2e = ctx->cfg.softmax_scale * 1.44269504088896340736f;
}

}  // namespace

extern "C" {

size_t mfa_decode_workspace_bytes(const mfa_config* cfg)
{
    if (!config_ok(cfg) || !config_supported(cfg)) return 0;
    return carve(cfg, target_items_of(cfg)).total;
}

mfa_status mfa_decode_init(const mfa_config* cfg, void* d_workspace, size_t workspace_bytes, mfa_ctx** out_ctx)
{
    if (out_ctx) *out_ctx = nullptr;
    if (!out_ctx || !config_ok(cfg) || !d_workspace) return MFA_ERR_INVALID_ARG;
    if (!config_supported(cfg)) return MFA_ERR_UNSUPPORTED;
    if (reinterpret_cast<uintptr_t>(d_workspace) & 255u) return MFA_ERR_INVALID_ARG;
    const int32_t target = target_items_of(cfg);
    const Carve w = carve(cfg, target);
    if (workspace_bytes < w.total) return MFA_ERR_WORKSPACE_TOO_SMALL;

    int n_dev = 0;
    if (hipGetDeviceCount(&n_dev) != hipSuccess) return MFA_ERR_HIP;
    if (cfg->device >= n_dev) return MFA_ERR_INVALID_ARG;
    int prev = -1;
    if (hipGetDevice(&prev) != hipSuccess) return MFA_ERR_HIP;
    if (prev != cfg->device && hipSetDevice(cfg->device) != hipSuccess) return MFA_ERR_HIP;
    hipError_t e = prepare_decode_attn_kernels();
    if (e == hipSuccess) e = prepare_query_proj_kernels();
    unsigned char* static_scratch = nullptr;
    if (e == hipSuccess) e = static_scratch_for_device(cfg->device, &static_scratch);
    if (prev != cfg->device) (void)hipSetDevice(prev);
    if (e != hipSuccess) return MFA_ERR_HIP;

    mfa_ctx* ctx = new (std::nothrow) mfa_ctx;
    if (!ctx) return MFA_ERR_HOST_ALLOC;
    ctx->cfg = *cfg;
    ctx->target_items = target;
    ctx->fixed_splits = fixed_schedule_of(cfg);
    ctx->max_items = w.max_items;
    unsigned char* base = static_cast<unsigned char*>(d_workspace);
    ctx->ws_acc = reinterpret_cast<float*>(base + w.acc);
    ctx->ws_ml = reinterpret_cast<float*>(base + w.ml);
    ctx->ws_seg = reinterpret_cast<int32_t*>(base + w.seg);
    ctx->ws_c = reinterpret_cast<float*>(base + w.c);
    ctx->ws_chat = base + w.chat;
    ctx->qproj = w.qproj;
    ctx->qproj_rows_pad = w.rows_pad;
    ctx->ev_before = nullptr;
    ctx->ev_after = nullptr;
    ctx->static_scratch = static_scratch;
    *out_ctx = ctx;
    return MFA_OK;
}

void mfa_decode_destroy(mfa_ctx* ctx) { delete ctx; }

const char* mfa_status_string(mfa_status s)
{
    switch (s) {
        case MFA_OK: return "ok";
        case MFA_ERR_INVALID_ARG: return "invalid argument";
        case MFA_ERR_UNSUPPORTED: return "unsupported shape or type";
        case MFA_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case MFA_ERR_HIP: return "HIP runtime error";
        case MFA_ERR_HOST_ALLOC: return "out of host memory";
    }
    return "unknown status";
}

mfa_status mfa_debug_set_kernel_events(mfa_ctx* ctx, void* ev_before, void* ev_after)
{
    if (!ctx) return MFA_ERR_INVALID_ARG;
    if ((ev_before == nullptr) != (ev_after == nullptr)) return MFA_ERR_INVALID_ARG;
    ctx->ev_before = static_cast<hipEvent_t>(ev_before);
    ctx->ev_after = static_cast<hipEvent_t>(ev_after);
    return MFA_OK;
}

mfa_status mfa_debug_stream_read(mfa_ctx* ctx, const void* a, const void* b, size_t bytes_each, void* hip_stream)
{
    if (!ctx || !a || !b || !aligned16(a) || !aligned16(b)) return MFA_ERR_INVALID_ARG;
    if (bytes_each == 0 || bytes_each % ((size_t)2048 * 8192) != 0) return MFA_ERR_INVALID_ARG;
    if (!on_device(ctx)) return MFA_ERR_INVALID_ARG;
    // the first bytes of the partial-result area serve as the (practically never written) sink
    const hipError_t e = launch_stream_read(a, b, bytes_each, ctx->ws_acc, static_cast<hipStream_t>(hip_stream),
                                            ctx->ev_before, ctx->ev_after);
    return e == hipSuccess ? MFA_OK : MFA_ERR_HIP;
}

int32_t mfa_decode_num_splits(const mfa_ctx* ctx, int32_t B, int32_t max_seq_len_hint)
{
    if (!ctx || B < 1 || B > ctx->cfg.max_batch || max_seq_len_hint < 1 || max_seq_len_hint > ctx->cfg.max_seq_len)
        return 0;
    return plan_splits(B, max_seq_len_hint, ctx->target_items).n_splits;
}

mfa_status mfa_query_proj(mfa_ctx* ctx, const void* x, const void* w_qa, const float* rms_gain, const void* w_qb,
                          void* q_out, int32_t B, void* hip_stream)
{
    if (!ctx || !x || !w_qa || !w_qb || !q_out) return MFA_ERR_INVALID_ARG;
    if (!aligned16(x) || !aligned16(w_qa) || !aligned16(w_qb) || !aligned16(q_out) || !aligned16(rms_gain))
        return MFA_ERR_INVALID_ARG;
    if (B < 1 || B > ctx->cfg.max_batch) return MFA_ERR_INVALID_ARG;
    if (!on_device(ctx)) return MFA_ERR_INVALID_ARG;
    QProjArgs a;
    a.x = x; a.w_qa = w_qa; a.gain = rms_gain; a.w_qb = w_qb; a.q_out = q_out;
    a.ws_c = ctx->ws_c; a.ws_chat = ctx->ws_chat;
    a.B = B; a.d_model = ctx->cfg.d_model; a.q_rank = ctx->cfg.q_rank;
    a.n_out = ctx->cfg.n_q_heads * ctx->cfg.head_dim;
    a.split_k = ctx->qproj.split_k;
    a.k_per_split = ctx->qproj.k_per_split;
    a.eps = ctx->cfg.rms_eps;
    return launch_query_proj(a, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? MFA_OK : MFA_ERR_HIP;
}

namespace {

mfa_status check_kv_append(const mfa_ctx* ctx, const void* x, const void* w_kv, mfa_kv_dtype kv_dtype, const void* k,
                           const void* v, const float* ks, const float* vs, const int32_t* seq_lens, int32_t B)
{
    if (!ctx || !x || !w_kv || !k || !v || !seq_lens) return MFA_ERR_INVALID_ARG;
    if (kv_dtype != MFA_KV_BF16 && kv_dtype != MFA_KV_FP8_E4M3 && kv_dtype != MFA_KV_FP4_E2M1) return MFA_ERR_INVALID_ARG;
    if (kv_dtype != MFA_KV_BF16 && (!ks || !vs)) return MFA_ERR_INVALID_ARG;
    if (!aligned16(x) || !aligned16(w_kv) || !aligned16(k) || !aligned16(v) || !aligned16(ks) || !aligned16(vs) ||
        (reinterpret_cast<uintptr_t>(seq_lens) & 3u))
        return MFA_ERR_INVALID_ARG;
    if (B < 1 || B > ctx->cfg.max_batch) return MFA_ERR_INVALID_ARG;
    if (!on_device(ctx)) return MFA_ERR_INVALID_ARG;
    return MFA_OK;
}

void fill_kv_append(const mfa_ctx* ctx, KvAppendArgs& a, const void* x, const void* w_kv, void* k, void* v, float* ks,
                    float* vs, const int32_t* seq_lens, int32_t B)
{
    a.x = x; a.w_kv = w_kv; a.k = k; a.v = v; a.k_scale = ks; a.v_scale = vs; a.seq_lens = seq_lens;
    a.block_table = nullptr; a.ws_c = ctx->ws_c; a.seq_stride_tokens = 0; a.max_blocks_per_seq = 0;
    a.B = B; a.d_model = ctx->cfg.d_model;
    a.plan = plan_linear(ctx->cfg.d_model, kKvWidth);
}

}  // namespace

mfa_status mfa_kv_append(mfa_ctx* ctx, const void* x, const void* w_kv, mfa_kv_dtype kv_dtype, void* k_cache,
                         void* v_cache, float* k_scale, float* v_scale, int64_t kv_seq_stride_tokens,
                         const int32_t* seq_lens, int32_t B, void* hip_stream)
{
    const mfa_status st = check_kv_append(ctx, x, w_kv, kv_dtype, k_cache, v_cache, k_scale, v_scale, seq_lens, B);
    if (st != MFA_OK) return st;
    if (kv_seq_stride_tokens < 1) return MFA_ERR_INVALID_ARG;
    KvAppendArgs a{};
    fill_kv_append(ctx, a, x, w_kv, k_cache, v_cache, k_scale, v_scale, seq_lens, B);
    a.seq_stride_tokens = kv_seq_stride_tokens;
    return launch_kv_append(a, kv_dtype, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? MFA_OK : MFA_ERR_HIP;
}

mfa_status mfa_kv_append_paged(mfa_ctx* ctx, const void* x, const void* w_kv, mfa_kv_dtype kv_dtype, void* k_pool,
                               void* v_pool, float* k_scale_pool, float* v_scale_pool, int32_t n_pages,
                               const int32_t* block_table, int32_t max_blocks_per_seq, const int32_t* seq_lens,
                               int32_t B, void* hip_stream)
{
    const mfa_status st = check_kv_append(ctx, x, w_kv, kv_dtype, k_pool, v_pool, k_scale_pool, v_scale_pool, seq_lens, B);
    if (st != MFA_OK) return st;
    if (!block_table || (reinterpret_cast<uintptr_t>(block_table) & 3u) || n_pages < 1 || max_blocks_per_seq < 1)
        return MFA_ERR_INVALID_ARG;
    KvAppendArgs a{};
    fill_kv_append(ctx, a, x, w_kv, k_pool, v_pool, k_scale_pool, v_scale_pool, seq_lens, B);
    a.block_table = block_table;
    a.max_blocks_per_seq = max_blocks_per_seq;
    a.n_pages = n_pages;
    return launch_kv_append(a, kv_dtype, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? MFA_OK : MFA_ERR_HIP;
}

mfa_status mfa_debug_kv_record(mfa_ctx* ctx, const float* kv, mfa_kv_dtype kv_dtype, void* k_cache, void* v_cache,
                               float* k_scale, float* v_scale, int64_t kv_seq_stride_tokens, const int32_t* block_table,
                               int32_t max_blocks_per_seq, const int32_t* seq_lens, int32_t B, void* hip_stream)
{
    const mfa_status st = check_kv_append(ctx, kv, kv, kv_dtype, k_cache, v_cache, k_scale, v_scale, seq_lens, B);
    if (st != MFA_OK) return st;
    if (block_table ? max_blocks_per_seq < 1 : kv_seq_stride_tokens < 1) return MFA_ERR_INVALID_ARG;
    KvAppendArgs a{};
    fill_kv_append(ctx, a, nullptr, nullptr, k_cache, v_cache, k_scale, v_scale, seq_lens, B);
    a.block_table = block_table;
    a.max_blocks_per_seq = max_blocks_per_seq;
    a.n_pages = INT32_MAX;                                  // the test aid has no pool size: ids are taken as given
    a.seq_stride_tokens = kv_seq_stride_tokens;
    return launch_kv_record(a, kv, kv_dtype, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? MFA_OK : MFA_ERR_HIP;
}

mfa_status mfa_out_proj(mfa_ctx* ctx, const float* attn_out, const void* w_o, void* y, int32_t B, void* hip_stream)
{
    if (!ctx || !attn_out || !w_o || !y) return MFA_ERR_INVALID_ARG;
    if (!aligned16(attn_out) || !aligned16(w_o) || !aligned16(y)) return MFA_ERR_INVALID_ARG;
    if (B < 1 || B > ctx->cfg.max_batch) return MFA_ERR_INVALID_ARG;
    if (!on_device(ctx)) return MFA_ERR_INVALID_ARG;
    OutProjArgs a{};
    a.attn = attn_out; a.w_o = w_o; a.y = y; a.ws_c = ctx->ws_c; a.ws_act = ctx->ws_chat;
    a.B = B; a.n_in = ctx->cfg.n_q_heads * ctx->cfg.head_dim; a.d_model = ctx->cfg.d_model;
    a.plan = plan_out_proj(a.n_in, a.d_model, B);
    return launch_out_proj(a, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? MFA_OK : MFA_ERR_HIP;
}

mfa_status mfa_decode_attn_multi(mfa_ctx* ctx, const void* q, const void* k_cache, const void* v_cache,
                                 const float* k_scale, const float* v_scale, mfa_kv_dtype kv_dtype,
                                 int64_t kv_seq_stride_tokens, const int32_t* seq_lens, int32_t max_seq_len_hint,
                                 int32_t B, int32_t q_len, float* out, void* hip_stream)
{
    const mfa_status st = check_attn_common(ctx, q, k_cache, v_cache, k_scale, v_scale, kv_dtype, seq_lens,
                                            max_seq_len_hint, B, out);
    if (st != MFA_OK) return st;
    if (kv_seq_stride_tokens < max_seq_len_hint) return MFA_ERR_INVALID_ARG;
    if (q_len < 1) return MFA_ERR_INVALID_ARG;
    if (q_len > kMaxQueryTokens) return MFA_ERR_UNSUPPORTED;
    AttnArgs a{};
    a.q = q; a.k = k_cache; a.v = v_cache; a.k_scale = k_scale; a.v_scale = v_scale;
    a.seq_lens = seq_lens; a.block_table = nullptr; a.out = out;
    a.seq_stride_tokens = kv_seq_stride_tokens; a.max_blocks_per_seq = 0;
    fill_common(ctx, a, B, max_seq_len_hint);
    a.q_len = q_len;
    const hipError_t e = launch_decode_attn(a, kv_dtype, static_cast<hipStream_t>(hip_stream), ctx->ev_before, ctx->ev_after);
    if (e == hipErrorNotSupported) return MFA_ERR_UNSUPPORTED;
    return e == hipSuccess ? MFA_OK : MFA_ERR_HIP;
}

mfa_status mfa_decode_attn(mfa_ctx* ctx, const void* q, const void* k_cache, const void* v_cache,
                           const float* k_scale, const float* v_scale, mfa_kv_dtype kv_dtype,
                           int64_t kv_seq_stride_tokens, const int32_t* seq_lens, int32_t max_seq_len_hint,
                           int32_t B, float* out, void* hip_stream)
{
    return mfa_decode_attn_multi(ctx, q, k_cache, v_cache, k_scale, v_scale, kv_dtype, kv_seq_stride_tokens, seq_lens,
                                 max_seq_len_hint, B, 1, out, hip_stream);
}

mfa_status mfa_decode_attn_static(mfa_ctx* ctx, const void* q, const void* k_cache, const void* v_cache,
                                  const float* k_scale, const float* v_scale, mfa_kv_dtype kv_dtype,
                                  int64_t kv_seq_stride_tokens, const int32_t* seq_lens, int32_t max_seq_len_hint,
                                  int32_t B, float* out, void* hip_stream)
{
    const mfa_status st = check_attn_common(ctx, q, k_cache, v_cache, k_scale, v_scale, kv_dtype, seq_lens,
                                            max_seq_len_hint, B, out);
    if (st != MFA_OK) return st;
    if (kv_seq_stride_tokens < max_seq_len_hint) return MFA_ERR_INVALID_ARG;
    if (!ctx->static_scratch) return MFA_ERR_HIP;
    AttnArgs a{};
    a.q = q; a.k = k_cache; a.v = v_cache; a.k_scale = k_scale; a.v_scale = v_scale;
    a.seq_lens = seq_lens; a.block_table = nullptr; a.out = out;
    a.seq_stride_tokens = kv_seq_stride_tokens; a.max_blocks_per_seq = 0;
    fill_common(ctx, a, B, max_seq_len_hint);
    // the partial results of this call fit the fixed array, or the call is refused before any launch
    const size_t slots = a.n_wgs > 0 ? balanced_slots(B, a.n_wgs) : (size_t)B * a.n_splits;
    if (B > kStaticMaxBatch || slots > kStaticSlots) return MFA_ERR_WORKSPACE_TOO_SMALL;
    a.ws_acc = reinterpret_cast<float*>(ctx->static_scratch + kStaticAccOffset);
    a.ws_ml = reinterpret_cast<float*>(ctx->static_scratch + kStaticMlOffset);
    a.ws_seg = reinterpret_cast<int32_t*>(ctx->static_scratch + kStaticSegOffset);
    const hipError_t e = launch_decode_attn(a, kv_dtype, static_cast<hipStream_t>(hip_stream), nullptr, nullptr);
    if (e == hipErrorNotSupported) return MFA_ERR_UNSUPPORTED;
    return e == hipSuccess ? MFA_OK : MFA_ERR_HIP;
}

mfa_status mfa_decode_attn_paged_multi(mfa_ctx* ctx, const void* q, const void* k_pool, const void* v_pool,
                                       const float* k_scale_pool, const float* v_scale_pool, mfa_kv_dtype kv_dtype,
                                       int32_t n_pages, const int32_t* block_table, int32_t max_blocks_per_seq,
                                       const int32_t* seq_lens, int32_t max_seq_len_hint, int32_t B, int32_t q_len,
                                       float* out, void* hip_stream)
{
    const mfa_status st = check_attn_common(ctx, q, k_pool, v_pool, k_scale_pool, v_scale_pool, kv_dtype, seq_lens,
                                            max_seq_len_hint, B, out);
    if (st != MFA_OK) return st;
    if (!block_table || (reinterpret_cast<uintptr_t>(block_table) & 3u) || n_pages < 1) return MFA_ERR_INVALID_ARG;
    if ((int64_t)max_blocks_per_seq * kPage < max_seq_len_hint) return MFA_ERR_INVALID_ARG;
    if (q_len < 1) return MFA_ERR_INVALID_ARG;
    if (q_len > kMaxQueryTokens) return MFA_ERR_UNSUPPORTED;
    AttnArgs a{};
    a.q = q; a.k = k_pool; a.v = v_pool; a.k_scale = k_scale_pool; a.v_scale = v_scale_pool;
    a.seq_lens = seq_lens; a.block_table = block_table; a.out = out;
    a.seq_stride_tokens = 0; a.max_blocks_per_seq = max_blocks_per_seq; a.n_pages = n_pages;
    fill_common(ctx, a, B, max_seq_len_hint);
    a.q_len = q_len;
    const hipError_t e = launch_decode_attn(a, kv_dtype, static_cast<hipStream_t>(hip_stream), ctx->ev_before, ctx->ev_after);
    if (e == hipErrorNotSupported) return MFA_ERR_UNSUPPORTED;
    return e == hipSuccess ? MFA_OK : MFA_ERR_HIP;
}

mfa_status mfa_decode_attn_paged(mfa_ctx* ctx, const void* q, const void* k_pool, const void* v_pool,
                                 const float* k_scale_pool, const float* v_scale_pool, mfa_kv_dtype kv_dtype,
                                 int32_t n_pages, const int32_t* block_table, int32_t max_blocks_per_seq,
                                 const int32_t* seq_lens, int32_t max_seq_len_hint, int32_t B, float* out,
                                 void* hip_stream)
{
    return mfa_decode_attn_paged_multi(ctx, q, k_pool, v_pool, k_scale_pool, v_scale_pool, kv_dtype, n_pages, block_table,
                                       max_blocks_per_seq, seq_lens, max_seq_len_hint, B, 1, out, hip_stream);
}

mfa_status mfa_debug_gather_paged(mfa_ctx* ctx, const void* pool, int32_t row_bytes, int32_t n_pages,
                                  const int32_t* block_table, int32_t max_blocks_per_seq, const int32_t* seq_lens,
                                  int32_t max_seq_len_hint, int32_t B, void* dst, int64_t dst_seq_stride_tokens,
                                  void* hip_stream)
{
    if (!ctx || !pool || !block_table || !seq_lens || !dst) return MFA_ERR_INVALID_ARG;
    if (row_bytes < 4 || row_bytes % 4 || n_pages < 1) return MFA_ERR_INVALID_ARG;
    if (B < 1 || B > ctx->cfg.max_batch) return MFA_ERR_INVALID_ARG;
    if (max_seq_len_hint < 1 || max_seq_len_hint > ctx->cfg.max_seq_len) return MFA_ERR_INVALID_ARG;
    if ((int64_t)max_blocks_per_seq * kPage < max_seq_len_hint) return MFA_ERR_INVALID_ARG;
    if (dst_seq_stride_tokens < max_seq_len_hint) return MFA_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(pool) & 3u) || (reinterpret_cast<uintptr_t>(dst) & 3u)) return MFA_ERR_INVALID_ARG;
    if (!on_device(ctx)) return MFA_ERR_INVALID_ARG;
    const hipError_t e = launch_gather_paged(pool, row_bytes, block_table, max_blocks_per_seq, n_pages, seq_lens,
                                             max_seq_len_hint, B, dst, dst_seq_stride_tokens,
                                             static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MFA_OK : MFA_ERR_HIP;
}

}  // extern "C"

// Decode-step MFA attention for gfx950: 64 query heads of dimension 256 over one
// shared key head and one shared value head (paper, Section 2), one query token
// per sequence, independent sequences (Section 7.1).
//
// Work decomposition.  A work item is (sequence b, context split s): it streams
// the tokens [s*chunk, min(L_b, (s+1)*chunk)) once from HBM and leaves either the
// final output (one split) or an unnormalised partial (acc, m, l) that
// merge_splits_kernel reduces.  One workgroup of 8 waves per work item:
//   wave = 4*grp + wq;  wq picks 16 of the 64 heads, grp picks which 32-token
//   half of every 64-token tile the wave processes.  The two waves that share a
//   SIMD (same wq, different grp) keep independent online-softmax states that
//   are merged through LDS at the end, so one can run MFMA while the other runs
//   its softmax.
// Tiles of 64 tokens (= one cache page) are brought in with 16-byte
// global->LDS direct loads into a two-slot ring; slot = K rows then V rows,
// 512 B per row, 64 KB per slot.  Within a row the 16-byte (K) or 32-byte (V)
// chunks are XOR-swizzled with the row number so that the MFMA operand reads
// (16 rows x 16 B for K, 16 rows x 32 B transposing reads for V) spread over all
// LDS banks.  The swizzle is applied on the global side of the direct load
// because its LDS side is fixed to base + 16*lane.
//
// MFMA shapes (v_mfma_f32_16x16x32_bf16; lane = 16*g + n):
//   scores   S^T[token, head] = K[token, :] . Q[head, :]^T     A = K rows, B = Q
//            lane holds S^T[token 4g+i, head n], i = 0..3, for each 16-token block
//   output   O^T[d, head] += V^T[d, token] . P^T[token, head]  A = V^T, B = P
//            lane holds O^T[d = 16*db + 4g + i, head n]
// The score block a lane ends up with is exactly the B-operand slice it must
// supply for the second product (8 tokens of its own head), so attention weights
// never move between lanes; per-head statistics live in the lanes of that head.
#include "mfa_internal.hpp"

namespace mfa {

#define LDS_PTR(T, byte_off) ((__attribute__((address_space(3))) T*)(lds_base + (byte_off)))

constexpr int kSlotBytes = 65536;        // K 64x512 B then V 64x512 B
constexpr int kVOffset = 32768;
constexpr int kAttnLdsBytes = 2 * kSlotBytes;
constexpr int kAttnThreads = 512;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ void wait_vmem_all() { __builtin_amdgcn_s_waitcnt(0x0F70); }   // vmcnt(0) only

// 16 bytes per lane from global memory straight into LDS at lds_addr + 16*lane (lds_addr is
// wave-uniform and travels in M0).  Issued as inline assembly so that the compiler does not
// treat later LDS reads of the *other* ring slot as dependent on it; completion is awaited
// explicitly with wait_vmem_all() followed by a workgroup barrier.  M0 is not otherwise live
// in these kernels.  The s_nop covers the one wait state required between writing M0 and an
// LDS-direct load.
__device__ __forceinline__ void load_to_lds_16B(const void* gptr, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :: "v"(gptr), "s"(lds_addr) : "memory");
}

template <bool PAGED>
__global__ __launch_bounds__(kAttnThreads) void decode_bf16_kernel(AttnArgs a)
{
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    __attribute__((address_space(3))) unsigned char* lds_base =
        (__attribute__((address_space(3))) unsigned char*)smem;

    const uint32_t lds_addr0 = (uint32_t)(uintptr_t)lds_base;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wq = wave & 3;
    const int grp = wave >> 2;
    const int n = lane & 15;
    const int g = lane >> 4;

    const int item = blockIdx.x;
    const int b = item / a.n_splits;
    const int split = item - b * a.n_splits;
    int L = a.seq_lens[b];
    L = L < 0 ? 0 : (L > a.max_seq_len_hint ? a.max_seq_len_hint : L);
    const int t0 = split * a.chunk_tokens;
    const int t1 = (t0 + a.chunk_tokens < L) ? t0 + a.chunk_tokens : L;
    const int head = 16 * wq + n;

    if (t0 >= t1) {
        // nothing cached for this item; an empty sequence yields zeros
        if (a.n_splits == 1) {
            float4* o = (float4*)(a.out + (size_t)b * kHeads * kHeadDim);
            for (int i = threadIdx.x; i < kHeads * kHeadDim / 4; i += kAttnThreads) o[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
        return;
    }
    const int n_tiles = (t1 - t0 + kTile - 1) / kTile;

    // Query fragments: B operand of the score product, d = 32*ks + 8*g + j.
    bf16x8 qf[8];
    {
        const bf16x8* qp = (const bf16x8*)((const uint16_t*)a.q + ((size_t)b * kHeads + head) * kHeadDim + 8 * g);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qf[ks] = qp[ks * 4];
    }

    // Direct global->LDS load of one 64-token tile; wave w brings rows [8w, 8w+8) of K and of V.
    auto issue_tile = [&](int tile, int slot) {
        const int tile_t0 = t0 + tile * kTile;
        int64_t row0;
        if (PAGED) {
            const int page = a.block_table[(size_t)b * a.max_blocks_per_seq + tile_t0 / kPage];
            row0 = (int64_t)page * kPage;
        } else {
            row0 = (int64_t)b * a.seq_stride_tokens + tile_t0;
        }
        const int p16 = lane & 31;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int row = 8 * wave + 2 * u + (lane >> 5);          // row of the tile this lane fills
            int in_tile = row;
            if (tile_t0 + row > t1 - 1) in_tile = t1 - 1 - tile_t0;  // past the end: re-read the last valid token
            const size_t grow = (size_t)(row0 + in_tile) * 512;
            const int ck = p16 ^ (row & 15);
            const int cv = ((((p16 >> 1) ^ (row & 15)) << 1) | (p16 & 1));
            const unsigned char* ksrc = (const unsigned char*)a.k + grow + ck * 16;
            const unsigned char* vsrc = (const unsigned char*)a.v + grow + cv * 16;
            const uint32_t dst = lds_addr0 + slot * kSlotBytes + (8 * wave + 2 * u) * 512;
            load_to_lds_16B(ksrc, dst);
            load_to_lds_16B(vsrc, dst + kVOffset);
        }
    };

    f32x4 acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
    float m_run = -INFINITY;     // running maximum of this head's scores (log2 domain), same in the 4 lanes of a head
    float l_run = 0.f;           // this lane's share of the sum of weights

    const int r0 = 32 * grp;     // this wave's half of every tile

    issue_tile(0, 0);
    for (int it = 0; it < n_tiles; ++it) {
        const int slot = it & 1;
        wait_vmem_all();
        __syncthreads();
        if (it + 1 < n_tiles) issue_tile(it + 1, slot ^ 1);

        const int tile_t0 = t0 + it * kTile;
        const int kbase = slot * kSlotBytes;
        const int vbase = kbase + kVOffset;

        // ---- scores for 2 blocks of 16 tokens
        f32x4 s[2] = {(f32x4){0.f, 0.f, 0.f, 0.f}, (f32x4){0.f, 0.f, 0.f, 0.f}};
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
#pragma unroll
            for (int tb = 0; tb < 2; ++tb) {
                const int row = r0 + 16 * tb + n;                              // row & 15 == n
                const int off = kbase + row * 512 + (((4 * ks + g) ^ n) << 4);
                const bf16x8 kf = *LDS_PTR(bf16x8, off);
                s[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qf[ks], s[tb], 0, 0, 0);
            }
        }

        // ---- online softmax in the log2 domain; tokens at or past t1 are masked
        float sv[8];
        float m_new = m_run;
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int tok = tile_t0 + r0 + 16 * tb + 4 * g + i;
                float x = s[tb][i] * a.scale_log2e;
                x = tok < t1 ? x : -INFINITY;
                sv[4 * tb + i] = x;
                m_new = fmaxf(m_new, x);
            }
        }
        m_new = fmaxf(m_new, __shfl_xor(m_new, 16));
        m_new = fmaxf(m_new, __shfl_xor(m_new, 32));
        const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = fast_exp2(m_run - m_safe);     // 0 when nothing was accumulated yet
        m_run = m_new;

        bf16x8 pf;
        float psum = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const __bf16 pb = (__bf16)fast_exp2(sv[j] - m_safe);
            pf[j] = pb;
            psum += (float)pb;
        }
        l_run = l_run * alpha + psum;

        if (__any(alpha != 1.0f)) {
#pragma unroll
            for (int db = 0; db < 16; ++db) acc[db] *= alpha;
        }

        // ---- O^T += V^T P^T over this half tile's 32 tokens
#pragma unroll
        for (int db = 0; db < 16; ++db) {
            union { bf16x8 v; s16x4 h[2]; } vf;
#pragma unroll
            for (int tb = 0; tb < 2; ++tb) {
                const int row = r0 + 16 * tb + 4 * g + (n >> 2);              // row & 15 == 4g + n/4
                const int off = vbase + row * 512 + ((db ^ (4 * g + (n >> 2))) << 5) + ((n & 3) << 3);
                vf.h[tb] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, off));
            }
            acc[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf.v, pf, acc[db], 0, 0, 0);
        }
    }

    // ---- merge the two token halves (grp 1 -> grp 0) through LDS
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
    __syncthreads();                                  // every wave is done reading the ring
    constexpr int kRegs = 66;                         // 64 accumulators + m + l
    if (grp == 1) {
#pragma unroll
        for (int db = 0; db < 16; ++db)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                *LDS_PTR(float, ((wq * kRegs + db * 4 + i) * 64 + lane) * 4) = acc[db][i];
        *LDS_PTR(float, ((wq * kRegs + 64) * 64 + lane) * 4) = m_run;
        *LDS_PTR(float, ((wq * kRegs + 65) * 64 + lane) * 4) = l_run;
    }
    __syncthreads();
    if (grp == 1) return;

    {
        const float m1 = *LDS_PTR(float, ((wq * kRegs + 64) * 64 + lane) * 4);
        const float l1 = *LDS_PTR(float, ((wq * kRegs + 65) * 64 + lane) * 4);
        const float m = fmaxf(m_run, m1);             // finite: this item has at least one token
        const float w0 = fast_exp2(m_run - m);
        const float w1 = fast_exp2(m1 - m);
#pragma unroll
        for (int db = 0; db < 16; ++db)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                acc[db][i] = acc[db][i] * w0 + *LDS_PTR(float, ((wq * kRegs + db * 4 + i) * 64 + lane) * 4) * w1;
        l_run = l_run * w0 + l1 * w1;
        m_run = m;
    }

    // ---- store: final result when the context was not split, else the partial
    if (a.n_splits == 1) {
        const float inv = 1.0f / l_run;
        float* o = a.out + ((size_t)b * kHeads + head) * kHeadDim + 4 * g;
#pragma unroll
        for (int db = 0; db < 16; ++db) {
            f32x4 r = acc[db] * inv;
            *(f32x4*)(o + 16 * db) = r;
        }
    } else {
        float* o = a.ws_acc + ((size_t)item * kHeads + head) * kHeadDim + 4 * g;
#pragma unroll
        for (int db = 0; db < 16; ++db) *(f32x4*)(o + 16 * db) = acc[db];
        if (g == 0) {
            float2* ml = (float2*)(a.ws_ml + ((size_t)item * kHeads + head) * 2);
            *ml = make_float2(m_run, l_run);
        }
    }
}

// Merge the partial results of the splits of one sequence:
//   out = sum_s 2^(m_s - m*) acc_s / sum_s 2^(m_s - m*) l_s,  m* = max_s m_s.
// One thread per 4 consecutive output elements.
__global__ __launch_bounds__(256) void merge_splits_kernel(AttnArgs a)
{
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;        // over B*64*64 float4
    const int d4 = (int)(idx & 63);
    const int h = (int)((idx >> 6) & 63);
    const int b = (int)(idx >> 12);
    if (b >= a.B) return;
    int L = a.seq_lens[b];
    L = L < 0 ? 0 : (L > a.max_seq_len_hint ? a.max_seq_len_hint : L);
    float4* o = (float4*)(a.out + ((size_t)b * kHeads + h) * kHeadDim) + d4;
    if (L == 0) { *o = make_float4(0.f, 0.f, 0.f, 0.f); return; }
    const int n_valid = (L + a.chunk_tokens - 1) / a.chunk_tokens;    // <= n_splits
    const size_t item0 = (size_t)b * a.n_splits;
    float m = -INFINITY;
    for (int s = 0; s < n_valid; ++s) m = fmaxf(m, a.ws_ml[((item0 + s) * kHeads + h) * 2]);
    float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
    float l = 0.f;
    for (int s = 0; s < n_valid; ++s) {
        const float2 ml = *(const float2*)(a.ws_ml + ((item0 + s) * kHeads + h) * 2);
        const float w = fast_exp2(ml.x - m);
        const float4 v = *((const float4*)(a.ws_acc + ((item0 + s) * kHeads + h) * kHeadDim) + d4);
        sum.x += w * v.x; sum.y += w * v.y; sum.z += w * v.z; sum.w += w * v.w;
        l += w * ml.y;
    }
    const float inv = 1.0f / l;
    *o = make_float4(sum.x * inv, sum.y * inv, sum.z * inv, sum.w * inv);
}

// Copy the logical rows of every sequence out of a paged pool (test aid).
__global__ __launch_bounds__(256) void gather_paged_kernel(const uint32_t* pool, int32_t row_words,
                                                           const int32_t* block_table, int32_t max_blocks_per_seq,
                                                           const int32_t* seq_lens, int32_t hint, uint32_t* dst,
                                                           int64_t dst_seq_stride_tokens)
{
    const int b = blockIdx.y;
    const int blk = blockIdx.x;
    int L = seq_lens[b];
    L = L < 0 ? 0 : (L > hint ? hint : L);
    const int tok0 = blk * kPage;
    if (tok0 >= L) return;
    const int n_tok = (L - tok0 < kPage) ? L - tok0 : kPage;
    const int page = block_table[(size_t)b * max_blocks_per_seq + blk];
    const uint32_t* src = pool + (size_t)page * kPage * row_words;
    uint32_t* d = dst + ((size_t)b * dst_seq_stride_tokens + tok0) * row_words;
    for (int i = threadIdx.x; i < n_tok * row_words; i += 256) d[i] = src[i];
}

SplitPlan plan_splits(int32_t B, int32_t max_seq_len_hint, int32_t target_items)
{
    const int32_t max_tiles = (max_seq_len_hint + kTile - 1) / kTile;
    int32_t want = (target_items + B - 1) / B;
    if (want < 1) want = 1;
    if (want > max_tiles) want = max_tiles;
    const int32_t chunk_tiles = (max_tiles + want - 1) / want;
    SplitPlan p;
    p.chunk_tokens = chunk_tiles * kTile;
    p.n_splits = (max_tiles + chunk_tiles - 1) / chunk_tiles;
    return p;
}

hipError_t prepare_decode_attn_kernels()
{
    hipError_t e;
    e = hipFuncSetAttribute((const void*)decode_bf16_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize, kAttnLdsBytes);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void*)decode_bf16_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize, kAttnLdsBytes);
    return e;
}

hipError_t launch_decode_attn(const AttnArgs& a, mfa_kv_dtype kv_dtype, hipStream_t stream)
{
    if (kv_dtype != MFA_KV_BF16) return hipErrorNotSupported;
    const dim3 grid((unsigned)(a.B * a.n_splits));
    if (a.block_table)
        hipLaunchKernelGGL(decode_bf16_kernel<true>, grid, dim3(kAttnThreads), kAttnLdsBytes, stream, a);
    else
        hipLaunchKernelGGL(decode_bf16_kernel<false>, grid, dim3(kAttnThreads), kAttnLdsBytes, stream, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (a.n_splits > 1) {
        const unsigned blocks = (unsigned)(((size_t)a.B * kHeads * (kHeadDim / 4) + 255) / 256);
        hipLaunchKernelGGL(merge_splits_kernel, dim3(blocks), dim3(256), 0, stream, a);
        e = hipGetLastError();
    }
    return e;
}

hipError_t launch_gather_paged(const void* pool, int32_t row_bytes, const int32_t* block_table,
                               int32_t max_blocks_per_seq, const int32_t* seq_lens, int32_t max_seq_len_hint,
                               int32_t B, void* dst, int64_t dst_seq_stride_tokens, hipStream_t stream)
{
    const int blocks = (max_seq_len_hint + kPage - 1) / kPage;
    hipLaunchKernelGGL(gather_paged_kernel, dim3((unsigned)blocks, (unsigned)B), dim3(256), 0, stream,
                       (const uint32_t*)pool, row_bytes / 4, block_table, max_blocks_per_seq, seq_lens,
                       max_seq_len_hint, (uint32_t*)dst, dst_seq_stride_tokens);
    return hipGetLastError();
}

}  // namespace mfa

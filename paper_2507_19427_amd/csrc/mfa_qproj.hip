// Low-rank query path of MFA (paper, Section 2): c = x.W_qa, RMS normalisation over the
// rank axis, q = c_hat.W_qb.  Three launches on the caller's stream:
//   1. split-K bf16 MFMA GEMM, fp32 partial sums of c into the workspace;
//   2. reduce the partials, normalise, apply the gain, round to bf16;
//   3. bf16 MFMA GEMM writing q in bf16.
// With at most a few hundred rows of x both products are bound by streaming the weights
// once, so the GEMM is built like the attention kernel's value product: a workgroup owns a
// strip of 64 output columns and all (up to 128) rows of x, streams its [K, 64] slice of W
// through LDS with global->LDS direct loads (128 B per row, two stages of 512 rows = 64 KB each,
// one in flight while the other is multiplied), and feeds v_mfma_f32_16x16x32_bf16 with
//   A = W^T  (16 columns x 32 k) read with the LDS transposing read,
//   B = x^T  (32 k x 16 rows)    loaded from global memory (L2-resident) one stage ahead,
// giving C^T[column, row]; a lane ends up with 4 consecutive columns of one row.  The eight
// waves are 4 row groups x 2 interleaved halves of the k steps, so every x element is fetched
// by one wave only; the two halves are added through LDS at the end.  64-column strips give the
// second product (16384 columns) 256 workgroups, one per compute unit, each with 64 KB in flight.
#include "mfa_attn_core.hpp"

namespace mfa {

namespace {

constexpr int kStripN = 64;                  // output columns per workgroup
constexpr int kRowBytes = kStripN * 2;       // 128 B of W per k row
constexpr int kStageRows = 512;              // k rows per stage
constexpr int kStageBytes = kStageRows * kRowBytes;   // 64 KB
constexpr int kGemmLdsBytes = 2 * kStageBytes;
constexpr int kGemmThreads = 512;
constexpr int kStepsPerStage = kStageRows / 32;
constexpr int kColBlocks = kStripN / 16;

// Swizzle key of a W row in LDS: its 32-byte chunk c is stored at position c ^ key.  A transposing
// read touches rows 8g + 4t + i (g = 0..3, i = 0..3) at one chunk each.  Rows are 128 bytes, so rows
// of equal parity share their banks; with key = 2*(g & 1) + i/2 the four rows of equal parity read
// by each half of the wave (g = 0, 1 or g = 2, 3) take the four chunk positions once each.
__device__ __forceinline__ int w_key(int row) { return (((row >> 3) & 1) << 1) | ((row >> 1) & 1); }

// OUT_BF16 = false: fp32 partial sums to out[(kz*rows_pad + m)*N + n] for every row of the tile.
// OUT_BF16 = true : bf16 result to out[m*N + n] for m < M (requires gridDim.z == 1).
// X_TILED = false: x is row-major [M, K].
// X_TILED = true : x is stored k-step-major, element (m, k) at ((k/32)*rows_pad + m)*32 + k%32, so
//                  that the 16 rows x 64 B a wave loads per k step are contiguous.
template <bool OUT_BF16, bool X_TILED>
__global__ __launch_bounds__(kGemmThreads) void gemm_stream_kernel(const uint16_t* __restrict__ X,
                                                                   const uint16_t* __restrict__ W,
                                                                   void* __restrict__ out, int M, int K, int N,
                                                                   int k_per_split, int rows_pad)
{
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    const lds_ptr_t lds_base = (lds_ptr_t)smem;
    const uint32_t lds_addr0 = (uint32_t)(uintptr_t)lds_base;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int mp = wave & 3;                  // rows 32*mp .. 32*mp+31 of the 128-row tile
    const int kh = wave >> 2;                 // takes the k steps of every stage with (step & 1) == kh
    const int n = lane & 15;
    const int g = lane >> 4;

    const int n0 = blockIdx.x * kStripN;
    const int m0 = blockIdx.y * kQProjRows;
    const int kz = blockIdx.z;
    const int k_begin = kz * k_per_split;
    const int k_end = (k_begin + k_per_split < K) ? k_begin + k_per_split : K;
    const int n_stages = (k_end - k_begin + kStageRows - 1) / kStageRows;

    // Direct load of one stage of W: 64 loads of 8 rows; wave w issues loads 8w .. 8w+7.
    auto issue_stage = [&](int stage, int slot) {
        const int k0 = k_begin + stage * kStageRows;
        const int rows_valid = (k_end - k0 < kStageRows) ? k_end - k0 : kStageRows;   // multiple of 32
        const int p8 = lane & 7;                                       // 16-byte position in the 128-byte row
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int first_row = 8 * (8 * wave + i);                  // wave-uniform
            if (first_row < rows_valid) {
                const int row = first_row + (lane >> 3);
                const int c16 = ((((p8 >> 1) ^ w_key(row)) << 1) | (p8 & 1));
                const unsigned char* src = (const unsigned char*)W + ((size_t)(k0 + row) * N + n0) * 2 + c16 * 16;
                load_to_lds_16B(src, lds_addr0 + slot * kStageBytes + first_row * kRowBytes);
            }
        }
    };

    // x fragments of this wave's k steps of one stage: lane (row n of a 16-row block, k group g)
    // holds x[row][k0 + 32*(2j + kh) + 8g .. +7].  Every x element is loaded by exactly one wave.
    // Two sets: the next stage's fragments are requested right after its W, a whole stage ahead.
    constexpr int kMySteps = kStepsPerStage / 2;
    bf16x8 xf[2][2][kMySteps];                // [buffer][row block][own k step]
    int xrow[2];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
        const int r = m0 + 32 * mp + 16 * mb + n;
        xrow[mb] = r < M ? r : M - 1;         // rows past M repeat the last one; their results are not stored
    }
    auto load_x_stage = [&](int stage, int buf) {
        const int k0 = k_begin + stage * kStageRows;
#pragma unroll
        for (int j = 0; j < kMySteps; ++j) {
            int k = k0 + 32 * (2 * j + kh) + 8 * g;
            k = k + 8 <= K ? k : K - 8;       // steps past k_end are never used; keep the address inside x
#pragma unroll
            for (int mb = 0; mb < 2; ++mb) {
                const size_t idx = X_TILED ? ((size_t)(k >> 5) * rows_pad + xrow[mb]) * 32 + (k & 31)
                                           : (size_t)xrow[mb] * K + k;
                xf[buf][mb][j] = *(const bf16x8*)(X + idx);
            }
        }
    };

    f32x4 acc[2][kColBlocks];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < kColBlocks; ++j) acc[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};

    const int a_lane_off = (8 * g + (n >> 2)) * kRowBytes + ((n & 3) << 3);   // row 8g + i, 8 bytes per lane
    const int a_key = ((g & 1) << 1) | ((n >> 3) & 1);                        // w_key of rows 8g + 4t + i

    // A operands of one k step: for each 16-column block the two transposing reads that make W^T.
    struct AFrag { union { bf16x8 v; s16x4 h[2]; } nb[kColBlocks]; };
    auto read_a = [&](AFrag& f, int base, int ks) {
#pragma unroll
        for (int nb = 0; nb < kColBlocks; ++nb)
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int off = base + (32 * ks + 4 * t) * kRowBytes + a_lane_off + ((nb ^ a_key) << 5);
                f.nb[nb].h[t] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_AT(s16x4, lds_base, off));
            }
    };
    auto multiply = [&](const AFrag& f, const bf16x8& x0, const bf16x8& x1) {
#pragma unroll
        for (int nb = 0; nb < kColBlocks; ++nb) {
            acc[0][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.nb[nb].v, x0, acc[0][nb], 0, 0, 0);
            acc[1][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.nb[nb].v, x1, acc[1][nb], 0, 0, 0);
        }
    };
    // The A operands of the next own step are read from LDS while the current one is multiplied, so
    // that the LDS latency hides behind eight MFMAs instead of stalling each pair.
    auto compute_stage = [&](int stage, int slot, int buf) {
        const int k0 = k_begin + stage * kStageRows;
        const int steps = ((k_end - k0 < kStageRows) ? k_end - k0 : kStageRows) / 32;
        const int base = slot * kStageBytes;
        AFrag fa, fb;
        if (steps == kStepsPerStage) {                 // full stage: straight-line code
            // (the scheduling fences keep the compiler from sinking the reads back to their uses)
            read_a(fa, base, kh);
#pragma unroll
            for (int j = 0; j < kMySteps; j += 2) {
                read_a(fb, base, 2 * (j + 1) + kh);
                __builtin_amdgcn_sched_barrier(0);
                multiply(fa, xf[buf][0][j], xf[buf][1][j]);
                __builtin_amdgcn_sched_barrier(0);
                if (j + 2 < kMySteps) read_a(fa, base, 2 * (j + 2) + kh);
                __builtin_amdgcn_sched_barrier(0);
                multiply(fb, xf[buf][0][j + 1], xf[buf][1][j + 1]);
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
#pragma unroll
            for (int j = 0; j < kMySteps; ++j)
                if (2 * j + kh < steps) {
                    read_a(fa, base, 2 * j + kh);
                    multiply(fa, xf[buf][0][j], xf[buf][1][j]);
                }
        }
    };

    // While a stage is multiplied the next one (W by direct loads, x into the other register set) is
    // in flight; everything requested is awaited at the barrier that opens a stage.
    // Workgroups walk the stages of their k range starting at different points (strip index modulo
    // the stage count) and wrapping round: at any moment the strips that share an L2 then ask it for
    // different parts of x instead of all for the same lines.
    const int phase = (int)((blockIdx.x >> 3) % (unsigned)n_stages);   // workgroups 8 apart share an XCD's L2
    auto stage_of = [&](int it) { const int s = it + phase; return s < n_stages ? s : s - n_stages; };
    issue_stage(stage_of(0), 0);
    load_x_stage(stage_of(0), 0);
    for (int st = 0; st < n_stages; st += 2) {
        // even step: slot 0, x buffer 0
        wait_vmem_all();
        __syncthreads();
        if (st + 1 < n_stages) { issue_stage(stage_of(st + 1), 1); load_x_stage(stage_of(st + 1), 1); }
        compute_stage(stage_of(st), 0, 0);
        if (st + 1 >= n_stages) break;
        // odd step: slot 1, x buffer 1
        wait_vmem_all();
        __syncthreads();
        if (st + 2 < n_stages) { issue_stage(stage_of(st + 2), 0); load_x_stage(stage_of(st + 2), 0); }
        compute_stage(stage_of(st + 1), 1, 1);
    }

    // The two waves that share 32 rows (kh = 0, 1) hold sums over disjoint k steps: exchange halves
    // through LDS (the stage buffers are dead, no direct load is in flight); kh 0 finishes column
    // blocks 0..1, kh 1 blocks 2..3.  Fixed order ((kh 0 part) + (kh 1 part)) keeps the result
    // reproducible.
    __syncthreads();
    {
        constexpr int kHalf = kColBlocks / 2;
        const int mine = (mp * 2 + kh) * 2 * kHalf;   // slots of 1 KB: [row block][kHalf column blocks]
        const int theirs = (mp * 2 + (kh ^ 1)) * 2 * kHalf;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int j = 0; j < kHalf; ++j) {
                const f32x4 v = kh == 0 ? acc[mb][kHalf + j] : acc[mb][j];
                *LDS_AT(f32x4, lds_base, (mine + mb * kHalf + j) * 1024 + lane * 16) = v;
            }
        __syncthreads();
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
            const int m = m0 + 32 * mp + 16 * mb + n;
#pragma unroll
            for (int j = 0; j < kHalf; ++j) {
                const f32x4 other = *LDS_AT(f32x4, lds_base, (theirs + mb * kHalf + j) * 1024 + lane * 16);
                const f32x4 own = kh == 0 ? acc[mb][j] : acc[mb][kHalf + j];
                const f32x4 r = kh == 0 ? own + other : other + own;     // always (kh 0 part) + (kh 1 part)
                const int col = n0 + 16 * (kHalf * kh + j) + 4 * g;
                if (OUT_BF16) {
                    if (m < M) {
                        union { __bf16 h[4]; uint2 u; } o;
#pragma unroll
                        for (int i = 0; i < 4; ++i) o.h[i] = (__bf16)r[i];
                        *(uint2*)((__bf16*)out + (size_t)m * N + col) = o.u;
                    }
                } else {
                    *(f32x4*)((float*)out + ((size_t)kz * rows_pad + m) * N + col) = r;
                }
            }
        }
    }
}

// One workgroup per row of x: c = sum of the split-K partials (in split order),
// c_hat = c / sqrt(mean(c^2) + eps) * gain.  A thread owns float4 pieces of the row; the partials
// of a piece are loaded eight splits at a time so that the loads are in flight together.
__global__ __launch_bounds__(256) void rmsnorm_reduce_kernel(const float* __restrict__ ws_c, const float* __restrict__ gain,
                                                             __bf16* __restrict__ chat, int r, int split_k, int rows_pad,
                                                             float eps)
{
    __shared__ float red[4];
    extern __shared__ float crow[];           // r floats: the reduced row, kept between the two passes
    const int m = blockIdx.x;
    const int tid = threadIdx.x;
    const size_t split_stride = (size_t)rows_pad * r;
    float ss = 0.f;
    for (int j = 4 * tid; j < r; j += 1024) {
        const float* p = ws_c + (size_t)m * r + j;
        f32x4 c = {0.f, 0.f, 0.f, 0.f};
        for (int z0 = 0; z0 < split_k; z0 += 8) {
            f32x4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int z = z0 + u < split_k ? z0 + u : split_k - 1;
                v[u] = *(const f32x4*)(p + (size_t)z * split_stride);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (z0 + u < split_k) c += v[u];
        }
        *(f32x4*)(crow + j) = c;
        ss += c[0] * c[0] + c[1] * c[1] + c[2] * c[2] + c[3] * c[3];
    }
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    const float total = red[0] + red[1] + red[2] + red[3];
    const float inv = 1.0f / sqrtf(total / (float)r + eps);
    for (int j = 4 * tid; j < r; j += 1024) {
        const f32x4 c = *(const f32x4*)(crow + j);
        union { __bf16 h[4]; uint2 u; } o;
#pragma unroll
        for (int i = 0; i < 4; ++i) o.h[i] = (__bf16)(c[i] * inv * (gain ? gain[j + i] : 1.0f));
        *(uint2*)(chat + ((size_t)(j >> 5) * rows_pad + m) * 32 + (j & 31)) = o.u;   // k-step-major for the second product
    }
}

}  // namespace

QProjPlan plan_qproj(int32_t d_model, int32_t q_rank)
{
    const int32_t strips = q_rank / kStripN;
    int32_t want = 256 / (strips > 0 ? strips : 1);
    if (want < 1) want = 1;
    if (want > 16) want = 16;
    const int32_t ksteps = d_model / 32;
    const int32_t per = (ksteps + want - 1) / want;
    QProjPlan p;
    p.k_per_split = per * 32;
    p.split_k = (ksteps + per - 1) / per;
    return p;
}

hipError_t prepare_query_proj_kernels()
{
    hipError_t e = hipFuncSetAttribute((const void*)gemm_stream_kernel<false, false>, hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLdsBytes);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute((const void*)gemm_stream_kernel<true, true>, hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLdsBytes);
}

hipError_t launch_query_proj(const QProjArgs& a, hipStream_t stream)
{
    const int m_blocks = (a.B + kQProjRows - 1) / kQProjRows;
    const int rows_pad = m_blocks * kQProjRows;
    hipLaunchKernelGGL((gemm_stream_kernel<false, false>), dim3(a.q_rank / kStripN, m_blocks, a.split_k), dim3(kGemmThreads),
                       kGemmLdsBytes, stream, (const uint16_t*)a.x, (const uint16_t*)a.w_qa, (void*)a.ws_c, a.B,
                       a.d_model, a.q_rank, a.k_per_split, rows_pad);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(rmsnorm_reduce_kernel, dim3(a.B), dim3(256), a.q_rank * sizeof(float), stream,
                       (const float*)a.ws_c, a.gain, (__bf16*)a.ws_chat, a.q_rank, a.split_k, rows_pad, a.eps);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((gemm_stream_kernel<true, true>), dim3(a.n_out / kStripN, m_blocks, 1), dim3(kGemmThreads),
                       kGemmLdsBytes, stream, (const uint16_t*)a.ws_chat, (const uint16_t*)a.w_qb, a.q_out, a.B,
                       a.q_rank, a.n_out, a.q_rank, rows_pad);
    return hipGetLastError();
}

}  // namespace mfa

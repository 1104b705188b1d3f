// Low-rank query path of MFA (paper, Section 2): c = x.W_qa, RMS normalisation over the
// rank axis, q = c_hat.W_qb.  Three launches on the caller's stream:
//   1. split-K bf16 MFMA GEMM, fp32 partial sums of c into the workspace;
//   2. reduce the partials, normalise, apply the gain, round to bf16;
//   3. bf16 MFMA GEMM writing q in bf16.
// With at most a few hundred rows of x both products are bound by streaming the
// weights once; every workgroup covers all (up to 128) rows of x so each weight is
// read from HBM exactly once.
#include "mfa_internal.hpp"

namespace mfa {

namespace {

constexpr int kTileN = 64;       // output columns per workgroup
constexpr int kStepK = 32;       // one MFMA K step
constexpr int kLdsRow = 80;      // bytes per LDS row: 32 bf16 + 16 B pad (odd multiple of 16 B -> no bank clash)

// OUT_BF16 = false: fp32 partial sums to out[(kz*rows_pad + m)*N + n] for every row of the tile.
// OUT_BF16 = true : bf16 result to out[m*N + n] for m < M.
template <bool OUT_BF16>
__global__ __launch_bounds__(256) void gemm_rows128_kernel(const uint16_t* __restrict__ A, const uint16_t* __restrict__ W,
                                                           void* __restrict__ out, int M, int K, int N, int k_per_split,
                                                           int rows_pad)
{
    __shared__ __attribute__((aligned(16))) unsigned char sA[kQProjRows * kLdsRow];
    __shared__ __attribute__((aligned(16))) unsigned char sW[kTileN * kLdsRow];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int n = lane & 15, g = lane >> 4;
    const int n0 = blockIdx.x * kTileN;
    const int m0 = blockIdx.y * kQProjRows;
    const int kz = blockIdx.z;
    const int k_begin = kz * k_per_split;
    const int k_end = k_begin + k_per_split;

    f32x4 acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};

    for (int k0 = k_begin; k0 < k_end; k0 += kStepK) {
        __syncthreads();
        // A tile: 128 rows x 32 k, two 16-byte pieces per thread
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int r = (tid >> 2) + 64 * i;
            const int c = tid & 3;
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (m0 + r < M) v = *(const uint4*)(A + (size_t)(m0 + r) * K + k0 + 8 * c);
            *(uint4*)(sA + r * kLdsRow + 16 * c) = v;
        }
        // W tile: 32 k x 64 n, transposed into [n][k] so that a lane reads 8 consecutive k
        {
            const int kk = tid >> 3;
            const int n8 = (tid & 7) * 8;
            union { uint4 v; uint16_t h[8]; } w;
            w.v = *(const uint4*)(W + (size_t)(k0 + kk) * N + n0 + n8);
#pragma unroll
            for (int e = 0; e < 8; ++e) *(uint16_t*)(sW + (n8 + e) * kLdsRow + 2 * kk) = w.h[e];
        }
        __syncthreads();
        bf16x8 bfrag[4];
#pragma unroll
        for (int nb = 0; nb < 4; ++nb) bfrag[nb] = *(const bf16x8*)(sW + (16 * nb + n) * kLdsRow + 16 * g);
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
            const bf16x8 afrag = *(const bf16x8*)(sA + (32 * wave + 16 * mb + n) * kLdsRow + 16 * g);
#pragma unroll
            for (int nb = 0; nb < 4; ++nb)
                acc[mb][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(afrag, bfrag[nb], acc[mb][nb], 0, 0, 0);
        }
    }

    // lane holds C[row 4g+i][col n] of each 16x16 block
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < 4; ++nb)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int m = m0 + 32 * wave + 16 * mb + 4 * g + i;
                const int col = n0 + 16 * nb + n;
                if (OUT_BF16) {
                    if (m < M) ((__bf16*)out)[(size_t)m * N + col] = (__bf16)acc[mb][nb][i];
                } else {
                    ((float*)out)[((size_t)kz * rows_pad + m) * N + col] = acc[mb][nb][i];
                }
            }
}

// One workgroup per row of x: c = sum of the split-K partials, c_hat = c / sqrt(mean(c^2) + eps) * gain.
__global__ __launch_bounds__(256) void rmsnorm_reduce_kernel(const float* __restrict__ ws_c, const float* __restrict__ gain,
                                                             __bf16* __restrict__ chat, int r, int split_k, int rows_pad,
                                                             float eps)
{
    __shared__ float red[4];
    const int m = blockIdx.x;
    const int tid = threadIdx.x;
    float ss = 0.f;
    for (int j = tid; j < r; j += 256) {
        float c = 0.f;
        for (int z = 0; z < split_k; ++z) c += ws_c[((size_t)z * rows_pad + m) * r + j];
        ss += c * c;
    }
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    const float total = red[0] + red[1] + red[2] + red[3];
    const float inv = 1.0f / sqrtf(total / (float)r + eps);
    for (int j = tid; j < r; j += 256) {
        float c = 0.f;
        for (int z = 0; z < split_k; ++z) c += ws_c[((size_t)z * rows_pad + m) * r + j];
        const float gj = gain ? gain[j] : 1.0f;
        chat[(size_t)m * r + j] = (__bf16)(c * inv * gj);
    }
}

}  // namespace

int32_t qproj_split_k(int32_t d_model)
{
    for (int32_t s = 8; s > 1; --s)
        if (d_model % (kStepK * s) == 0) return s;
    return 1;
}

hipError_t launch_query_proj(const QProjArgs& a, hipStream_t stream)
{
    const int m_blocks = (a.B + kQProjRows - 1) / kQProjRows;
    const int rows_pad = m_blocks * kQProjRows;
    hipLaunchKernelGGL(gemm_rows128_kernel<false>, dim3(a.q_rank / kTileN, m_blocks, a.split_k), dim3(256), 0, stream,
                       (const uint16_t*)a.x, (const uint16_t*)a.w_qa, (void*)a.ws_c, a.B, a.d_model, a.q_rank,
                       a.d_model / a.split_k, rows_pad);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(rmsnorm_reduce_kernel, dim3(a.B), dim3(256), 0, stream, (const float*)a.ws_c, a.gain,
                       (__bf16*)a.ws_chat, a.q_rank, a.split_k, rows_pad, a.eps);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(gemm_rows128_kernel<true>, dim3(a.n_out / kTileN, m_blocks, 1), dim3(256), 0, stream,
                       (const uint16_t*)a.ws_chat, (const uint16_t*)a.w_qb, a.q_out, a.B, a.q_rank, a.n_out, a.q_rank,
                       rows_pad);
    return hipGetLastError();
}

}  // namespace mfa

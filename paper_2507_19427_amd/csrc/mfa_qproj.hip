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
// MB = 2 or 1: 16-row blocks per wave; a workgroup covers 64 * MB rows of x (MB = 1 when there are
//                  no more than 64 rows: half the x traffic and MFMA work).
// NS = 1, 2 or 4: adjacent 64-column strips per workgroup.  A stage holds 512 / NS k rows of each; the x
//                  fragments of a k step are multiplied into all NS strips, so x is fetched once per
//                  64 * NS columns (for products whose x is as large as a workgroup's share of W: the
//                  output projection).
template <bool OUT_BF16, bool X_TILED, int MB, int NS>
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
    const int mp = wave & 3;                  // rows 16*MB*mp .. of the workgroup's tile
    const int kh = wave >> 2;                 // takes the k steps of every stage with (step & 1) == kh
    const int n = lane & 15;
    const int g = lane >> 4;

    constexpr int kSubRows = kStageRows / NS;            // k rows of one stage
    constexpr int kSubBytes = kSubRows * kRowBytes;       // one strip's part of a stage buffer
    constexpr int kStepsPerStage = kSubRows / 32;
    constexpr int kCols = kColBlocks * NS;                // 16-column blocks of the workgroup
    const int n0 = blockIdx.x * kStripN * NS;
    const int m0 = blockIdx.y * 64 * MB;
    const int kz = blockIdx.z;
    const int k_begin = kz * k_per_split;
    const int k_end = (k_begin + k_per_split < K) ? k_begin + k_per_split : K;
    const int n_stages = (k_end - k_begin + kSubRows - 1) / kSubRows;

    // Direct load of one stage of W: 64 loads of 8 rows; wave w issues loads 8w .. 8w+7.  Load l brings rows
    // 8*(l % (64/NS)) .. of strip l / (64/NS).
    auto issue_stage = [&](int stage, int slot) {
        const int k0 = k_begin + stage * kSubRows;
        const int rows_valid = (k_end - k0 < kSubRows) ? k_end - k0 : kSubRows;       // multiple of 32
        const int p8 = lane & 7;                                       // 16-byte position in the 128-byte row
        const unsigned char* w_stage = (const unsigned char*)W + ((size_t)k0 * N + n0) * 2;   // wave-uniform
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int l = 8 * wave + i;                                // wave-uniform
            const int strip = l / (64 / NS);
            const int first_row = 8 * (l % (64 / NS));
            if (first_row < rows_valid) {
                const int row = first_row + (lane >> 3);
                const int c16 = ((((p8 >> 1) ^ w_key(row)) << 1) | (p8 & 1));
                load_to_lds_16B(w_stage, (uint32_t)(row * N * 2 + strip * kRowBytes + c16 * 16),
                                lds_addr0 + slot * kStageBytes + strip * kSubBytes + first_row * kRowBytes);
            }
        }
    };

    // x fragments of this wave's k steps of one stage: lane (row n of a 16-row block, k group g)
    // holds x[row][k0 + 32*(2j + kh) + 8g .. +7].  Every x element is loaded by exactly one wave.
    // Two sets: the next stage's fragments are requested right after its W, a whole stage ahead.
    constexpr int kMySteps = kStepsPerStage / 2;
    bf16x8 xf[2][MB][kMySteps];               // [buffer][row block][own k step]
    int xrow[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int r = m0 + 16 * MB * mp + 16 * mb + n;
        xrow[mb] = r < M ? r : M - 1;         // rows past M repeat the last one; their results are not stored
    }
    auto load_x_stage = [&](int stage, int buf) {
        const int k0 = k_begin + stage * kSubRows;
#pragma unroll
        for (int j = 0; j < kMySteps; ++j) {
            int k = k0 + 32 * (2 * j + kh) + 8 * g;
            k = k + 8 <= K ? k : K - 8;       // steps past k_end are never used; keep the address inside x
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                const size_t idx = X_TILED ? ((size_t)(k >> 5) * rows_pad + xrow[mb]) * 32 + (k & 31)
                                           : (size_t)xrow[mb] * K + k;
                xf[buf][mb][j] = *(const bf16x8*)(X + idx);
            }
        }
    };

    f32x4 acc[MB][kCols];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < kCols; ++j) acc[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};

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
    auto multiply = [&](const AFrag& f, int buf, int j, int strip) {
#pragma unroll
        for (int nb = 0; nb < kColBlocks; ++nb)
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
                acc[mb][strip * kColBlocks + nb] =
                    __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.nb[nb].v, xf[buf][mb][j], acc[mb][strip * kColBlocks + nb], 0, 0, 0);
    };
    // A stage is worked off in units (own k step j, strip): unit u = j * NS + strip.  The A operands of
    // the next unit are read from LDS while the current one is multiplied, so that the LDS latency
    // hides behind the MFMAs instead of stalling each pair.
    constexpr int kUnits = kMySteps * NS;
    static_assert(kUnits % 2 == 0, "units are taken in pairs");
    auto compute_stage = [&](int stage, int slot, int buf) {
        const int k0 = k_begin + stage * kSubRows;
        const int steps = ((k_end - k0 < kSubRows) ? k_end - k0 : kSubRows) / 32;
        const int base = slot * kStageBytes;
        auto unit_base = [&](int u) { return base + (u % NS) * kSubBytes; };
        auto unit_step = [&](int u) { return 2 * (u / NS) + kh; };
        AFrag fa, fb;
        if (steps == kStepsPerStage) {                 // full stage: straight-line code
            // (the scheduling fences keep the compiler from sinking the reads back to their uses)
            read_a(fa, unit_base(0), unit_step(0));
#pragma unroll
            for (int u = 0; u < kUnits; u += 2) {
                read_a(fb, unit_base(u + 1), unit_step(u + 1));
                __builtin_amdgcn_sched_barrier(0);
                multiply(fa, buf, u / NS, u % NS);
                __builtin_amdgcn_sched_barrier(0);
                if (u + 2 < kUnits) read_a(fa, unit_base(u + 2), unit_step(u + 2));
                __builtin_amdgcn_sched_barrier(0);
                multiply(fb, buf, (u + 1) / NS, (u + 1) % NS);
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
#pragma unroll
            for (int u = 0; u < kUnits; ++u)
                if (unit_step(u) < steps) {
                    read_a(fa, unit_base(u), unit_step(u));
                    multiply(fa, buf, u / NS, u % NS);
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
    // blocks of the lower half, kh 1 those of the upper half.  Fixed order ((kh 0 part) + (kh 1 part)) keeps the result
    // reproducible.
    __syncthreads();
    {
        constexpr int kHalf = kCols / 2;
        const int mine = (mp * 2 + kh) * MB * kHalf;  // slots of 1 KB: [row block][kHalf column blocks]
        const int theirs = (mp * 2 + (kh ^ 1)) * MB * kHalf;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int j = 0; j < kHalf; ++j) {
                const f32x4 v = kh == 0 ? acc[mb][kHalf + j] : acc[mb][j];
                *LDS_AT(f32x4, lds_base, (mine + mb * kHalf + j) * 1024 + lane * 16) = v;
            }
        __syncthreads();
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const int m = m0 + 16 * MB * mp + 16 * mb + n;
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

// ---- the new token's cache record (Section 6: the cache holds one key row and one value row per
// token, 8 bits per element in the deployed system).
// One workgroup per sequence, thread t owns key element t and value element t.  The fp32 rows are the
// sum of the projection's split-K partials in split order.  bf16 cache: round to nearest even.
// fp8 cache: per token and tensor scale = max(max|x|, 1e-12) / 448 and code = e4m3(x / scale), the
// quotient clamped to +-448; all in single precision with correctly rounded divisions, so that the
// codes are a function of the fp32 row alone.  The row written is seq_lens[b] (the tokens already
// cached); a row outside the cache or the block table is not written.
// 4-bit cache (BITS = 4): the same with e2m1's largest magnitude 6 in place of 448; the codes of
// elements 2i and 2i + 1 share byte i, the even one in the low four bits.
template <int BITS, bool PAGED>
__global__ __launch_bounds__(kHeadDim) void kv_record_kernel(const float* __restrict__ parts, int split_k, int rows_pad,
                                                             KvAppendArgs a)
{
    __shared__ float red[2][kHeadDim / 64];
    const int b = blockIdx.x;
    const int t = threadIdx.x;
    float kx = -0.f, vx = -0.f;                         // -0 + x = x for every x, the sign of a zero included
    for (int z0 = 0; z0 < split_k; z0 += 8) {           // eight splits' loads in flight together, summed in split order
        float kp[8], vp[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int z = z0 + u < split_k ? z0 + u : split_k - 1;
            const float* row = parts + ((size_t)z * rows_pad + b) * kKvWidth;
            kp[u] = row[t];
            vp[u] = row[kHeadDim + t];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (z0 + u < split_k) { kx += kp[u]; vx += vp[u]; }
    }
    const int pos = a.seq_lens[b];
    int64_t row;
    if (PAGED) {
        const int blk = pos / kPage;
        if (pos < 0 || blk >= a.max_blocks_per_seq) return;
        const int page = a.block_table[(size_t)b * a.max_blocks_per_seq + blk];
        if (page < 0 || page >= a.n_pages) return;                  // never write outside the pools
        row = (int64_t)page * kPage + pos % kPage;
    } else {
        if (pos < 0 || pos >= a.seq_stride_tokens) return;
        row = (int64_t)b * a.seq_stride_tokens + pos;
    }
    if (BITS == 16) {
        ((__bf16*)a.k)[row * kHeadDim + t] = (__bf16)kx;
        ((__bf16*)a.v)[row * kHeadDim + t] = (__bf16)vx;
        return;
    }
    float ka = fabsf(kx), va = fabsf(vx);
    for (int off = 32; off > 0; off >>= 1) {
        ka = fmaxf(ka, __shfl_xor(ka, off));
        va = fmaxf(va, __shfl_xor(va, off));
    }
    if ((t & 63) == 0) { red[0][t >> 6] = ka; red[1][t >> 6] = va; }
    __syncthreads();
    ka = fmaxf(fmaxf(red[0][0], red[0][1]), fmaxf(red[0][2], red[0][3]));
    va = fmaxf(fmaxf(red[1][0], red[1][1]), fmaxf(red[1][2], red[1][3]));
    constexpr float kTop = BITS == 8 ? 448.0f : 6.0f;
    const float ks = fmaxf(ka, 1e-12f) / kTop;
    const float vs = fmaxf(va, 1e-12f) / kTop;
    const float ky = fminf(fmaxf(kx / ks, -kTop), kTop);
    const float vy = fminf(fmaxf(vx / vs, -kTop), kTop);
    if (BITS == 8) {
        ((uint8_t*)a.k)[row * kHeadDim + t] = (uint8_t)(__builtin_amdgcn_cvt_pk_fp8_f32(ky, 0.f, 0, false) & 0xFF);
        ((uint8_t*)a.v)[row * kHeadDim + t] = (uint8_t)(__builtin_amdgcn_cvt_pk_fp8_f32(vy, 0.f, 0, false) & 0xFF);
    } else {
        // the odd neighbour's quotient comes over by a lane shuffle; the even thread converts and stores the pair
        const float ky1 = __shfl_down(ky, 1), vy1 = __shfl_down(vy, 1);
        if ((t & 1) == 0) {
            ((uint8_t*)a.k)[row * (kHeadDim / 2) + (t >> 1)] = (uint8_t)(__builtin_amdgcn_cvt_scalef32_pk_fp4_f32(0u, ky, ky1, 1.0f, 0) & 0xFF);
            ((uint8_t*)a.v)[row * (kHeadDim / 2) + (t >> 1)] = (uint8_t)(__builtin_amdgcn_cvt_scalef32_pk_fp4_f32(0u, vy, vy1, 1.0f, 0) & 0xFF);
        }
    }
    if (t == 0) { a.k_scale[row] = ks; a.v_scale[row] = vs; }
}
static_assert(kHeadDim == 256, "kv_record_kernel reduces over four waves");

// fp32 [M, K] -> bf16, k-step-major: element (m, k) at ((k/32)*rows_pad + m)*32 + k%32.
__global__ __launch_bounds__(256) void to_bf16_tiled_kernel(const float* __restrict__ src, __bf16* __restrict__ dst, int M, int K,
                                                            int rows_pad)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;          // over M * K / 4
    if (i >= (size_t)M * K / 4) return;
    const int m = (int)(i / (K / 4));
    const int k = (int)(i % (K / 4)) * 4;
    const f32x4 v = *(const f32x4*)(src + (size_t)m * K + k);
    union { __bf16 h[4]; uint2 u; } o;
#pragma unroll
    for (int j = 0; j < 4; ++j) o.h[j] = (__bf16)v[j];
    *(uint2*)(dst + ((size_t)(k >> 5) * rows_pad + m) * 32 + (k & 31)) = o.u;
}

// y[m][n] = bf16(sum over splits, in split order, of the fp32 partials).
__global__ __launch_bounds__(256) void reduce_partials_bf16_kernel(const float* __restrict__ parts, __bf16* __restrict__ y, int M, int N,
                                                                   int split_k, int rows_pad)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;          // over M * N / 4
    if (i >= (size_t)M * N / 4) return;
    const int m = (int)(i / (N / 4));
    const int n = (int)(i % (N / 4)) * 4;
    f32x4 c = {0.f, 0.f, 0.f, 0.f};
    for (int z = 0; z < split_k; ++z) c += *(const f32x4*)(parts + ((size_t)z * rows_pad + m) * N + n);
    union { __bf16 h[4]; uint2 u; } o;
#pragma unroll
    for (int j = 0; j < 4; ++j) o.h[j] = (__bf16)c[j];
    *(uint2*)(y + (size_t)m * N + n) = o.u;
}

}  // namespace

namespace {

// One streaming product: rows of x in tiles of 128 (64 when there are no more), strips of 64 columns (groups of
// two or four strips when the plan says so: fp32 partial output, k-step-major x, at most 128 rows), k splits.
template <bool OUT_BF16, bool X_TILED>
hipError_t launch_gemm(const void* X, const void* Wt, void* out, int M, int K, int N, const QProjPlan& plan, int split_k,
                       int rows_pad, hipStream_t stream)
{
    if (plan.strips_per_wg > 1) {
        if constexpr (!OUT_BF16 && X_TILED) {
            const int ns = plan.strips_per_wg;
            if (M > 128 || (ns != 2 && ns != 4) || (ns == 4 && M > 64) || N % (ns * kStripN) != 0) return hipErrorInvalidValue;
            const dim3 grid(N / (ns * kStripN), 1, split_k);
            const void* kernel = M <= 64 ? (ns == 2 ? (const void*)gemm_stream_kernel<false, true, 1, 2> : (const void*)gemm_stream_kernel<false, true, 1, 4>)
                                         : (const void*)gemm_stream_kernel<false, true, 2, 2>;
            const uint16_t* xp = (const uint16_t*)X;
            const uint16_t* wp = (const uint16_t*)Wt;
            int k_per_split = plan.k_per_split;
            void* params[] = {&xp, &wp, &out, &M, &K, &N, &k_per_split, &rows_pad};
            return hipLaunchKernel(kernel, grid, dim3(kGemmThreads), params, kGemmLdsBytes, stream);
        } else {
            return hipErrorInvalidValue;
        }
    }
    if (M <= 64)
        hipLaunchKernelGGL((gemm_stream_kernel<OUT_BF16, X_TILED, 1, 1>), dim3(N / kStripN, 1, split_k), dim3(kGemmThreads), kGemmLdsBytes,
                           stream, (const uint16_t*)X, (const uint16_t*)Wt, out, M, K, N, plan.k_per_split, rows_pad);
    else
        hipLaunchKernelGGL((gemm_stream_kernel<OUT_BF16, X_TILED, 2, 1>), dim3(N / kStripN, (M + 127) / 128, split_k), dim3(kGemmThreads),
                           kGemmLdsBytes, stream, (const uint16_t*)X, (const uint16_t*)Wt, out, M, K, N, plan.k_per_split, rows_pad);
    return hipGetLastError();
}

}  // namespace

QProjPlan plan_linear(int32_t K, int32_t N, int32_t strips_per_wg)
{
    const int32_t strips = N / (kStripN * strips_per_wg);
    int32_t want = 256 / (strips > 0 ? strips : 1);
    if (want < 1) want = 1;
    if (want > 32) want = 32;
    const int32_t ksteps = K / 32;
    const int32_t per = (ksteps + want - 1) / want;
    QProjPlan p;
    p.k_per_split = per * 32;
    p.split_k = (ksteps + per - 1) / per;
    p.strips_per_wg = strips_per_wg;
    return p;
}

// Output projection: with at most 64 rows a workgroup's share of the activations is as large as its share
// of W, so groups of four strips (activations fetched once per 256 columns) pay for the fourfold k split
// (16384 -> 7168 on MI355X: 66.6 us with single strips, 54.8 with pairs, 48.6 with fours).  With 65 to 128
// rows: pairs (whole call 105 -> 82 us).
QProjPlan plan_out_proj(int32_t K, int32_t N, int32_t B)
{
    int32_t ns = 1;
    if (B <= 64) ns = N % (4 * kStripN) == 0 ? 4 : (N % (2 * kStripN) == 0 ? 2 : 1);
    else if (B <= 128) ns = N % (2 * kStripN) == 0 ? 2 : 1;      // (four strips of 128 rows do not fit the registers)
    return plan_linear(K, N, ns);
}

hipError_t prepare_query_proj_kernels()
{
    const void* kernels[] = {(const void*)gemm_stream_kernel<false, false, 1, 1>, (const void*)gemm_stream_kernel<false, false, 2, 1>,
                             (const void*)gemm_stream_kernel<true, true, 1, 1>, (const void*)gemm_stream_kernel<true, true, 2, 1>,
                             (const void*)gemm_stream_kernel<false, true, 1, 1>, (const void*)gemm_stream_kernel<false, true, 2, 1>,
                             (const void*)gemm_stream_kernel<false, true, 1, 2>, (const void*)gemm_stream_kernel<false, true, 1, 4>,
                             (const void*)gemm_stream_kernel<false, true, 2, 2>};
    for (const void* k : kernels) {
        const hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLdsBytes);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_query_proj(const QProjArgs& a, hipStream_t stream)
{
    const int m_blocks = (a.B + kQProjRows - 1) / kQProjRows;
    const int rows_pad = m_blocks * kQProjRows;
    QProjPlan plan;
    plan.split_k = a.split_k;
    plan.k_per_split = a.k_per_split;
    plan.strips_per_wg = 1;
    hipError_t e = launch_gemm<false, false>(a.x, a.w_qa, a.ws_c, a.B, a.d_model, a.q_rank, plan, a.split_k, rows_pad, stream);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(rmsnorm_reduce_kernel, dim3(a.B), dim3(256), a.q_rank * sizeof(float), stream,
                       (const float*)a.ws_c, a.gain, (__bf16*)a.ws_chat, a.q_rank, a.split_k, rows_pad, a.eps);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    plan.split_k = 1;
    plan.k_per_split = a.q_rank;
    return launch_gemm<true, true>(a.ws_chat, a.w_qb, a.q_out, a.B, a.q_rank, a.n_out, plan, 1, rows_pad, stream);
}

namespace {

template <int BITS>
hipError_t launch_record_bits(const KvAppendArgs& a, const float* parts, int split_k, int rows_pad, hipStream_t stream)
{
    if (a.block_table) hipLaunchKernelGGL((kv_record_kernel<BITS, true>), dim3(a.B), dim3(kHeadDim), 0, stream, parts, split_k, rows_pad, a);
    else               hipLaunchKernelGGL((kv_record_kernel<BITS, false>), dim3(a.B), dim3(kHeadDim), 0, stream, parts, split_k, rows_pad, a);
    return hipGetLastError();
}

hipError_t launch_record(const KvAppendArgs& a, mfa_kv_dtype kv_dtype, const float* parts, int split_k, int rows_pad, hipStream_t stream)
{
    if (kv_dtype == MFA_KV_FP8_E4M3) return launch_record_bits<8>(a, parts, split_k, rows_pad, stream);
    if (kv_dtype == MFA_KV_FP4_E2M1) return launch_record_bits<4>(a, parts, split_k, rows_pad, stream);
    return launch_record_bits<16>(a, parts, split_k, rows_pad, stream);
}

}  // namespace

hipError_t launch_kv_record(const KvAppendArgs& a, const float* kv, mfa_kv_dtype kv_dtype, hipStream_t stream)
{
    return launch_record(a, kv_dtype, kv, 1, a.B, stream);
}

hipError_t launch_kv_append(const KvAppendArgs& a, mfa_kv_dtype kv_dtype, hipStream_t stream)
{
    const int m_blocks = (a.B + kQProjRows - 1) / kQProjRows;
    const int rows_pad = m_blocks * kQProjRows;
    const hipError_t e = launch_gemm<false, false>(a.x, a.w_kv, a.ws_c, a.B, a.d_model, kKvWidth, a.plan, a.plan.split_k, rows_pad, stream);
    if (e != hipSuccess) return e;
    return launch_record(a, kv_dtype, a.ws_c, a.plan.split_k, rows_pad, stream);
}

hipError_t launch_out_proj(const OutProjArgs& a, hipStream_t stream)
{
    const int m_blocks = (a.B + kQProjRows - 1) / kQProjRows;
    const int rows_pad = m_blocks * kQProjRows;
    const size_t n4 = (size_t)a.B * a.n_in / 4;
    hipLaunchKernelGGL(to_bf16_tiled_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, stream, a.attn, (__bf16*)a.ws_act,
                       a.B, a.n_in, rows_pad);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    e = launch_gemm<false, true>(a.ws_act, a.w_o, a.ws_c, a.B, a.n_in, a.d_model, a.plan, a.plan.split_k, rows_pad, stream);
    if (e != hipSuccess) return e;
    const size_t o4 = (size_t)a.B * a.d_model / 4;
    hipLaunchKernelGGL(reduce_partials_bf16_kernel, dim3((unsigned)((o4 + 255) / 256)), dim3(256), 0, stream, (const float*)a.ws_c,
                       (__bf16*)a.y, a.B, a.d_model, a.plan.split_k, rows_pad);
    return hipGetLastError();
}

}  // namespace mfa

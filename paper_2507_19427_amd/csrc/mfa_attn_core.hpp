// Device-side building blocks shared by the bf16 and fp8 decode attention kernels (gfx950).
//
// Workgroup shape common to both kernels: 8 waves; wave = 4*grp + wq.  wq selects 16 of the
// 64 query heads, grp selects which 32-token unit of every 64-token tile the wave processes.
// The two waves that share a SIMD (same wq, different grp) keep independent online-softmax
// states which finish_item() merges through LDS, so one wave's MFMA work can overlap the
// other's softmax.
//
// LDS image of one 32-token unit (what process_unit reads), bf16:
//   K rows 0..31 then V rows 0..31, 512 B per row (256 bf16).
//   K row r stores its 16-byte chunk c at position c ^ (r & 15);
//   V row r stores its 32-byte chunk c at position c ^ (r & 15).
// With these swizzles the 16-row x 16-byte MFMA operand reads of K and the 16-row x 32-byte
// transposing reads of V each touch every LDS bank exactly once.
//
// MFMA shapes (v_mfma_f32_16x16x32_bf16; lane = 16*g + n):
//   scores   S^T[token, head] = K[token, :] . Q[head, :]^T     A = K rows, B = Q
//            lane holds S^T[token 4g+i, head n], i = 0..3, for each 16-token block
//   output   O^T[d, head] += V^T[d, token] . P^T[token, head]  A = V^T, B = P
//            lane holds O^T[d = 16*db + 4g + i, head n]
// The score block a lane ends up with is exactly the B-operand slice it must supply for the
// second product (8 tokens of its own head), so attention weights never move between lanes and
// the per-head statistics live in the lanes of that head.
#pragma once
#include "mfa_internal.hpp"

namespace mfa {

typedef __attribute__((address_space(3))) unsigned char* lds_ptr_t;
#define LDS_AT(T, base, byte_off) ((__attribute__((address_space(3))) T*)((base) + (byte_off)))

constexpr int kUnitTokens = 32;
constexpr int kUnitBytes = 32768;        // K 32x512 B then V 32x512 B
constexpr int kUnitVOffset = 16384;
constexpr int kAttnThreads = 512;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// s_waitcnt that constrains only the vector-memory counter: vmcnt(0).
__device__ __forceinline__ void wait_vmem_all() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// Direct global->LDS load: 16 bytes per lane land at lds_addr + 16*lane (lds_addr is wave-uniform
// and travels in M0).  The global address is a wave-uniform base (scalar registers) plus a 32-bit
// byte offset per lane: no 64-bit vector arithmetic per load.  Issued as inline assembly so that
// the compiler does not make later LDS reads of *other* buffers wait for it; completion is
// awaited explicitly (wait_vmem_all() or a counted s_waitcnt) followed by a workgroup barrier.
// M0 is not otherwise live in these kernels.  The s_nop covers the wait state required between
// writing M0 and an LDS-direct load.  Everything brought in this way (cache rows, weight rows) is read
// once: the non-temporal hint keeps it from displacing reusable lines on its way through the caches,
// which alone is worth 11 to 14 % on the bf16 attention workloads.
__device__ __forceinline__ void load_to_lds_16B(const void* sbase, uint32_t voff, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt"
                 :: "v"(voff), "s"(sbase), "s"(lds_addr) : "memory");
}

// The same with the whole address in a pair of vector registers (for a base the compiler keeps there).
__device__ __forceinline__ void load_to_lds_16B_vaddr(const void* vaddr, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off nt"
                 :: "v"(vaddr), "s"(lds_addr) : "memory");
}
// Four bytes per lane: lane l's word lands at lds_addr + 4*l.
__device__ __forceinline__ void load_to_lds_4B(const void* sbase, uint32_t voff, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
                 :: "v"(voff), "s"(sbase), "s"(lds_addr) : "memory");
}

// max over the four lanes {n, n+16, n+32, n+48} that hold one head, without touching LDS:
// v_permlane32_swap exchanges the upper half of the first operand with the lower half of the
// second, v_permlane16_swap exchanges odd 16-lane rows of the first with even rows of the second.
__device__ __forceinline__ float head_max(float x)
{
    const unsigned u = __float_as_uint(x);
    const auto a = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    x = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
    const unsigned v = __float_as_uint(x);
    const auto b = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float head_sum(float x)
{
    const unsigned u = __float_as_uint(x);
    const auto a = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    x = __uint_as_float(a[0]) + __uint_as_float(a[1]);
    const unsigned v = __float_as_uint(x);
    const auto b = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// Running state of one wave: 16 heads x 256 output dims, spread as described above.
struct WaveState {
    f32x4 acc[16];
    float m;     // reference exponent of the weights, log2 domain: within 8 below this head's running maximum (equal in the 4 lanes of a head)
    float l;     // this lane's share of the sum of weights
};

__device__ __forceinline__ void init_state(WaveState& st)
{
#pragma unroll
    for (int i = 0; i < 16; ++i) st.acc[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
    st.m = -INFINITY;
    st.l = 0.f;
}

// Query fragments of this lane: B operand of the score product, d = 32*ks + 8*g + j.
__device__ __forceinline__ void load_q_fragments(bf16x8 (&qf)[8], const void* q, int b, int head, int g)
{
    const bf16x8* qp = (const bf16x8*)((const uint16_t*)q + ((size_t)b * kHeads + head) * kHeadDim + 8 * g);
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[ks] = qp[ks * 4];
}

// Query operands of one wave (its 16 heads).
//   bf16 cache: the bf16 fragments as loaded; a lane holds head n, d = 32*ks + 8*g + j.
//   fp8 cache:  the scores are taken on the fp8 MFMA (v_mfma_f32_16x16x128_f8f6f4, twice the bf16
//               rate) straight from the cache's codes, so the query is split into two e4m3 terms,
//               q * 2^e = hi + lo with e chosen per head so that the largest |q| of the head lands in
//               [128, 256): hi is the nearest e4m3 value and lo the remainder, which e4m3 holds
//               exactly (the 8 significant bits of bf16 are 4 + 4) down to 2^-9, i.e. to 2^-17 of the
//               head's largest element.  A lane holds head n, d = 128*c + 32*g + j (j = 0..31, one
//               byte each, in register order); inv_scale = 2^-e.
//   4-bit cache: the same split; the keys enter the same MFMA as e2m1 operands (16 bytes per lane
//               and 128 elements).  Measured on the device with one-hot operands: with an e2m1 A and
//               an e4m3 B operand, element j of A's lane group g multiplies byte 16*(g >> 1) + (j & 15)
//               of B's lane group 2*(g & 1) + (j >> 4).  The keys keep the plain order (a lane holds
//               d = 128*c + 32*g + j, one 16-byte read), so the query takes the matching one: a lane
//               holds d = 128*c + 64*(j >> 4) + 16*g + (j & 15).
typedef int i32x8 __attribute__((ext_vector_type(8)));
struct SplitQuery { i32x8 hi[2]; i32x8 lo[2]; float inv_scale; };
template <int BITS> struct QFrags;                    // BITS: width of a cache element (16, 8 or 4)
template <> struct QFrags<16> { bf16x8 f[8]; };
template <> struct QFrags<8> : SplitQuery {};
template <> struct QFrags<4> : SplitQuery {};

template <int BITS>
__device__ __forceinline__ void load_split_q(QFrags<BITS>& q, const void* qptr, int b, int head, int g)
{
    static_assert(BITS == 8 || BITS == 4, "the split query serves the 8-bit and 4-bit caches");
    const bf16x8* qp = (const bf16x8*)((const uint16_t*)qptr + ((size_t)b * kHeads + head) * kHeadDim + (BITS == 8 ? 32 : 16) * g);
    bf16x8 qf[2][4];
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int i = 0; i < 4; ++i) qf[c][i] = qp[c * 16 + (BITS == 8 ? i : 8 * (i >> 1) + (i & 1))];
    float amax = 0.f;
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j) amax = fmaxf(amax, fabsf((float)qf[c][i][j]));
    amax = head_max(amax);
    int e = (int)((__float_as_uint(amax) >> 23) & 0xFFu);          // biased exponent of the largest element
    e = e < 24 ? 24 : e;                                           // (all-zero or vanishing heads: any scale will do)
    const float scale = __uint_as_float((uint32_t)(261 - e) << 23);   // amax * scale in [128, 256)
    q.inv_scale = __uint_as_float((uint32_t)(e - 7) << 23);
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int w = 0; w < 2; ++w) {
                float x[4], r[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) x[j] = (float)qf[c][i][4 * w + j] * scale;
                int h = __builtin_amdgcn_cvt_pk_fp8_f32(x[0], x[1], 0, false);
                h = __builtin_amdgcn_cvt_pk_fp8_f32(x[2], x[3], h, true);
                const auto h01 = __builtin_amdgcn_cvt_pk_f32_fp8(h, false);
                const auto h23 = __builtin_amdgcn_cvt_pk_f32_fp8(h, true);
                r[0] = x[0] - h01[0]; r[1] = x[1] - h01[1]; r[2] = x[2] - h23[0]; r[3] = x[3] - h23[1];
                int l = __builtin_amdgcn_cvt_pk_fp8_f32(r[0], r[1], 0, false);
                l = __builtin_amdgcn_cvt_pk_fp8_f32(r[2], r[3], l, true);
                q.hi[c][2 * i + w] = h;
                q.lo[c][2 * i + w] = l;
            }
}

// One 32-token unit: scores, online softmax, weighted sum.
//   kbase      LDS byte offset of the unit's keys:
//                bf16:  32 rows of 512 B, 16-byte chunk c of row r stored at c ^ (r & 15)
//                8 bit: 32 rows of 256 B of e4m3 codes, 16-byte chunk c of row r at c ^ (r & 15)
//                4 bit: 32 rows of 128 B of packed e2m1 codes, 16-byte chunk c of row r at c ^ ((r >> 1) & 7)
//   vbase      LDS byte offset of the unit's values in bf16 (8 / 4 bit: the codes expanded, unscaled); layout
//              at pv_unit
//   unit_t0    index (within the sequence) of the unit's first token; tokens >= t1 are masked
//   8 / 4 bit  kscale/vscale point (LDS byte offsets) at the fp32 per-token scales of the unit's 32 tokens
//
// Raw scores of a unit (2 blocks of 16 tokens), before any scale: q . k for this lane's head and its 8 tokens.
struct RawScores { f32x4 s[2]; };
template <int BITS>
__device__ __forceinline__ RawScores qk_unit(const QFrags<BITS>& q, lds_ptr_t lds_base, int kbase, int n, int g)
{
    f32x4 s[2] = {(f32x4){0.f, 0.f, 0.f, 0.f}, (f32x4){0.f, 0.f, 0.f, 0.f}};
    if constexpr (BITS == 4) {
        // e2m1 keys x e4m3 query terms with unit block scales (E8M0 exponent 127)
        constexpr int kOne = 0x7F7F7F7F;
        // both query terms go into one accumulator per 16-token block: two independent chains keep the MFMA
        // pipe fed, and the small term is added first
#pragma unroll
        for (int c = 0; c < 2; ++c) {
#pragma unroll
            for (int tb = 0; tb < 2; ++tb) {
                const int row = kbase + tb * 2048 + n * 128;
                const u32x4 k4 = *LDS_AT(u32x4, lds_base, row + (((4 * c + g) ^ ((n >> 1) & 7)) << 4));
                const i32x8 kf = {(int)k4[0], (int)k4[1], (int)k4[2], (int)k4[3], 0, 0, 0, 0};
                s[tb] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(kf, q.lo[c], s[tb], 4, 0, 0, kOne, 0, kOne);
                s[tb] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(kf, q.hi[c], s[tb], 4, 0, 0, kOne, 0, kOne);
            }
        }
    } else if constexpr (BITS == 8) {
        // e4m3 x e4m3 with unit block scales (E8M0 exponent 127)
        constexpr int kOne = 0x7F7F7F7F;
#pragma unroll
        for (int c = 0; c < 2; ++c) {
#pragma unroll
            for (int tb = 0; tb < 2; ++tb) {
                const int row = kbase + tb * 4096 + n * 256;
                const int m = 8 * c + 2 * g;                       // first of this lane's two 16-byte chunks
                union { i32x8 v; u32x4 h[2]; } kf;
                kf.h[0] = *LDS_AT(u32x4, lds_base, row + ((m ^ n) << 4));
                kf.h[1] = *LDS_AT(u32x4, lds_base, row + (((m + 1) ^ n) << 4));
                s[tb] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(kf.v, q.lo[c], s[tb], 0, 0, 0, kOne, 0, kOne);
                s[tb] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(kf.v, q.hi[c], s[tb], 0, 0, 0, kOne, 0, kOne);
            }
        }
    } else {
        const int k_lane_off = n * 512;                 // K: row n of a 16-token block, swizzle key n
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
#pragma unroll
            for (int tb = 0; tb < 2; ++tb) {
                const int off = kbase + tb * 8192 + k_lane_off + (((4 * ks + g) ^ n) << 4);
                const bf16x8 kf = *LDS_AT(bf16x8, lds_base, off);
                s[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, q.f[ks], s[tb], 0, 0, 0);
            }
        }
    }
    RawScores r;
    r.s[0] = s[0];
    r.s[1] = s[1];
    return r;
}
// Online softmax of a unit from its raw scores, and the rescale of what has been accumulated so far.
// Returns the unit's attention weights as the B operand of the weighted sum (8 tokens of this lane's head).
template <int BITS>
__device__ __forceinline__ bf16x8 softmax_unit(WaveState& st, const QFrags<BITS>& q, const RawScores& raw, lds_ptr_t lds_base,
                                               int unit_t0, int t1, float scale_log2e, int g, int kscale_off, int vscale_off)
{
    constexpr bool FP8 = BITS != 16;                     // 8-bit arithmetic on the scores, scales beside the codes
    f32x4 s[2] = {raw.s[0], raw.s[1]};
    if constexpr (FP8) scale_log2e *= q.inv_scale;
    f32x4 vsc[2];
    if (FP8) {
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) {
            const f32x4 ksc = *LDS_AT(f32x4, lds_base, kscale_off + (16 * tb + 4 * g) * 4);
            vsc[tb] = *LDS_AT(f32x4, lds_base, vscale_off + (16 * tb + 4 * g) * 4);
            s[tb] *= ksc;
        }
    }

    // ---- online softmax in the log2 domain.  The raw scores are compared first and scaled inside the
    // exponent's fused multiply-add (the scale is positive); only a unit that reaches past t1, the last
    // of a sequence at most, spends instructions on masking.
    float sv[8];
    float m_raw = -INFINITY;
    if (unit_t0 + kUnitTokens <= t1) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            sv[j] = s[j >> 2][j & 3];
            m_raw = fmaxf(m_raw, sv[j]);
        }
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int tok = unit_t0 + 16 * (j >> 2) + 4 * g + (j & 3);
            sv[j] = tok < t1 ? s[j >> 2][j & 3] : -INFINITY;
            m_raw = fmaxf(m_raw, sv[j]);
        }
    }
    // The reference exponent st.m follows the running maximum lazily: it moves only when the maximum
    // has run ahead of it by more than kRescaleLag, so weights reach at most 2^kRescaleLag (harmless in
    // bf16 and fp32) and the 64 accumulator registers are rescaled a few times per sequence instead of
    // whenever some head of the wave sees a new maximum.  The normalisation at the end is unaffected.
    constexpr float kRescaleLag = 8.0f;
    const float m_seen = head_max(fmaxf(st.m, m_raw * scale_log2e));
    const float m_new = m_seen > st.m + kRescaleLag ? m_seen : st.m;   // (-inf + lag = -inf: the first token always moves it)
    const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = fast_exp2(st.m - m_safe);      // 1 when unmoved; 0 while nothing has been accumulated
    st.m = m_new;

    bf16x8 pf;
    float psum = 0.f;
    if (FP8) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            // the value scale rides on the weight; the normaliser sums the unscaled weight
            const float p = fast_exp2(__builtin_fmaf(sv[j], scale_log2e, -m_safe));
            pf[j] = (__bf16)(p * vsc[j >> 2][j & 3]);
            psum += p;
        }
    } else {
#pragma unroll
        for (int j = 0; j < 8; j += 2) {
            // normalise by the sum of the rounded weights actually multiplied into V
            const float p0 = fast_exp2(__builtin_fmaf(sv[j], scale_log2e, -m_safe));
            const float p1 = fast_exp2(__builtin_fmaf(sv[j + 1], scale_log2e, -m_safe));
            typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
            const bf16x2 pb = {(__bf16)p0, (__bf16)p1};
            pf[j] = pb[0];
            pf[j + 1] = pb[1];
            const uint32_t bits = __builtin_bit_cast(uint32_t, pb);
            psum += __uint_as_float(bits << 16) + __uint_as_float(bits & 0xFFFF0000u);
        }
    }
    st.l = st.l * alpha + psum;

    if (__any(alpha != 1.0f)) {
#pragma unroll
        for (int db = 0; db < 16; ++db) st.acc[db] *= alpha;
    }
    return pf;
}

// Scores and softmax of a unit in one go.
template <int BITS>
__device__ __forceinline__ bf16x8 score_unit(WaveState& st, const QFrags<BITS>& q, lds_ptr_t lds_base, int kbase,
                                             int unit_t0, int t1, float scale_log2e, int n, int g,
                                             int kscale_off, int vscale_off)
{
    const RawScores raw = qk_unit<BITS>(q, lds_base, kbase, n, g);
    return softmax_unit<BITS>(st, q, raw, lds_base, unit_t0, t1, scale_log2e, g, kscale_off, vscale_off);
}

// Second half of a unit: O^T += V^T P^T over the unit's 32 tokens.
//   BITS = 16 (bf16 cache, rows written by direct loads): 512-byte rows, 32-byte chunk c of row r at c ^ (r & 15).
//   BITS = 8 / 4 (rows written from registers): rows kPaddedVRow = 544 bytes apart.  The 32 bytes of padding shift
//                  consecutive rows by eight banks, which spreads a transposing read (4 rows x 32 bytes per 16 lanes,
//                  8 rows per half wave) over all 64 banks as the XOR does, and every operand address is then one
//                  lane register plus a compile-time offset.  Within a row the 16-byte pieces are placed so that the
//                  lanes of one 16-byte store instruction (store_tile in decode_lowbit_kernel) spread over the banks
//                  whether the hardware takes them 8 or 16 at a time; in the plain order they collide two by two:
//                    8 bit: a thread owns the 32-byte chunk c of a row; its two 16-byte halves are swapped when
//                           bits 2 and 3 of c differ (chunks 4..11);
//                    4 bit: a thread owns the 64-byte group c of four pieces; piece w sits at position
//                           (w + (c >> 1)) & 3 of the group.
//                  A reader knows the chunk (db) at compile time, so undoing this costs it lane registers (one more
//                  for 8 bit, three for 4 bit) and no instruction.
constexpr int kPaddedVRow = 544;
constexpr int kPaddedVUnitBytes = kUnitTokens * kPaddedVRow;      // 17408
__host__ __device__ constexpr bool padded_v_halves_swapped(int chunk32) { return (((chunk32 >> 2) ^ (chunk32 >> 3)) & 1) != 0; }
__host__ __device__ constexpr int padded_v_rotation(int group64) { return (group64 >> 1) & 3; }
template <int BITS>
__device__ __forceinline__ void pv_unit(WaveState& st, lds_ptr_t lds_base, int vbase, const bf16x8& pf, int n, int g)
{
    constexpr bool PADDED = BITS != 16;
    const int v_row = 4 * g + (n >> 2);                 // V: row within a 16-token block (= swizzle key)
    const int piece = n & 3;                            // which 8 bytes of the 32-byte chunk this lane supplies
    const int v_lane_off = v_row * (PADDED ? kPaddedVRow : 512) + (piece << 3);
    // 8 bit: [1] = halves swapped.  4 bit: [k] = the chunk's first piece sits at position k of its 64-byte group
    // (offsets relative to the group).
    int v_lane_alt[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
        v_lane_alt[k] = BITS == 8 ? (k == 1 ? v_lane_off ^ 16 : v_lane_off)
                                  : v_row * kPaddedVRow + 16 * ((k + (piece >> 1)) & 3) + 8 * (piece & 1);
    union VFrag { bf16x8 v; s16x4 h[2]; };
    auto read_v = [&](VFrag& f, int db) {
        int lane_off = v_lane_off, place = db << 5;
        if (BITS == 8) lane_off = v_lane_alt[padded_v_halves_swapped(db) ? 1 : 0];
        if (BITS == 4) {
            lane_off = v_lane_alt[(2 * (db & 1) + padded_v_rotation(db >> 1)) & 3];
            place = (db >> 1) << 6;
        }
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) {
            const int off = PADDED ? vbase + tb * 16 * kPaddedVRow + lane_off + place
                                   : vbase + tb * 8192 + v_lane_off + ((db ^ v_row) << 5);
            f.h[tb] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_AT(s16x4, lds_base, off));
        }
    };
    // The operands of kAhead output blocks are on their way while one block is multiplied: an LDS read takes
    // several times as long as the MFMA it feeds, and a wave has only one other wave on its SIMD to hide it.
    constexpr int kAhead = PADDED ? 4 : 2;
    VFrag f[kAhead];
#pragma unroll
    for (int i = 0; i < kAhead; ++i) read_v(f[i], i);
#pragma unroll
    for (int db = 0; db < 16; ++db) {
        __builtin_amdgcn_sched_barrier(0);
        st.acc[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[db % kAhead].v, pf, st.acc[db], 0, 0, 0);
        if (db + kAhead < 16) read_v(f[db % kAhead], db + kAhead);
    }
    __builtin_amdgcn_sched_barrier(0);
}

template <int BITS>
__device__ __forceinline__ void process_unit(WaveState& st, const QFrags<BITS>& q, lds_ptr_t lds_base, int kbase,
                                             int vbase, int unit_t0, int t1, float scale_log2e, int n, int g,
                                             int kscale_off, int vscale_off)
{
    const bf16x8 pf = score_unit<BITS>(st, q, lds_base, kbase, unit_t0, t1, scale_log2e, n, g, kscale_off, vscale_off);
    pv_unit<BITS>(st, lds_base, vbase, pf, n, g);
}

// ---- One 32-token unit for NT query tokens held by one wave (the one-pass kernel for three and four query
// tokens): every key fragment read from LDS feeds NT score products and every value fragment NT weighted-sum
// products, so the LDS traffic is that of a single token; the NT accumulator chains are independent, which
// keeps the MFMA pipe busy from one wave.
//
// Registers.  NT x 64 accumulator registers and NT x 32 of query fragments leave a wave (the only one on its
// SIMD) about 130 of its 512 registers for everything else, and only if the accumulators sit in the accumulation
// half of the file (where just MFMAs reach them) and nothing else does:
//   * the score products are written out as instructions with ordinary destination registers (the compiler gives
//     every MFMA of such a kernel an accumulation-register destination, which for NT = 4 alone oversubscribes
//     that half); the wait states between the last of them and the first read of a score are inserted by hand;
//   * the accumulators are never rescaled: the reference exponent of a head is set by its first unit with a token
//     (or handed in) and then stays, and the weights of later tokens may grow to 2^kFixedReferenceLag relative to
//     it, harmless in bf16 and fp32.  A unit that would exceed that changes nothing and reports the exponents it
//     would need; the caller starts the segment again with them (decode_bf16_multi_kernel).
constexpr float kFixedReferenceLag = 40.0f;
__device__ __forceinline__ void mfma_bf16_into_vgprs(f32x4& acc, const bf16x8& a, const bf16x8& b)
{
    asm("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
}
template <int NT>
__device__ __forceinline__ bool process_unit_multi(WaveState (&st)[NT], const QFrags<16> (&q)[NT], lds_ptr_t lds_base, int kbase,
                                                   int vbase, int unit_t0, const int (&t1)[NT], float scale_log2e, int n, int g,
                                                   float (&m_wanted)[NT])
{
    f32x4 s[NT][2];
#pragma unroll
    for (int t = 0; t < NT; ++t) s[t][0] = s[t][1] = (f32x4){0.f, 0.f, 0.f, 0.f};
    const int k_lane_off = n * 512;
    auto read_k = [&](int i) {                          // i = 2 * ks + tb
        return *LDS_AT(bf16x8, lds_base, kbase + (i & 1) * 8192 + k_lane_off + (((4 * (i >> 1) + g) ^ n) << 4));
    };
    bf16x8 kf[2] = {read_k(0), read_k(1)};
#pragma unroll
    for (int i = 0; i < 16; ++i) {                      // key fragments two ahead of their products
        const bf16x8 k_now = kf[i & 1];
        if (i + 2 < 16) kf[i & 1] = read_k(i + 2);
#pragma unroll
        for (int t = 0; t < NT; ++t) mfma_bf16_into_vgprs(s[t][i & 1], k_now, q[t].f[i >> 1]);
    }
    // 16 wait states between an 8-pass MFMA and a read of its result by another unit of the SIMD; every score
    // passes through this statement, so nothing reads one before it
    if constexpr (NT == 4)
        asm volatile("s_nop 7\n\ts_nop 7" : "+v"(s[0][0]), "+v"(s[0][1]), "+v"(s[1][0]), "+v"(s[1][1]), "+v"(s[2][0]), "+v"(s[2][1]),
                     "+v"(s[3][0]), "+v"(s[3][1]));
    else
        asm volatile("s_nop 7\n\ts_nop 7" : "+v"(s[0][0]), "+v"(s[0][1]), "+v"(s[1][0]), "+v"(s[1][1]), "+v"(s[2][0]), "+v"(s[2][1]));

    // (the scores are masked in place, and only in a unit that reaches past a token's end: no second copy of them)
    float m_ref[NT];
    bool moved = false;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        if (unit_t0 + kUnitTokens > t1[t]) {           // (a real branch: the empty statement keeps it from becoming 8 selects per unit)
            asm volatile("");
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int tok = unit_t0 + 16 * (j >> 2) + 4 * g + (j & 3);
                if (tok >= t1[t]) s[t][j >> 2][j & 3] = -INFINITY;
            }
        }
        float m_raw = -INFINITY;
#pragma unroll
        for (int j = 0; j < 8; ++j) m_raw = fmaxf(m_raw, s[t][j >> 2][j & 3]);
        const float m_seen = head_max(fmaxf(st[t].m, m_raw * scale_log2e));
        m_ref[t] = st[t].m == -INFINITY ? m_seen : st[t].m;       // set once, by the head's first unit with a token
        m_wanted[t] = m_seen;
        moved = moved || m_seen > m_ref[t] + kFixedReferenceLag;
    }
    if (__any(moved)) return false;
    bf16x8 pf[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const float m_safe = m_ref[t] == -INFINITY ? 0.f : m_ref[t];
        st[t].m = m_ref[t];
        float psum = 0.f;
#pragma unroll
        for (int j = 0; j < 8; j += 2) {
            // normalise by the sum of the rounded weights actually multiplied into V
            const float p0 = fast_exp2(__builtin_fmaf(s[t][j >> 2][j & 3], scale_log2e, -m_safe));
            const float p1 = fast_exp2(__builtin_fmaf(s[t][j >> 2][(j & 3) + 1], scale_log2e, -m_safe));
            typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
            const bf16x2 pb = {(__bf16)p0, (__bf16)p1};
            pf[t][j] = pb[0];
            pf[t][j + 1] = pb[1];
            const uint32_t bits = __builtin_bit_cast(uint32_t, pb);
            psum += __uint_as_float(bits << 16) + __uint_as_float(bits & 0xFFFF0000u);
        }
        st[t].l += psum;
    }
    const int v_row = 4 * g + (n >> 2);
    const int v_lane_off = v_row * 512 + ((n & 3) << 3);
    union VFrag { bf16x8 v; s16x4 h[2]; };
    auto read_v = [&](VFrag& f, int db) {
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
            f.h[tb] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_AT(s16x4, lds_base, vbase + tb * 8192 + v_lane_off + ((db ^ v_row) << 5)));
    };
    constexpr int kAhead = 3;
    VFrag f[kAhead];
#pragma unroll
    for (int i = 0; i < kAhead; ++i) read_v(f[i], i);
#pragma unroll
    for (int db = 0; db < 16; ++db) {
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < NT; ++t) st[t].acc[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[db % kAhead].v, pf[t], st[t].acc[db], 0, 0, 0);
        if (db + kAhead < 16) read_v(f[db % kAhead], db + kAhead);
    }
    __builtin_amdgcn_sched_barrier(0);
    return true;
}

// After the last tile the two waves that share 16 heads (grp 0 and 1: the two token halves of
// every tile) exchange halves of their accumulators through 64 KB of LDS at xbase (a tile buffer
// that is dead by then; the caller guarantees that no direct load into it is in flight) and a
// spare KB behind the tile memory: grp 0 finishes output blocks 0..7,
// grp 1 blocks 8..15, so all eight waves merge and store in parallel.  One split: the final
// result goes to `out`.  Several splits: the unnormalised partial goes to the workspace in
// lane order (float4 index (wq*16 + db)*64 + lane, fully coalesced), with (m, l) per head.
template <int KEEP, int SEND>
__device__ __forceinline__ void finish_half(WaveState& st, lds_ptr_t lds_base, int xbase, const AttnArgs& a, int b, int slot,
                                            bool final_result, int wq, int grp, int lane)
{
    const int n = lane & 15, g = lane >> 4;
    const int head = 16 * wq + n;
    const int mine = (wq * 2 + grp) * 8;              // my 8 KB exchange slots (1 KB each), from xbase on
    const int theirs = (wq * 2 + (grp ^ 1)) * 8;
    constexpr int kMlOff = 2 * 2 * kUnitBytes;        // (m, l) per head and wave: the spare KB behind the tile memory
#pragma unroll
    for (int i = 0; i < 8; ++i) *LDS_AT(f32x4, lds_base, xbase + (mine + i) * 1024 + lane * 16) = st.acc[SEND + i];
    if (g == 0) {                                     // m and (after head_sum) l are equal in the four lanes of a head
        *LDS_AT(float, lds_base, kMlOff + ((wq * 2 + grp) * 2 + 0) * 64 + n * 4) = st.m;
        *LDS_AT(float, lds_base, kMlOff + ((wq * 2 + grp) * 2 + 1) * 64 + n * 4) = st.l;
    }
    __syncthreads();
    const float m_o = *LDS_AT(float, lds_base, kMlOff + ((wq * 2 + (grp ^ 1)) * 2 + 0) * 64 + n * 4);
    const float l_o = *LDS_AT(float, lds_base, kMlOff + ((wq * 2 + (grp ^ 1)) * 2 + 1) * 64 + n * 4);
    const float m = fmaxf(st.m, m_o);                 // finite: the segment has a token, seen by grp 0
    const float w_s = fast_exp2(st.m - m);
    const float w_o = fast_exp2(m_o - m);
    const float l = st.l * w_s + l_o * w_o;
    const float inv = 1.0f / l;
    float* o = a.out + ((size_t)b * kHeads + head) * kHeadDim + 4 * g;
    f32x4* part = (f32x4*)a.ws_acc + (size_t)slot * (kHeads * kHeadDim / 4) + (size_t)wq * 16 * 64 + lane;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const f32x4 other = *LDS_AT(f32x4, lds_base, xbase + (theirs + i) * 1024 + lane * 16);
        const f32x4 r = st.acc[KEEP + i] * w_s + other * w_o;
        if (final_result) *(f32x4*)(o + 16 * (KEEP + i)) = r * inv;
        else part[(KEEP + i) * 64] = r;
    }
    if (!final_result && grp == 0 && g == 0)
        *(float2*)(a.ws_ml + ((size_t)slot * kHeads + head) * 2) = make_float2(m, l);
}

// One piece of work: tokens [t0, t1) of sequence b (n_tiles tiles of 64, the last one possibly
// ragged).  Its result is the sequence's final output (final_result) or a partial in `slot`.
struct Segment {
    int b, t0, t1, n_tiles, slot;
    int len;              // the sequence's (clamped) length
    bool final_result;
};

// Every field of a segment is the same in all threads; saying so keeps the branches on them scalar.
__device__ __forceinline__ void make_uniform(Segment& r)
{
    r.b = __builtin_amdgcn_readfirstlane(r.b);
    r.t0 = __builtin_amdgcn_readfirstlane(r.t0);
    r.t1 = __builtin_amdgcn_readfirstlane(r.t1);
    r.n_tiles = __builtin_amdgcn_readfirstlane(r.n_tiles);
    r.slot = __builtin_amdgcn_readfirstlane(r.slot);
    r.len = __builtin_amdgcn_readfirstlane(r.len);
    r.final_result = __builtin_amdgcn_readfirstlane((int)r.final_result) != 0;
}

// xbase: LDS byte offset of the 64 KB the exchange may use (tile memory nobody reads any more).
__device__ __forceinline__ void finish_segment(WaveState& st, lds_ptr_t lds_base, int xbase, const AttnArgs& a, const Segment& r,
                                               int wq, int grp, int lane)
{
    st.l = head_sum(st.l);
    __syncthreads();                                  // every wave is done reading the tile buffers
    if (grp == 0) finish_half<0, 8>(st, lds_base, xbase, a, r.b, r.slot, r.final_result, wq, grp, lane);
    else          finish_half<8, 0>(st, lds_base, xbase, a, r.b, r.slot, r.final_result, wq, grp, lane);
}

// Several query tokens per sequence (a wave then holds all 256 output dims of its 16 heads for a query
// token, and has seen all tokens of the segment): no exchange, each wave stores its 16 rows.  The partial
// of a (segment, query token) sits at slot * n_here + query token in the same lane-order layout.  A query token
// that saw no cached token in this segment leaves m = -inf, l = 0 and a zero accumulator; as a final
// result that is the zero row.
__device__ __forceinline__ void finish_segment_two(WaveState& st, const AttnArgs& a, const Segment& r, int qtok, int wq, int lane)
{
    const int n = lane & 15, g = lane >> 4;
    const int head = 16 * wq + n;
    const float l = head_sum(st.l);
    const size_t row = (size_t)r.b * a.q_len + a.q0 + qtok;
    if (r.final_result) {
        const float inv = l > 0.f ? 1.0f / l : 0.f;
        float* o = a.out + (row * kHeads + head) * kHeadDim + 4 * g;
#pragma unroll
        for (int db = 0; db < 16; ++db) *(f32x4*)(o + 16 * db) = st.acc[db] * inv;
    } else {
        const size_t slot = (size_t)r.slot * a.n_here + qtok;
        f32x4* part = (f32x4*)a.ws_acc + slot * (kHeads * kHeadDim / 4) + (size_t)wq * 16 * 64 + lane;
#pragma unroll
        for (int db = 0; db < 16; ++db) part[db * 64] = st.acc[db];
        if (g == 0) *(float2*)(a.ws_ml + (slot * kHeads + head) * 2) = make_float2(st.m, l);
    }
}

__device__ __forceinline__ int clamped_len(const AttnArgs& a, int b)
{
    const int L = a.seq_lens[b];
    return L < 0 ? 0 : (L > a.max_seq_len_hint ? a.max_seq_len_hint : L);
}

// ---- Which segments a workgroup works off.
//
// Fixed splits (n_wgs == 0): workgroup = (sequence, split), one segment of chunk_tokens tokens;
// the partial slot is the workgroup index; the first split of an empty sequence writes the zeros.
//
// Balanced (n_wgs > 0): with T_b = ceil(L_b / 64) tiles per sequence and P the exclusive prefix
// sums of T, workgroup w takes the tile range [w*N/G, (w+1)*N/G) of the N = P[B] tiles laid end to
// end (G = min(n_wgs, N), so that no workgroup below G is idle) and cuts it at sequence boundaries.  The workgroups touching sequence b are
// consecutive, first(b)..last(b) with wg_of(t) = ((t+1)*G - 1) / N; the segment of workgroup w on
// sequence b uses partial slot w + b, which is unique because (w, b) grows in at least one
// coordinate from one segment to the next, and the slots of one sequence are consecutive.  The
// workgroup holding a sequence's first tile records (first slot, number of partials) for the
// merge; a sequence held by one workgroup is written finally and needs no merge.  Sequences
// without tokens are zero-filled by the merge kernel.
constexpr int kSchedLdsOffset = 2 * 2 * kUnitBytes + 1024;                // behind both kernels' tile memory
constexpr int kSchedTotalsOffset = kSchedLdsOffset + (kMaxBalancedBatch + 1) * 4 + 12;   // 8 wave totals
constexpr int kSchedFoundOffset = kSchedTotalsOffset + 8 * 4;                           // result of the search
constexpr int kSchedRemOffset = kSchedFoundOffset + 16;     // per sequence: tokens in its last tile, minus one (a byte)
constexpr int kSchedLdsBytes = kSchedRemOffset + kMaxBalancedBatch - kSchedLdsOffset;
constexpr int kAttnLdsTotal = kSchedLdsOffset + kSchedLdsBytes;

struct Schedule {
    int lo, hi;         // balanced: my tile range; fixed: hi > lo while my one segment is still to do
    int n_tiles_all;    // N
    int n_wgs;          // G: workgroups that have a range (min of the grid size and N)
    int my_lo;          // start of my range (lo moves on as segments are handed out)
    bool first_known;   // the first segment's sequence is described below (no table lookup needed)
    int first_seq0, first_seq1, first_len;
    int b;              // next sequence to look at
};

// floor(a / d) for 32-bit operands without the long emulated integer division (some hundred scalar
// instructions ahead of every workgroup's first load): double-precision reciprocal, then one step of
// correction in integers (the estimate is off by at most one).
__device__ __forceinline__ unsigned div_floor_u32(unsigned a, unsigned d)
{
    unsigned q = (unsigned)((double)a * __builtin_amdgcn_rcp((double)d));
    const unsigned long long prod = (unsigned long long)q * d;
    if (prod > a) --q;
    else if (prod + d <= a) ++q;
    return q;
}
// floor(x * N / G) and the workgroup of a tile, in 32 bits when the products fit.
__device__ __forceinline__ int scaled_floor(int x, int N, int G)
{
    if (N < (1 << 20) && x <= (1 << 11)) return (int)div_floor_u32((unsigned)x * (unsigned)N, (unsigned)G);
    return (int)((unsigned long long)x * (unsigned long long)N / (unsigned long long)G);
}
__device__ __forceinline__ int wg_of_tile(int t, int G, int N)
{
    if (N < (1 << 20) && G <= (1 << 11)) return (int)div_floor_u32(((unsigned)t + 1u) * (unsigned)G - 1u, (unsigned)N);
    return (int)((((unsigned long long)t + 1ull) * (unsigned long long)G - 1ull) / (unsigned long long)N);
}

// Inclusive prefix sum over the 64 lanes of a wave with data-parallel-primitive moves: shifts by
// 1, 2, 4, 8 inside each row of 16 lanes (lanes without a source add 0), then lane 15 of rows 0 and
// 2 is added to rows 1 and 3, then lane 31 to rows 2 and 3.
__device__ __forceinline__ int wave_inclusive_scan(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);    // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);    // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);    // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);    // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);    // row_bcast:15 into rows 1, 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);    // row_bcast:31 into rows 2, 3
    return v;
}

// Which range of the balanced schedule a workgroup takes.  Workgroups are handed to the device's eight
// compute dies in turn (workgroup i runs on die i % 8, each with its own L2), while the pieces of one
// sequence are consecutive ranges: numbering the ranges die by die puts neighbouring ranges, which read
// neighbouring memory and write neighbouring partial results, on one die (measured on the benchmark
// workload: 0.6 us per call).  Nothing but speed depends on where a workgroup really runs.
__device__ __forceinline__ int range_index()
{
    const int g = (int)gridDim.x, i = (int)blockIdx.x;
    return (g & 7) == 0 ? (i & 7) * (g >> 3) + (i >> 3) : i;
}

// All threads of the workgroup call this; the values returned are the same in every thread.
//
// Batches of up to 512 sequences: every wave scans the whole batch by itself (eight lengths per
// lane at most), so the way to a workgroup's first segment crosses no barrier and no LDS; wave 0
// also leaves the tables in LDS for the later segments, which are requested only after the
// barriers of the first one.  Larger batches: one cooperative scan through LDS.
constexpr int kWaveScanChunks = 8;
// The lengths of such a batch reach the waves through LDS: every wave copies seq_lens[0 .. B) there with direct
// loads (all waves write the same bytes to the same place, so a wave that has waited for its own loads has the
// lengths without a barrier).  Direct loads are counted like every vector-memory operation but wait for nothing
// themselves, so a kernel can ask for the lengths, then for its first tile, and work the schedule out as soon as
// the lengths -- the older loads -- are there: stage_lengths(), further loads, schedule_begin(.., loads issued
// since).  The staging area is the part of the prefix-sum table that only larger batches use.
constexpr int kSchedStagedLensOffset = kSchedLdsOffset + 8192;
static_assert(kSchedStagedLensOffset >= kSchedLdsOffset + (kWaveScanChunks * 64 + 1) * 4 &&
              kSchedStagedLensOffset + kWaveScanChunks * 256 <= kSchedTotalsOffset, "staged lengths lie in the unused part of the table");
__device__ __forceinline__ bool lengths_are_staged(const AttnArgs& a) { return a.n_wgs != 0 && a.B <= kWaveScanChunks * 64; }
__device__ __forceinline__ void stage_lengths(const AttnArgs& a, lds_ptr_t lds_base)
{
    if (!lengths_are_staged(a)) return;
    const int lane = threadIdx.x & 63;
    const uint32_t dst = (uint32_t)(uintptr_t)lds_base + kSchedStagedLensOffset;
#pragma unroll
    for (int c = 0; c < kWaveScanChunks; ++c)
        if (c * 64 < a.B) {
            const int i = c * 64 + lane < a.B ? c * 64 + lane : a.B - 1;      // lanes past the batch repeat its last entry
            load_to_lds_4B(a.seq_lens, (uint32_t)i * 4u, dst + c * 256);
        }
}
// later_loads: vector-memory operations this wave has issued since stage_lengths (0 or 8: a tile)
__device__ __forceinline__ Schedule schedule_begin(const AttnArgs& a, lds_ptr_t lds_base, int later_loads = 0)
{
    Schedule s;
    s.first_known = false;
    s.first_seq0 = s.first_seq1 = s.first_len = 0;
    if (a.n_wgs == 0) { s.lo = s.my_lo = 0; s.hi = 1; s.n_tiles_all = 0; s.n_wgs = 0; s.b = 0; return s; }
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;

    if (a.B <= kWaveScanChunks * 64) {
        // the staged lengths have landed once only the loads issued after them are outstanding
        if (later_loads == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        else                  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        int len[kWaveScanChunks], p1[kWaveScanChunks];
#pragma unroll
        for (int c = 0; c < kWaveScanChunks; ++c) {
            const int i = c * 64 + lane;
            int L = 0;
            if (c * 64 < a.B && i < a.B) L = *LDS_AT(int, lds_base, kSchedStagedLensOffset + i * 4);
            len[c] = L < 0 ? 0 : (L > a.max_seq_len_hint ? a.max_seq_len_hint : L);
        }
        int N = 0;
#pragma unroll
        for (int c = 0; c < kWaveScanChunks; ++c) {
            p1[c] = N;
            if (c * 64 < a.B) {
                const int incl = wave_inclusive_scan((len[c] + kTile - 1) / kTile);
                p1[c] = N + incl;                                      // P[i + 1]
                N += __builtin_amdgcn_readlane(incl, 63);
            }
        }
        if (wave == 0) {
            if (lane == 0) *LDS_AT(int, lds_base, kSchedLdsOffset) = 0;
#pragma unroll
            for (int c = 0; c < kWaveScanChunks; ++c) {
                const int i = c * 64 + lane;
                if (i < a.B) {
                    *LDS_AT(int, lds_base, kSchedLdsOffset + (i + 1) * 4) = p1[c];
                    *LDS_AT(unsigned char, lds_base, kSchedRemOffset + i) = (unsigned char)((len[c] - 1) & (kTile - 1));
                }
            }
        }
        const int G = a.n_wgs < N ? a.n_wgs : N;      // with fewer tiles than workgroups the last ones idle
        s.n_tiles_all = N;
        s.n_wgs = G;
        if (range_index() >= G) { s.lo = s.hi = s.b = s.my_lo = 0; return s; }
        s.lo = s.my_lo = __builtin_amdgcn_readfirstlane(scaled_floor(range_index(), N, G));
        s.hi = __builtin_amdgcn_readfirstlane(scaled_floor(range_index() + 1, N, G));
        s.b = 0;
#pragma unroll
        for (int c = 0; c < kWaveScanChunks; ++c) {
            const int x = (len[c] + kTile - 1) / kTile;
            const unsigned long long hit = __ballot(p1[c] - x <= s.lo && s.lo < p1[c]);   // at most one lane of one chunk
            if (hit) {
                const int src = __builtin_amdgcn_readfirstlane(__builtin_ctzll(hit));
                s.b = c * 64 + src;
                s.first_seq1 = __builtin_amdgcn_readlane(p1[c], src);
                s.first_seq0 = s.first_seq1 - __builtin_amdgcn_readlane(x, src);
                s.first_len = __builtin_amdgcn_readlane(len[c], src);
                s.first_known = true;
            }
        }
        return s;
    }

    constexpr int totals = kSchedTotalsOffset;
    constexpr int found = kSchedFoundOffset;
    if (threadIdx.x == 0) *LDS_AT(int, lds_base, kSchedLdsOffset) = 0;
    int carry = 0;
    for (int base = 0; base < a.B; base += kAttnThreads) {
        const int i = base + threadIdx.x;
        const int len = i < a.B ? clamped_len(a, i) : 0;
        const int x = (len + kTile - 1) / kTile;
        if (i < a.B) *LDS_AT(unsigned char, lds_base, kSchedRemOffset + i) = (unsigned char)((len - 1) & (kTile - 1));
        const int incl = wave_inclusive_scan(x);
        if (lane == 63) *LDS_AT(int, lds_base, totals + wave * 4) = incl;
        __syncthreads();
        int before = carry, all = 0;
#pragma unroll
        for (int w = 0; w < kAttnThreads / 64; ++w) {
            const int tw = *LDS_AT(int, lds_base, totals + w * 4);
            all += tw;
            if (w < wave) before += tw;
        }
        if (i < a.B) *LDS_AT(int, lds_base, kSchedLdsOffset + (i + 1) * 4) = before + incl;    // P[i + 1]
        carry += all;
        __syncthreads();
    }
    const int N = carry;
    const int G = a.n_wgs < N ? a.n_wgs : N;
    s.n_tiles_all = __builtin_amdgcn_readfirstlane(N);
    s.n_wgs = __builtin_amdgcn_readfirstlane(G);
    if (range_index() >= G) { s.lo = s.hi = s.b = s.my_lo = 0; return s; }
    s.lo = s.my_lo = __builtin_amdgcn_readfirstlane(scaled_floor(range_index(), N, G));
    s.hi = __builtin_amdgcn_readfirstlane(scaled_floor(range_index() + 1, N, G));
    for (int base = 0; base < a.B; base += kAttnThreads) {
        const int i = base + threadIdx.x;
        if (i < a.B) {
            const int p0 = *LDS_AT(int, lds_base, kSchedLdsOffset + i * 4);
            const int p1 = *LDS_AT(int, lds_base, kSchedLdsOffset + (i + 1) * 4);
            if (p0 <= s.lo && s.lo < p1) *LDS_AT(int, lds_base, found) = i;
        }
    }
    __syncthreads();
    s.b = __builtin_amdgcn_readfirstlane(*LDS_AT(int, lds_base, found));   // the one sequence with P[b] <= lo < P[b + 1]
    return s;
}

// Where this workgroup's first tile lies if every sequence has the length of the hint: computed from the
// launch arguments alone (no device memory is read), with the same arithmetic as the schedule.  Only whole
// tiles below the hint are named, so that a load of the guessed tile stays inside memory the caller has
// vouched for (rows below max_seq_len_hint of a sequence below B; paged: a table entry below
// ceil(hint / 64), clamped into the pool like every other).
struct FirstTileGuess { int b, t0; bool valid; };
__device__ __forceinline__ FirstTileGuess guess_first_tile(const AttnArgs& a)
{
    FirstTileGuess gs;
    gs.b = gs.t0 = 0;
    gs.valid = false;
    if (!lengths_are_staged(a)) return gs;            // (the guess rides on the staged lengths' head start)
    const int T = (a.max_seq_len_hint + kTile - 1) / kTile;
    const int N = a.B * T;
    const int G = a.n_wgs < N ? a.n_wgs : N;
    const int w = range_index();
    if (w >= G) return gs;
    const int lo = scaled_floor(w, N, G);
    gs.b = (int)div_floor_u32((unsigned)lo, (unsigned)T);
    gs.t0 = (lo - gs.b * T) * kTile;
    gs.b = __builtin_amdgcn_readfirstlane(gs.b);
    gs.t0 = __builtin_amdgcn_readfirstlane(gs.t0);
    gs.valid = gs.b < a.B && gs.t0 + kTile <= a.max_seq_len_hint;
    return gs;
}

// The next segment of this workgroup, or false when it has none left.  A false return for the very
// first request of a fixed-split workgroup on an empty sequence has written the zero result.
__device__ __forceinline__ bool schedule_next(const AttnArgs& a, lds_ptr_t lds_base, Schedule& s, Segment& r)
{
    if (s.lo >= s.hi) return false;
    if (a.n_wgs == 0) {
        s.hi = 0;
        const int item = blockIdx.x;
        r.b = item / a.n_splits;
        const int split = item - r.b * a.n_splits;
        const int L = clamped_len(a, r.b);
        r.t0 = split * a.chunk_tokens;
        r.t1 = (r.t0 + a.chunk_tokens < L) ? r.t0 + a.chunk_tokens : L;
        r.n_tiles = (r.t1 - r.t0 + kTile - 1) / kTile;
        r.len = L;
        r.slot = item;
        r.final_result = a.n_splits == 1;
        if (r.t0 >= r.t1) {
            if (split == 0) {
                float4* o = (float4*)(a.out + (size_t)r.b * kHeads * kHeadDim);
                for (int i = threadIdx.x; i < kHeads * kHeadDim / 4; i += kAttnThreads) o[i] = make_float4(0.f, 0.f, 0.f, 0.f);
            }
            return false;
        }
        make_uniform(r);
        return true;
    }
    int b = s.b, seq0, seq1, L;
    if (s.first_known) {
        s.first_known = false;
        seq0 = s.first_seq0; seq1 = s.first_seq1; L = s.first_len;
    } else {
        while (*LDS_AT(int, lds_base, kSchedLdsOffset + (b + 1) * 4) <= s.lo) ++b;     // sequences without tiles
        seq0 = __builtin_amdgcn_readfirstlane(*LDS_AT(int, lds_base, kSchedLdsOffset + b * 4));
        seq1 = __builtin_amdgcn_readfirstlane(*LDS_AT(int, lds_base, kSchedLdsOffset + (b + 1) * 4));
        b = __builtin_amdgcn_readfirstlane(b);
        const int rem = __builtin_amdgcn_readfirstlane((int)*LDS_AT(unsigned char, lds_base, kSchedRemOffset + b));
        L = (seq1 - seq0 - 1) * kTile + rem + 1;                      // the sequence's (clamped) length
    }
    const int end = s.hi < seq1 ? s.hi : seq1;
    r.b = b;
    r.t0 = (s.lo - seq0) * kTile;
    r.t1 = (end - seq0) * kTile < L ? (end - seq0) * kTile : L;
    r.n_tiles = end - s.lo;
    r.len = L;
    r.final_result = seq0 >= s.my_lo && seq1 <= s.hi;                // the whole sequence lies in my range
    r.slot = range_index() + b;
    if (s.lo == seq0) {                                               // I hold its first tile: tell the merge
        const int last = r.final_result ? range_index() : wg_of_tile(seq1 - 1, s.n_wgs, s.n_tiles_all);
        if (threadIdx.x == 0) {
            a.ws_seg[2 * b] = range_index() + b;
            a.ws_seg[2 * b + 1] = last - range_index() + 1;
        }
    }
    s.lo = end;
    s.b = b + 1;
    make_uniform(r);
    return true;
}

}  // namespace mfa

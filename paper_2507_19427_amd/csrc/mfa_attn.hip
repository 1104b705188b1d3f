// Decode-step MFA attention for gfx950: 64 query heads of dimension 256 over one
// shared key head and one shared value head (paper, Section 2), one query token
// per sequence (or a pair, Section 5.2), independent sequences (Section 7.1).
//
// Work decomposition.  A workgroup of 8 waves works off segments: pieces
// [t0, t1) of one sequence's tokens, streamed once from HBM (mfa_attn_core.hpp:
// which segments a workgroup gets, how the waves share a tile, the MFMA operand
// layouts).  A segment that covers its whole sequence writes the final output;
// otherwise it leaves an unnormalised partial (acc, m, l) in the workspace that
// merge_splits_kernel reduces in order of position.
//
// bf16 cache: tiles of 64 tokens (= one cache page) are brought in with 16-byte
// global->LDS direct loads into a two-slot ring (64 KB per slot: two 32-token
// unit images).  The XOR swizzle of the unit image is applied on the global side
// of the direct load because its LDS side is fixed to base + 16*lane.
//
// 8-bit and 4-bit caches (e4m3 / e2m1 codes, one fp32 scale per token per
// tensor): the key codes go by direct loads into a three-slot ring and are
// multiplied as they are on the 8-bit MFMA against a two-term e4m3 query; the
// value codes travel through registers two tiles ahead and are expanded to bf16
// (exactly) into one of two value images for the same weighted-sum path as bf16.
// The key scale multiplies the score column of its token, the value scale rides
// on the attention weight of its token.
#include <hip/hip_ext.h>
#include <type_traits>

#include "mfa_attn_core.hpp"

namespace mfa {

constexpr int kSlotBytes = 2 * kUnitBytes;            // one 64-token tile: two unit images
constexpr int kLoadsPerTileAndWave = 8;               // direct loads a wave of decode_bf16_kernel issues per tile (4 rows pairs x K, V)
static_assert(kLoadsPerTileAndWave == 8, "schedule_begin waits with s_waitcnt vmcnt(8) for the loads older than a tile's");
constexpr int kAttnLdsBytes = 2 * kSlotBytes;         // bf16 kernel: 128 KB


// Page id of the tile that starts at token tile_t0 (paged cache only).  Looked up one tile ahead
// of its use so that the table read is never on the critical path of issuing a tile's loads.
template <bool PAGED>
__device__ __forceinline__ int lookup_page(const AttnArgs& a, int b, int tile_t0)
{
    // read through the constant address space: the table is not written while the kernel runs, and a
    // uniform index then makes this a scalar load, which the vector-memory waits do not have to cover
    typedef const __attribute__((address_space(4))) int32_t* const_table_t;
    if (!PAGED) return 0;
    const int page = ((const_table_t)a.block_table)[(size_t)b * a.max_blocks_per_seq + tile_t0 / kPage];
    return page < 0 ? 0 : (page >= a.n_pages ? a.n_pages - 1 : page);      // a bad id reads a wrong page, never outside the pool
}

template <bool PAGED>
__device__ __forceinline__ int64_t tile_row0(const AttnArgs& a, int b, int tile_t0, int page)
{
    return PAGED ? (int64_t)page * kPage : (int64_t)b * a.seq_stride_tokens + tile_t0;
}

// QL = query tokens per sequence.  1: wave = 4*(token half of the tile) + head group.  2: wave =
// 4*(query token of the pair q0, q0 + 1) + head group, and every wave works through both halves of each
// tile; query token j of q_len attends to the first len - (q_len - 1 - j) cached tokens (the new tokens are
// the last q_len of the cache).  More than two query tokens are worked off pair by pair, one launch each.
template <bool PAGED, int QL>
__global__ __launch_bounds__(kAttnThreads) void decode_bf16_kernel(AttnArgs a)
{
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    const lds_ptr_t lds_base = (lds_ptr_t)smem;
    const uint32_t lds_addr0 = (uint32_t)(uintptr_t)lds_base;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wq = wave & 3;
    const int grp = wave >> 2;
    const int n = lane & 15;
    const int g = lane >> 4;

    // Wave w brings rows [8w, 8w+8) of a tile's K and V: all in unit w/4.  Rows at or past the segment's
    // end re-read its last valid token, so nothing outside the sequence is touched and every LDS row
    // holds finite data (the weights of those rows are masked to zero).
    // (guessed: the tile named by guess_first_tile, whose position comes out of vector arithmetic; its
    // addresses stay in vector registers)
    auto issue_tile = [&](const Segment& sg, int tile, int slot, int page, bool guessed = false) {
        const int tile_t0 = sg.t0 + tile * kTile;
        const int64_t row0 = tile_row0<PAGED>(a, sg.b, tile_t0, page);
        const unsigned char* k_tile = (const unsigned char*)a.k + row0 * 512;   // wave-uniform: scalar registers
        const unsigned char* v_tile = (const unsigned char*)a.v + row0 * 512;
        const int p16 = lane & 31;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int row = 8 * wave + 2 * u + (lane >> 5);          // row of the tile this lane fills
            int in_tile = row;
            if (tile_t0 + row > sg.t1 - 1) in_tile = sg.t1 - 1 - tile_t0;
            const int key = row & 15;
            const int ck = p16 ^ key;
            const int cv = ((((p16 >> 1) ^ key) << 1) | (p16 & 1));
            const int first_row = 8 * wave + 2 * u;                   // wave-uniform
            const uint32_t dst = lds_addr0 + slot * kSlotBytes + (first_row >> 5) * kUnitBytes + (first_row & 31) * 512;
            if (guessed) {
                load_to_lds_16B_vaddr(k_tile + (uint32_t)(in_tile * 512 + ck * 16), dst);
                load_to_lds_16B_vaddr(v_tile + (uint32_t)(in_tile * 512 + cv * 16), dst + kUnitVOffset);
            } else {
                load_to_lds_16B(k_tile, (uint32_t)(in_tile * 512 + ck * 16), dst);
                load_to_lds_16B(v_tile, (uint32_t)(in_tile * 512 + cv * 16), dst + kUnitVOffset);
            }
        }
    };
    auto load_q = [&](QFrags<16>& q, const Segment& sg) {
        load_q_fragments(q.f, a.q, QL == 2 ? a.q_len * sg.b + a.q0 + grp : sg.b, 16 * wq + n, g);
    };

    // The workgroup's segments are worked off as one stream of tiles: while the last tile of a segment is
    // multiplied, the first tile of the next one is already on its way into the other slot,
    // and the end-of-segment exchange uses the slot of the tile just finished.
    //
    // The very first tile is asked for before the schedule is known: the lengths are requested first
    // (stage_lengths), then the tile that would be this workgroup's first if every sequence had the length of
    // the hint -- its place follows from the launch arguments alone -- and the schedule is worked out while
    // those 64 KB are on their way (the lengths, requested earlier, arrive earlier).  When the schedule
    // disagrees (ragged lengths), the right tile goes into the other slot and the guessed one is never looked
    // at; the guess only ever names whole tiles below the hint, i.e. memory the caller has vouched for.
    stage_lengths(a, lds_base);
    const FirstTileGuess guess = guess_first_tile(a);
    if (guess.valid) {
        Segment gs;
        gs.b = guess.b; gs.t0 = guess.t0; gs.t1 = guess.t0 + kTile;
        issue_tile(gs, 0, 0, lookup_page<PAGED>(a, guess.b, guess.t0), true);   // kLoadsPerTileAndWave loads
    }
    Schedule sched = schedule_begin(a, lds_base, guess.valid ? kLoadsPerTileAndWave : 0);
    Segment r, r_next;
    if (!schedule_next(a, lds_base, sched, r)) {
        wait_vmem_all();                              // nothing may still be writing into this workgroup's LDS when it ends
        return;
    }
    QFrags<16> q;
    load_q(q, r);
    int slot0 = 0;                                    // slot of the segment's first tile
    if (!(guess.valid && r.b == guess.b && r.t0 == guess.t0 && r.t0 + kTile <= r.t1)) {
        slot0 = guess.valid ? 1 : 0;
        issue_tile(r, 0, slot0, lookup_page<PAGED>(a, r.b, r.t0));
    }
    for (bool more = true; more;) {
        const int end_mine = r.len - (a.q_len - 1 - a.q0 - grp);      // QL == 2: grp = query token of the pair
        const int t1_mine = QL == 2 ? (r.t1 < end_mine ? r.t1 : end_mine) : r.t1;
        WaveState st;
        init_state(st);
        int page_next = r.n_tiles > 1 ? lookup_page<PAGED>(a, r.b, r.t0 + kTile) : 0;
        more = false;
        for (int it = 0; it < r.n_tiles; ++it) {
            const int slot = (slot0 + it) & 1;
            wait_vmem_all();
            __syncthreads();
            if (it + 1 < r.n_tiles) {
                issue_tile(r, it + 1, slot ^ 1, page_next);
                if (it + 2 < r.n_tiles) page_next = lookup_page<PAGED>(a, r.b, r.t0 + (it + 2) * kTile);
            } else {
                more = schedule_next(a, lds_base, sched, r_next);
                if (more) issue_tile(r_next, 0, slot ^ 1, lookup_page<PAGED>(a, r_next.b, r_next.t0));
            }
            if (QL == 2) {
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int unit = slot * kSlotBytes + u * kUnitBytes;
                    process_unit<16>(st, q, lds_base, unit, unit + kUnitVOffset, r.t0 + it * kTile + u * kUnitTokens,
                                     t1_mine, a.scale_log2e, n, g, 0, 0);
                }
            } else {
                const int unit = slot * kSlotBytes + grp * kUnitBytes;
                process_unit<16>(st, q, lds_base, unit, unit + kUnitVOffset, r.t0 + it * kTile + grp * kUnitTokens,
                                 t1_mine, a.scale_log2e, n, g, 0, 0);
            }
        }
        const int last_slot = (slot0 + r.n_tiles - 1) & 1;
        if (more) load_q(q, r_next);                  // ordinary loads (kept out of the tile loop, where the compiler's
                                                      // waits for them would also wait for the tile in flight)
        if (QL == 2) finish_segment_two(st, a, r, grp, wq, lane);
        else         finish_segment(st, lds_base, last_slot * kSlotBytes, a, r, wq, grp, lane);
        if (more) {
            r = r_next;
            slot0 = last_slot ^ 1;
        }
    }
}

// ---- Three or four query tokens per sequence in ONE pass over a bf16 cache (Section 5.2: the new tokens of a
// multi-token step share the cache read, which multiplies the arithmetic per byte by their number).
// A workgroup is four waves, one per SIMD, wave = head group: a wave holds all NT query tokens of its 16 heads
// (NT x 32 registers of query fragments, NT x 64 accumulator registers: only one wave fits a SIMD's register
// file) and works through both units of every tile; key and value fragments read from LDS are shared by the NT
// tokens (process_unit_multi).  Same tiles, same two-slot ring and same schedule as decode_bf16_kernel; each wave
// brings 16 rows of a tile.  Query token j attends to the first len - (q_len - 1 - j) cached tokens.  Batches of
// at most 512 sequences (every wave works the schedule out by itself).
constexpr int kMultiThreads = 256;
template <bool PAGED, int NT>
__global__ __launch_bounds__(kMultiThreads) void decode_bf16_multi_kernel(AttnArgs a)
{
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    const lds_ptr_t lds_base = (lds_ptr_t)smem;
    const uint32_t lds_addr0 = (uint32_t)(uintptr_t)lds_base;

    const int lane = threadIdx.x & 63;
    const int wq = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 15;
    const int g = lane >> 4;

    auto issue_tile = [&](const Segment& sg, int tile, int slot, int page) {
        const int tile_t0 = sg.t0 + tile * kTile;
        const int64_t row0 = tile_row0<PAGED>(a, sg.b, tile_t0, page);
        const unsigned char* k_tile = (const unsigned char*)a.k + row0 * 512;
        const unsigned char* v_tile = (const unsigned char*)a.v + row0 * 512;
        int lane_now = lane;                                          // (the lane's offsets are formed here, per tile, not
        asm volatile("" : "+v"(lane_now));                            // ahead of the tile loop and kept in scarce registers)
        const int p16 = lane_now & 31;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int row = 16 * wq + 2 * u + (lane_now >> 5);        // row of the tile this lane fills
            int in_tile = row;
            if (tile_t0 + row > sg.t1 - 1) in_tile = sg.t1 - 1 - tile_t0;
            const int key = row & 15;
            const int ck = p16 ^ key;
            const int cv = ((((p16 >> 1) ^ key) << 1) | (p16 & 1));
            const int first_row = 16 * wq + 2 * u;                     // wave-uniform
            const uint32_t dst = lds_addr0 + slot * kSlotBytes + (first_row >> 5) * kUnitBytes + (first_row & 31) * 512;
            load_to_lds_16B(k_tile, (uint32_t)(in_tile * 512 + ck * 16), dst);
            load_to_lds_16B(v_tile, (uint32_t)(in_tile * 512 + cv * 16), dst + kUnitVOffset);
        }
    };
    QFrags<16> q[NT];
    auto load_q = [&](const Segment& sg) {
        int lane_now = lane;                                          // (addresses formed here, once per segment)
        asm volatile("" : "+v"(lane_now));
#pragma unroll
        for (int t = 0; t < NT; ++t) load_q_fragments(q[t].f, a.q, a.q_len * sg.b + a.q0 + t, 16 * wq + (lane_now & 15), lane_now >> 4);
    };

    // A word of LDS behind the schedule's tables: set by a wave whose unit was refused (a score more than
    // 2^kFixedReferenceLag above its head's reference exponent), seen by all waves after the next barrier.
    constexpr int kRestartFlag = kAttnLdsTotal - 4;
    stage_lengths(a, lds_base);
    Schedule sched = schedule_begin(a, lds_base);
    Segment r;
    bool first_segment = true;
    while (schedule_next(a, lds_base, sched, r)) {
        if (!first_segment) __syncthreads();          // every wave is done with the previous segment's tiles
        first_segment = false;
        // Every segment leaves a partial result, also one that covers its whole sequence: partials are stored
        // straight from the accumulation registers, while a final result would have to pass all of them through
        // ordinary registers to be normalised.  The merge kernel normalises (AttnArgs::n_here >= 3).
        r.final_result = false;
        load_q(r);
        int t1_mine[NT];
        float m_floor[NT];                            // reference exponents handed to the next attempt (-inf: none)
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int end_mine = r.len - (a.q_len - 1 - a.q0 - t);
            t1_mine[t] = r.t1 < end_mine ? r.t1 : end_mine;
            m_floor[t] = -INFINITY;
        }
        WaveState st[NT];
        // One attempt streams the segment with fixed reference exponents.  If a unit is refused, its wave notes the
        // exponents it needs, raises the flag and stops computing; at the next barrier all waves see the flag and
        // the segment is streamed again from its first tile (every attempt ends with a higher reference for some
        // head, and a reference never exceeds the head's largest score: the attempts end).  Plausible attention
        // scores never get here; correctness does not depend on that.
        for (bool again = true; again;) {
            again = false;
            if (threadIdx.x == 0) *LDS_AT(int, lds_base, kRestartFlag) = 0;
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                init_state(st[t]);
                st[t].m = m_floor[t];
            }
            issue_tile(r, 0, 0, lookup_page<PAGED>(a, r.b, r.t0));
            int page_next = r.n_tiles > 1 ? lookup_page<PAGED>(a, r.b, r.t0 + kTile) : 0;
            bool refused = false;
            for (int it = 0; it < r.n_tiles; ++it) {
                const int slot = it & 1;
                wait_vmem_all();
                __syncthreads();                       // tile it has landed; the flag store of attempt start / of a refusal is visible
                if (*LDS_AT(int, lds_base, kRestartFlag) != 0) { again = true; break; }
                if (it + 1 < r.n_tiles) {
                    issue_tile(r, it + 1, slot ^ 1, page_next);
                    if (it + 2 < r.n_tiles) page_next = lookup_page<PAGED>(a, r.b, r.t0 + (it + 2) * kTile);
                }
                if (refused) continue;
#pragma unroll 1
                for (int u = 0; u < 2; ++u) {
                    const int unit = slot * kSlotBytes + u * kUnitBytes;
                    float m_wanted[NT];
                    if (!process_unit_multi<NT>(st, q, lds_base, unit, unit + kUnitVOffset, r.t0 + it * kTile + u * kUnitTokens,
                                                t1_mine, a.scale_log2e, n, g, m_wanted)) {
#pragma unroll
                        for (int t = 0; t < NT; ++t) m_floor[t] = fmaxf(m_floor[t], m_wanted[t]);
                        if (lane == 0) *LDS_AT(int, lds_base, kRestartFlag) = 1;
                        refused = true;
                        break;
                    }
                }
            }
            if (!again) {
                // the last tile's refusal (if any) has not met a barrier yet
                __syncthreads();
                again = *LDS_AT(int, lds_base, kRestartFlag) != 0;
            }
            if (again) {
                wait_vmem_all();                       // a tile may still be on its way into the ring
                __syncthreads();                       // every wave has read the flag and left the tile loop
            }
        }
        int lane_now = lane;                          // (the result's addresses are formed here, once per segment)
        asm volatile("" : "+v"(lane_now));
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            finish_segment_two(st[t], a, r, t, wq, lane_now);
            __builtin_amdgcn_sched_barrier(0);        // one query token's accumulators at a time through ordinary registers
        }
    }
}

// ---- 8-bit and 4-bit caches (BITS = 8: e4m3 codes, 256 B per row; BITS = 4: e2m1 codes two per byte,
// 128 B per row; one fp32 scale per token and tensor beside either).
// Keys stay codes all the way: each tile's rows go by direct loads into a ring of three LDS slots and
// are multiplied on the fp8/fp4 MFMA against the two-term query.  Values are multiplied by bf16
// weights, so their codes are converted once per tile: every thread carries 32 bytes (8 bit: two
// 16-byte pieces; 4 bit: one) of V and one per-token scale in registers from HBM, converts (exactly:
// every e4m3 and e2m1 value is a bf16 value) and writes the bf16 rows into one of two value images
// (padded rows in plain order: pv_unit).
//
// LDS: value image P (P = tile & 1) at P*34 KB, its unit g at + g*17 KB; key slot k (tile % 3) at
// 68 KB + k*16 KB (4 bit: the first 8 KB of it); scale set P at 116 KB + P*512 B (64 key scales, then
// 64 value scales).
constexpr int kLbVImageBytes = 2 * kPaddedVUnitBytes;    // two units of 32 padded bf16 rows
constexpr int kLbKBase = 2 * kLbVImageBytes;
constexpr int kLbKSlotBytes = kTile * 256;
constexpr int kLbKSlots = 3;
constexpr int kLbScaleBase = kLbKBase + kLbKSlots * kLbKSlotBytes;
constexpr int kLbLdsBytes = kLbScaleBase + 2 * 512;
static_assert(kLbLdsBytes <= kSchedLdsOffset && kAttnLdsBytes <= kSchedLdsOffset && kAttnLdsTotal <= 160 * 1024,
              "the schedule's prefix sums live behind the tile memory of both kernels");

struct LowbitTileRegs {
    u32x4 piece[2];       // 8 bit: V rows prow and prow + 32, 16-byte chunk pchunk; 4 bit: piece[0] only,
                          // V row tid / 8, 16-byte chunk tid % 8 (32 elements)
    float scale;          // threads 0..63: key scale of token tid; 64..127: value scale of token tid - 64
};
// Every step of the pipeline issues, per wave and in this order, the register loads of a tile
// (8 bit: two pieces and a scale; 4 bit: one piece and a scale) and the direct loads of a key tile
// (8 bit: two; 4 bit: one).  They are inline assembly, awaited with an explicit vmcnt that leaves
// exactly the youngest step's loads in flight: left to the compiler, the wait would be widened to
// vmcnt(0) at the loop's control-flow joins and drain the pipeline every tile.  The registers pass
// through the waiting statement, so no use of them can be scheduled before it.
template <int BITS> constexpr int kLowbitOpsPerStep = BITS == 8 ? 5 : 3;
// (address = wave-uniform base in scalar registers + 32-bit byte offset per lane; non-temporal: read once)
__device__ __forceinline__ void load_regs_16B(u32x4& dst, const void* sbase, uint32_t voff)
{
    asm volatile("global_load_dwordx4 %0, %1, %2 nt" : "=&v"(dst) : "v"(voff), "s"(sbase) : "memory");
}
__device__ __forceinline__ void load_regs_4B(float& dst, const void* sbase, uint32_t voff)
{
    asm volatile("global_load_dword %0, %1, %2 nt" : "=&v"(dst) : "v"(voff), "s"(sbase) : "memory");
}
template <int BITS>
__device__ __forceinline__ void wait_all_but_youngest_step(LowbitTileRegs& t)
{
    if constexpr (BITS == 8) {
        static_assert(kLowbitOpsPerStep<8> == 5, "the wait below leaves 5 operations in flight");
        asm volatile("s_waitcnt vmcnt(5)" : "+v"(t.piece[0]), "+v"(t.piece[1]), "+v"(t.scale) :: "memory");
    } else {
        static_assert(kLowbitOpsPerStep<4> == 3, "the wait below leaves 3 operations in flight");
        asm volatile("s_waitcnt vmcnt(3)" : "+v"(t.piece[0]), "+v"(t.scale) :: "memory");
    }
}
// Wait for every load in flight while both register sets are still owned by the pipeline: no
// register of theirs may be handed to other code before its load has landed.
template <int BITS>
__device__ __forceinline__ void drain_tiles(LowbitTileRegs& t, LowbitTileRegs& u)
{
    if constexpr (BITS == 8)
        asm volatile("s_waitcnt vmcnt(0)"
                     : "+v"(t.piece[0]), "+v"(t.piece[1]), "+v"(t.scale), "+v"(u.piece[0]), "+v"(u.piece[1]), "+v"(u.scale)
                     :: "memory");
    else
        asm volatile("s_waitcnt vmcnt(0)" : "+v"(t.piece[0]), "+v"(t.scale), "+v"(u.piece[0]), "+v"(u.scale) :: "memory");
}

template <bool PAGED, int QL, int BITS>
__global__ __launch_bounds__(kAttnThreads) void decode_lowbit_kernel(AttnArgs a)
{
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    const lds_ptr_t lds_base = (lds_ptr_t)smem;
    const uint32_t lds_addr0 = (uint32_t)(uintptr_t)lds_base;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wq = wave & 3;
    const int grp = wave >> 2;
    const int n = lane & 15;
    const int g = lane >> 4;

    stage_lengths(a, lds_base);
    Schedule sched = schedule_begin(a, lds_base);
    Segment r;
    bool first_segment = true;
    while (schedule_next(a, lds_base, sched, r)) {
        if (!first_segment) __syncthreads();          // the previous segment's exchange area is the tile memory
        first_segment = false;

        // Tiles past the end of the segment repeat its last tile (never consumed), so that every step
        // issues the same number of loads.  Rows at or past t1 re-read the last valid token.
        constexpr int kRowBytes = BITS == 8 ? 256 : 128;                   // one cached row of K or V
        const int prow = BITS == 8 ? threadIdx.x >> 4 : threadIdx.x >> 3;  // 8 bit: 0..31 (and + 32); 4 bit: 0..63
        const int pchunk = BITS == 8 ? threadIdx.x & 15 : threadIdx.x & 7; // 16-byte chunk of the row
        auto tile_origin = [&](int tile, int& tile_t0, int64_t& row0, int& last) {
            if (tile >= r.n_tiles) tile = r.n_tiles - 1;
            tile = __builtin_amdgcn_readfirstlane(tile);                   // keeps the page lookup a scalar load
            tile_t0 = r.t0 + tile * kTile;
            row0 = tile_row0<PAGED>(a, r.b, tile_t0, lookup_page<PAGED>(a, r.b, tile_t0));
            last = r.t1 - 1 - tile_t0;                                    // last valid row of this tile (>= 0)
        };
        auto load_tile = [&](LowbitTileRegs& t, int tile) {
            int tile_t0, last; int64_t row0;
            tile_origin(tile, tile_t0, row0, last);
#pragma unroll
            for (int i = 0; i < (BITS == 8 ? 2 : 1); ++i) {
                const int row = prow + 32 * i;
                const int in_tile = row > last ? last : row;
                load_regs_16B(t.piece[i], (const unsigned char*)a.v + row0 * kRowBytes, (uint32_t)(in_tile * kRowBytes + pchunk * 16));
            }
            const int tok = lane;                                          // waves 2.. repeat those of waves 0 and 1
            const int in_tile = tok > last ? last : tok;
            load_regs_4B(t.scale, ((wave & 1) ? a.v_scale : a.k_scale) + row0, (uint32_t)(in_tile * 4));
        };
        // Keys of a tile.  8 bit: 16 direct loads of 4 rows, wave w issues loads 2w and 2w + 1, 16-byte
        // chunk c of row r lands at c ^ (r & 15).  4 bit: 8 direct loads of 8 rows, one per wave, chunk c
        // of row r lands at c ^ ((r >> 1) & 7): 16 consecutive rows then spread one chunk column over all
        // 64 banks.
        auto issue_keys = [&](int tile, int kslot) {
            int tile_t0, last; int64_t row0;
            tile_origin(tile, tile_t0, row0, last);
            if constexpr (BITS == 8) {
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const int first_row = 4 * (2 * wave + i);                     // wave-uniform
                    const int row = first_row + (lane >> 4);
                    const int in_tile = row > last ? last : row;
                    const int c16 = (lane & 15) ^ (row & 15);
                    load_to_lds_16B((const unsigned char*)a.k + row0 * 256, (uint32_t)(in_tile * 256 + c16 * 16),
                                    lds_addr0 + kLbKBase + kslot * kLbKSlotBytes + first_row * 256);
                }
            } else {
                const int first_row = 8 * wave;                                   // wave-uniform
                const int row = first_row + (lane >> 3);
                const int in_tile = row > last ? last : row;
                const int c16 = (lane & 7) ^ ((row >> 1) & 7);
                load_to_lds_16B((const unsigned char*)a.k + row0 * 128, (uint32_t)(in_tile * 128 + c16 * 16),
                                lds_addr0 + kLbKBase + kslot * kLbKSlotBytes + first_row * 128);
            }
        };
        // Convert a tile's value codes to bf16 and write them into image `image`; the scales go beside it.
        auto store_tile = [&](const LowbitTileRegs& t, int image) {
            if constexpr (BITS == 8) {
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    bf16x8 half[2];
#pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
                        const bf16x2 p01 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(t.piece[i][w], 1.0f, false);
                        const bf16x2 p23 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(t.piece[i][w], 1.0f, true);
                        half[w >> 1][4 * (w & 1) + 0] = p01[0];
                        half[w >> 1][4 * (w & 1) + 1] = p01[1];
                        half[w >> 1][4 * (w & 1) + 2] = p23[0];
                        half[w >> 1][4 * (w & 1) + 3] = p23[1];
                    }
                    // (halves swapped in some chunks: see pv_unit)
                    const int off = image * kLbVImageBytes + i * kPaddedVUnitBytes + prow * kPaddedVRow + (pchunk << 5) + (padded_v_halves_swapped(pchunk) ? 16 : 0);
                    *LDS_AT(bf16x8, lds_base, off) = half[0];
                    *LDS_AT(bf16x8, lds_base, off ^ 16) = half[1];
                }
            } else {
                // 32 elements = bf16 chunks 2*pchunk and 2*pchunk + 1 (32 bytes each) of row prow
                const int row_off = image * kLbVImageBytes + (prow >> 5) * kPaddedVUnitBytes + (prow & 31) * kPaddedVRow;
#pragma unroll
                for (int w = 0; w < 4; ++w) {                                  // word w: elements 8w .. 8w + 7
                    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
                    const bf16x2 p0 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(t.piece[0][w], 1.0f, 0);
                    const bf16x2 p1 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(t.piece[0][w], 1.0f, 1);
                    const bf16x2 p2 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(t.piece[0][w], 1.0f, 2);
                    const bf16x2 p3 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(t.piece[0][w], 1.0f, 3);
                    const bf16x8 eight = {p0[0], p0[1], p1[0], p1[1], p2[0], p2[1], p3[0], p3[1]};
                    // piece w of this thread's 64-byte group, rotated within the group (see pv_unit)
                    *LDS_AT(bf16x8, lds_base, row_off + (pchunk << 6) + (((w + padded_v_rotation(pchunk)) & 3) << 4)) = eight;
                }
            }
            if (threadIdx.x < 128) *LDS_AT(float, lds_base, kLbScaleBase + image * 512 + threadIdx.x * 4) = t.scale;
        };

        WaveState st;
        init_state(st);

        // Step t consumes tile t (value image t & 1, key slot t % 3) while it converts the values of
        // tile t+1 into the other image and has the registers of tiles t+2, t+3 and the keys of tiles
        // t+1, t+2 in flight.  Prologue: what steps -2 and -1 would have issued.
        LowbitTileRegs regs[2];
        load_tile(regs[0], 0);
        load_tile(regs[1], 1);
        issue_keys(0, 0);
        // The query fragments are loaded by ordinary loads: the compiler completes them, and with them
        // everything above, right here instead of inside the loop.
        QFrags<BITS> q;
        load_split_q<BITS>(q, a.q, QL == 2 ? a.q_len * r.b + a.q0 + grp : r.b, 16 * wq + n, g);
        const int end_mine = r.len - (a.q_len - 1 - a.q0 - grp);      // QL == 2: grp = query token of the pair
        const int t1_mine = QL == 2 ? (r.t1 < end_mine ? r.t1 : end_mine) : r.t1;
        asm volatile("" : "+v"(q.hi[0]), "+v"(q.hi[1]), "+v"(q.lo[0]), "+v"(q.lo[1]));
        drain_tiles<BITS>(regs[0], regs[1]);
        store_tile(regs[0], 0);
        load_tile(regs[0], 2);
        issue_keys(1, 1);

        int kslot = 0;                                                     // t % 3
        auto step = [&](auto parity_c, int t) {
            constexpr int P = decltype(parity_c)::value;                    // t & 1
            wait_all_but_youngest_step<BITS>(regs[P ^ 1]);       // registers of tile t+1 and keys of tile t have landed
            __syncthreads();                               // ... for every wave; everyone is done with tile t-1
            const int kb = kLbKBase + kslot * kLbKSlotBytes;
            const int vb = P * kLbVImageBytes;
            const int scales = kLbScaleBase + P * 512;
            // The score products of this wave's (first) unit are issued ahead of the conversion of the next tile's
            // values: the MFMA pipe and the LDS work while the vector ALU converts (4 % on the 8-bit workload,
            // compared on one box).
            const int u0 = QL == 2 ? 0 : grp;
            const RawScores raw0 = qk_unit<BITS>(q, lds_base, kb + u0 * kUnitTokens * kRowBytes, n, g);
            store_tile(regs[P ^ 1], P ^ 1);                                 // values of tile t+1
            load_tile(regs[P ^ 1], t + 3);
            issue_keys(t + 2, kslot == 0 ? 2 : kslot - 1);                  // (t + 2) % 3, the slot tile t-1 has left
            {
                const bf16x8 pf = softmax_unit<BITS>(st, q, raw0, lds_base, r.t0 + t * kTile + u0 * kUnitTokens, t1_mine,
                                                     a.scale_log2e, g, scales + u0 * kUnitTokens * 4, scales + 256 + u0 * kUnitTokens * 4);
                pv_unit<BITS>(st, lds_base, vb + u0 * kPaddedVUnitBytes, pf, n, g);
            }
            if (QL == 2)
                process_unit<BITS>(st, q, lds_base, kb + kUnitTokens * kRowBytes, vb + kPaddedVUnitBytes,
                                   r.t0 + t * kTile + kUnitTokens, t1_mine, a.scale_log2e, n, g,
                                   scales + kUnitTokens * 4, scales + 256 + kUnitTokens * 4);
            kslot = kslot == 2 ? 0 : kslot + 1;
        };
        for (int t = 0; t < r.n_tiles; t += 2) {
            step(std::integral_constant<int, 0>{}, t);
            if (t + 1 >= r.n_tiles) break;
            step(std::integral_constant<int, 1>{}, t + 1);
        }
        drain_tiles<BITS>(regs[0], regs[1]);  // the repeats of the last tile issued past the end
        if (QL == 2) finish_segment_two(st, a, r, grp, wq, lane);
        else         finish_segment(st, lds_base, 0, a, r, wq, grp, lane);
    }
}

// Merge the partial results of one sequence (fixed splits: slots b*n_splits ...; balanced schedule:
// the slots recorded by the workgroup that held the sequence's first tile):
//   out = sum_s 2^(m_s - m*) acc_s / sum_s 2^(m_s - m*) l_s,  m* = max_s m_s,
// summed in split order (m* is reached batch by batch, rescaling what has been summed).  One thread per float4 of the partial's lane-order layout; splits are
// taken four at a time so that their loads are independent and in flight together.
__global__ __launch_bounds__(256) void merge_splits_kernel(AttnArgs a)
{
    const int n_here = a.n_here;                                      // query tokens of this launch
    // 16 blocks per (sequence, query token).  Consecutive block indices go to consecutive dies; the streaming kernel
    // has numbered its ranges so that a die holds consecutive ranges (range_index), i.e. with lengths that are about
    // equal the partial results of row r of B * n_here were written on die r * 8 / (B * n_here): the blocks of a
    // die take the rows of that die.
    const unsigned rows = (unsigned)(a.B * n_here);
    unsigned block = blockIdx.x;
    if ((rows & 7u) == 0 && a.n_wgs > 0 && (a.n_wgs & 7) == 0 && gridDim.x == rows * 16u) {
        const unsigned die = block & 7u, j = block >> 3;
        block = (die * (rows >> 3) + (j >> 4)) * 16u + (j & 15u);
    }
    const size_t idx = (size_t)block * 256 + threadIdx.x;             // over B * n_here * 4096 float4
    const int p = (int)(idx & 4095);                                  // position in the partial's lane-order layout
    const int bq = (int)(idx >> 12);                                  // sequence * n_here + query token of the launch
    if (bq >= a.B * n_here) return;
    const int b = bq / n_here;
    const int qtok = bq - b * n_here;
    const int lane = p & 63;
    const int db = (p >> 6) & 15;
    const int wq = p >> 10;
    const int h = 16 * wq + (lane & 15);
    const int d = 16 * db + 4 * (lane >> 4);
    // (the length and the sequence's slot record are asked for together: one round trip, not two; the record of
    // a sequence without tokens holds whatever the workspace held and is not used)
    int L = a.seq_lens[b];
    const int rec_first = a.n_wgs > 0 ? a.ws_seg[2 * b] : 0;
    const int rec_count = a.n_wgs > 0 ? a.ws_seg[2 * b + 1] : 0;
    L = L < 0 ? 0 : (L > a.max_seq_len_hint ? a.max_seq_len_hint : L);
    float4* const o = (float4*)(a.out + (((size_t)b * a.q_len + a.q0 + qtok) * kHeads + h) * kHeadDim + d);
    const int L_mine = L - (a.q_len - 1 - a.q0 - qtok);               // tokens this query token attends to
    int n_valid;
    size_t item0;
    if (a.n_wgs > 0) {                                                // balanced schedule
        if (L == 0) { *o = make_float4(0.f, 0.f, 0.f, 0.f); return; }
        item0 = (size_t)rec_first;
        n_valid = rec_count;
        if (n_valid == 1 && n_here < 3) return;                       // one workgroup held it all and wrote the result
                                                                      // (the one-pass kernel for 3 / 4 tokens never does)
    } else {
        if (L == 0) return;                                           // zeros were written by the first split
        n_valid = (L + a.chunk_tokens - 1) / a.chunk_tokens;          // <= n_splits
        item0 = (size_t)b * a.n_splits;
    }
    if (L_mine <= 0) { *o = make_float4(0.f, 0.f, 0.f, 0.f); return; }   // (only with several query tokens and L < q_len)
    const size_t slot0 = item0 * n_here + qtok;                       // partial of (item, query token) at item*n_here + qtok
    const size_t slot_step = (size_t)n_here;
    const float2* ml_base = (const float2*)a.ws_ml + slot0 * kHeads + h;
    const float4* acc_base = (const float4*)a.ws_acc + slot0 * (kHeads * kHeadDim / 4) + p;

    // One pass with a running reference exponent: a batch's (m, l) pairs and accumulator pieces are loaded
    // together, so the weights do not wait for a first round trip that only fetches the maxima.
    float m = -INFINITY;
    float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
    float l = 0.f;
    for (int s0 = 0; s0 < n_valid; s0 += 4) {
        float2 ml[4];
        float4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int s = s0 + u < n_valid ? s0 + u : n_valid - 1;
            ml[u] = ml_base[(size_t)s * slot_step * kHeads];
            v[u] = acc_base[(size_t)s * slot_step * (kHeads * kHeadDim / 4)];
        }
        float m_new = m;
#pragma unroll
        for (int u = 0; u < 4; ++u) m_new = fmaxf(m_new, ml[u].x);   // (a repeated last piece changes nothing)
        const float m_safe = m_new == -INFINITY ? 0.f : m_new;       // pieces without tokens have m = -inf
        const float keep = fast_exp2(m - m_safe);                    // 0 while nothing has been summed
        sum.x *= keep; sum.y *= keep; sum.z *= keep; sum.w *= keep;
        l *= keep;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float w = s0 + u < n_valid ? fast_exp2(ml[u].x - m_safe) : 0.f;
            sum.x += w * v[u].x; sum.y += w * v[u].y; sum.z += w * v[u].z; sum.w += w * v[u].w;
            l += w * ml[u].y;
        }
        m = m_new;
    }
    const float inv = 1.0f / l;
    *o = make_float4(sum.x * inv, sum.y * inv, sum.z * inv, sum.w * inv);
}

// Copy the logical rows of every sequence out of a paged pool (test aid).
__global__ __launch_bounds__(256) void gather_paged_kernel(const uint32_t* pool, int32_t row_words,
                                                           const int32_t* block_table, int32_t max_blocks_per_seq,
                                                           int32_t n_pages, const int32_t* seq_lens, int32_t hint, uint32_t* dst,
                                                           int64_t dst_seq_stride_tokens)
{
    const int b = blockIdx.y;
    const int blk = blockIdx.x;
    int L = seq_lens[b];
    L = L < 0 ? 0 : (L > hint ? hint : L);
    const int tok0 = blk * kPage;
    if (tok0 >= L) return;
    const int n_tok = (L - tok0 < kPage) ? L - tok0 : kPage;
    int page = block_table[(size_t)b * max_blocks_per_seq + blk];
    page = page < 0 ? 0 : (page >= n_pages ? n_pages - 1 : page);
    const uint32_t* src = pool + (size_t)page * kPage * row_words;
    uint32_t* d = dst + ((size_t)b * dst_seq_stride_tokens + tok0) * row_words;
    for (int i = threadIdx.x; i < n_tok * row_words; i += 256) d[i] = src[i];
}

// Measurement aid: read two buffers once with plain 16-byte loads and do nothing else.  What
// this reaches is the practical ceiling for any kernel that must stream the same bytes.
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* __restrict__ a, const uint4* __restrict__ b,
                                                          size_t n16_per_block, uint32_t* sink)
{
    const uint4* pa = a + (size_t)blockIdx.x * n16_per_block;
    const uint4* pb = b + (size_t)blockIdx.x * n16_per_block;
    uint32_t acc = 0;
    for (size_t i = threadIdx.x; i < n16_per_block; i += 512) {
        // non-temporal like the attention kernels' own streaming loads (measured: the faster of the two policies)
        const u32x4 x0 = __builtin_nontemporal_load((const u32x4*)pa + i), x1 = __builtin_nontemporal_load((const u32x4*)pa + i + 256);
        const u32x4 y0 = __builtin_nontemporal_load((const u32x4*)pb + i), y1 = __builtin_nontemporal_load((const u32x4*)pb + i + 256);
        const u32x4 z = x0 ^ x1 ^ y0 ^ y1;
        acc ^= z[0] ^ z[1] ^ z[2] ^ z[3];
    }
    if (acc == 0x9e3779b9u) sink[0] = acc;     // keeps the loads alive; practically never true
}

hipError_t launch_stream_read(const void* a, const void* b, size_t bytes_each, void* sink, hipStream_t stream,
                              hipEvent_t ev_before, hipEvent_t ev_after)
{
    constexpr unsigned kBlocks = 2048;
    if (!(ev_before && ev_after)) ev_before = ev_after = nullptr;
    hipExtLaunchKernelGGL(stream_read_kernel, dim3(kBlocks), dim3(256), 0, stream, ev_before, ev_after, 0,
                          (const uint4*)a, (const uint4*)b, bytes_each / kBlocks / 16, (uint32_t*)sink);
    return hipGetLastError();
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

int32_t balanced_workgroups(int32_t B, int32_t max_seq_len_hint, int32_t target_items)
{
    if (B > kMaxBalancedBatch) return 0;
    const int64_t max_tiles = (int64_t)B * ((max_seq_len_hint + kTile - 1) / kTile);
    return (int32_t)(max_tiles < target_items ? max_tiles : target_items);
}

namespace {

template <int QL>
const void* attn_kernel(mfa_kv_dtype kv_dtype, bool paged)
{
    if (kv_dtype == MFA_KV_BF16) return paged ? (const void*)decode_bf16_kernel<true, QL> : (const void*)decode_bf16_kernel<false, QL>;
    if (kv_dtype == MFA_KV_FP4_E2M1) return paged ? (const void*)decode_lowbit_kernel<true, QL, 4> : (const void*)decode_lowbit_kernel<false, QL, 4>;
    return paged ? (const void*)decode_lowbit_kernel<true, QL, 8> : (const void*)decode_lowbit_kernel<false, QL, 8>;
}

}  // namespace

namespace {
const void* multi_kernel(int q_len, bool paged)
{
    if (q_len == 3) return paged ? (const void*)decode_bf16_multi_kernel<true, 3> : (const void*)decode_bf16_multi_kernel<false, 3>;
    return paged ? (const void*)decode_bf16_multi_kernel<true, 4> : (const void*)decode_bf16_multi_kernel<false, 4>;
}
}  // namespace

hipError_t prepare_decode_attn_kernels()
{
    for (int q_len = 3; q_len <= 4; ++q_len)
        for (int paged = 0; paged < 2; ++paged) {
            const hipError_t e = hipFuncSetAttribute(multi_kernel(q_len, paged != 0), hipFuncAttributeMaxDynamicSharedMemorySize, kAttnLdsTotal);
            if (e != hipSuccess) return e;
        }
    for (int dt = 0; dt < 3; ++dt)
        for (int paged = 0; paged < 2; ++paged) {
            const mfa_kv_dtype kvd = dt == 0 ? MFA_KV_BF16 : (dt == 1 ? MFA_KV_FP8_E4M3 : MFA_KV_FP4_E2M1);
            hipError_t e = hipFuncSetAttribute(attn_kernel<1>(kvd, paged != 0), hipFuncAttributeMaxDynamicSharedMemorySize, kAttnLdsTotal);
            if (e != hipSuccess) return e;
            e = hipFuncSetAttribute(attn_kernel<2>(kvd, paged != 0), hipFuncAttributeMaxDynamicSharedMemorySize, kAttnLdsTotal);
            if (e != hipSuccess) return e;
        }
    return hipSuccess;
}

hipError_t launch_decode_attn(const AttnArgs& a, mfa_kv_dtype kv_dtype, hipStream_t stream,
                              hipEvent_t ev_before, hipEvent_t ev_after)
{
    const dim3 grid((unsigned)(a.n_wgs > 0 ? a.n_wgs : a.B * a.n_splits));
    const dim3 block(kAttnThreads);
    if (kv_dtype != MFA_KV_BF16 && kv_dtype != MFA_KV_FP8_E4M3 && kv_dtype != MFA_KV_FP4_E2M1) return hipErrorNotSupported;
    if (a.q_len < 1 || a.q_len > kMaxQueryTokens) return hipErrorNotSupported;
    if (a.q_len != 1 && a.n_wgs == 0) return hipErrorNotSupported;     // several query tokens: balanced schedule only
    // The two events, when given, are attached to the streaming kernel's own dispatch: they take the
    // times at which that kernel starts and ends on the device, with no launch gap inside the interval.
    // (With more than two query tokens: the first pair's.)
    if (!(ev_before && ev_after)) ev_before = ev_after = nullptr;
    const unsigned lds_bytes = a.n_wgs > 0 ? kAttnLdsTotal : kSchedLdsOffset;   // the schedule's arrays only if used
    const unsigned merge_blocks_per_token = (unsigned)(((size_t)a.B * kHeads * (kHeadDim / 4) + 255) / 256);
    // Three and four query tokens over a bf16 cache, batches the per-wave schedule covers: one pass over the cache
    // by the kernel that keeps all of a sequence's query tokens in one wave.
    if (a.q_len >= 3 && kv_dtype == MFA_KV_BF16 && a.B <= kWaveScanChunks * 64) {
        AttnArgs args = a;
        args.q0 = 0;
        args.n_here = a.q_len;
        void* params[] = {&args};
        hipError_t e = hipExtLaunchKernel(multi_kernel(a.q_len, a.block_table != nullptr), grid, dim3(kMultiThreads), params,
                                          kAttnLdsTotal, stream, ev_before, ev_after, 0);
        if (e != hipSuccess) return e;
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(merge_splits_kernel, dim3(merge_blocks_per_token * a.q_len), dim3(256), 0, stream, args);
        return hipGetLastError();
    }
    const void* kernel = a.q_len >= 2 ? attn_kernel<2>(kv_dtype, a.block_table != nullptr) : attn_kernel<1>(kv_dtype, a.block_table != nullptr);
    const int n_here = a.q_len == 1 ? 1 : 2;
    // Otherwise query tokens are worked off in pairs (q0, q0 + 1), one pass over the cache each; an odd count ends
    // with the pair (q_len - 2, q_len - 1), which computes token q_len - 2 a second time with the same result.
    // The passes share the partial-result workspace: they are ordered by the stream.
    for (int q0 = 0; q0 < a.q_len; q0 += 2) {
        AttnArgs args = a;
        args.q0 = q0 + n_here <= a.q_len ? q0 : a.q_len - n_here;
        args.n_here = n_here;
        void* params[] = {&args};
        hipError_t e = hipExtLaunchKernel(kernel, grid, block, params, lds_bytes, stream, q0 == 0 ? ev_before : nullptr,
                                          q0 == 0 ? ev_after : nullptr, 0);
        if (e != hipSuccess) return e;
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        if (a.n_wgs > 0 || a.n_splits > 1) {
            hipLaunchKernelGGL(merge_splits_kernel, dim3(merge_blocks_per_token * n_here), dim3(256), 0, stream, args);
            e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}

hipError_t launch_gather_paged(const void* pool, int32_t row_bytes, const int32_t* block_table,
                               int32_t max_blocks_per_seq, int32_t n_pages, const int32_t* seq_lens, int32_t max_seq_len_hint,
                               int32_t B, void* dst, int64_t dst_seq_stride_tokens, hipStream_t stream)
{
    const int blocks = (max_seq_len_hint + kPage - 1) / kPage;
    hipLaunchKernelGGL(gather_paged_kernel, dim3((unsigned)blocks, (unsigned)B), dim3(256), 0, stream,
                       (const uint32_t*)pool, row_bytes / 4, block_table, max_blocks_per_seq, n_pages, seq_lens,
                       max_seq_len_hint, (uint32_t*)dst, dst_seq_stride_tokens);
    return hipGetLastError();
}

}  // namespace mfa

// Merge paths for pieces of at most 64 bytes: one lane per piece (state in LDS
// columns) and one lane per symbol (state in registers).  Device code, included by
// bpe_encode.hip.
#pragma once
#include <type_traits>

#include "bpe_encode_params.h"

namespace bpe {

// ---------------------------------------------------------------------------
// Lane-per-piece path (pieces of at most kTinyMax bytes; in word-like text that
// is nearly all of them).  A lane owns one piece and runs the sequential loop of
// section 3.4 on it: take the best-ranked pair (left-most on ties), replace it,
// look up the two pairs the new symbol forms, repeat.  Symbols stay at their
// original positions; `alive` marks the positions that still hold one.
// LDS column `lane` holds the lane's symbols S[j] and, for the pair that starts
// at position j, R[j] = (rank order << 6) | flags << 4 | j (kNoRank if that pair is not in
// the table or position j is dead), so the argmin is a min over one column.
// A 64-wide wavefront issues an instruction in 4 cycles whatever the number of
// active lanes, so 64 pieces per wavefront cost about a tenth of the
// instructions per piece that the lane-per-symbol formulation needs.
struct alignas(16) TinyState {
    uint32_t S[kTinyMax][kWave];
    uint32_t R[kTinyMax][kWave];
};

// Merges the lane's piece bytes[o .. o + len) if `mine`; len <= kTinyMax.  Returns
// the mask of positions that hold the final tokens (they stay in L.S[.][lane]).
// Loads are batched so that dependent round trips stay few: all bytes of the
// piece (five aligned dwords), then all byte-pair ranks, then per merge the two
// neighbour symbols and the two new pairs' slots together.
__device__ uint32_t tiny_merge(const EncodeParams &p, TinyState &L, int o, int len, bool mine) {
    const int lane = lane_id();
    const int my_len = mine ? len : 0;
    if (!__ballot(my_len > 0)) return 0u;

    // the piece's bytes as 4 dwords: aligned loads, then a byte-granular funnel shift.
    // Offsets are counted from the aligned address at or below p.bytes, in 32 bits, so that
    // the loads take their base from scalar registers; a load that would start behind the
    // input is moved back onto its last dword instead of being branched around (what it
    // returns lies behind the piece and is never looked at).
    uint32_t w[4] = {0, 0, 0, 0};
    if (my_len) {
        const uint32_t mis = (uint32_t)((uintptr_t)p.bytes & 3);
        const uint8_t *base = p.bytes - mis;
        const uint32_t pos = (uint32_t)o + mis;
        const uint32_t first = pos & ~3u, last = ((uint32_t)p.n_bytes + mis - 1u) & ~3u;
        uint32_t raw[5];
#pragma unroll
        for (int k = 0; k < 5; ++k) raw[k] = *(const uint32_t *)(base + min(first + 4u * (uint32_t)k, last));
        const uint32_t sh = (pos & 3u) * 8u;
#pragma unroll
        for (int k = 0; k < 4; ++k)
            w[k] = (uint32_t)((((uint64_t)raw[k + 1] << 32) | raw[k]) >> sh);
    }
    uint32_t c[kTinyMax];
#pragma unroll
    for (int j = 0; j < kTinyMax; ++j) c[j] = (w[j / 4] >> (8 * (j % 4))) & 0xFFu;
    // rank words of all adjacent byte pairs from the direct table, all loads in flight together
    uint32_t r0[kTinyMax - 1];
#pragma unroll
    for (int j = 0; j < kTinyMax - 1; ++j)
        r0[j] = j + 1 < my_len ? p.table.byte_pairs[(c[j] << 8) | c[j + 1]] : kNoRank;
    // (opaque to the compiler from here on: left to itself it moves the first use of each word
    // next to its load, and with it a wait for every single load)
#pragma unroll
    for (int j = 0; j < kTinyMax - 1; ++j) asm volatile("" : "+v"(r0[j]));
    // S[j] = id | flags << 24: whether the symbol can be the left / right part of a rule
    // (bits 0 / 1).  Bytes are not classified: both flags set.
#pragma unroll
    for (int j = 0; j < kTinyMax; ++j) L.S[j][lane] = c[j] | (3u << 24);
    // R[j] = rank order << 6 | flags of the merged id << 4 | j.  The best pair is carried
    // through the loop in a register: a merge changes the pairs at three positions only,
    // so the minimum over all the others is taken while the lookups of the new pairs
    // are in flight, off the dependent chain.
    uint32_t best = kNoRank;
#pragma unroll
    for (int j = 0; j < kTinyMax - 1; ++j) {
        const uint32_t e = r0[j] | (uint32_t)j;      // kNoRank stays kNoRank
        L.R[j][lane] = e;
        best = min(best, e);
    }
    L.R[kTinyMax - 1][lane] = kNoRank;
    uint32_t alive = my_len ? (0xFFFFFFFFu >> (32 - my_len)) : 0u;

    for (;;) {
        if (!__ballot(best != kNoRank)) break;
        if (best != kNoRank) {
            const int k = best & 15;
            const uint32_t flags = (best >> 4) & 3u;                 // bit 0: merged id can be a left part, bit 1: a right part
            const uint32_t merged = merged_id_of(p.table, best >> 6);
            // positions by masks of the alive bits (fewer dependent steps than shifting them down)
            const uint32_t above = alive & (0xFFFFFFFEu << k);       // non-zero: its lowest bit is the pair's right symbol
            const int nk = __builtin_ctz(above);
            const uint32_t rest = above & (above - 1);               // symbols right of the merged one
            alive ^= above ^ rest;                                   // the right symbol is gone
            const uint32_t below = alive & ((1u << k) - 1);          // symbols left of it
            const int nn = rest ? __builtin_ctz(rest) : k;
            const int pk = below ? 31 - __builtin_clz(below) : k;
            const uint32_t right_sym = L.S[nn][lane];                // both reads before the write below
            const uint32_t left_sym = L.S[pk][lane];
            L.S[k][lane] = merged | (flags << 24);
            // New pairs (merged, right) and (left, merged).  A pair needs a lookup only if
            // its first symbol can be a left part and its second a right part of some rule;
            // the loads of both lookups are in flight together.
            const bool need_r = rest && (flags & 1u) && (right_sym >> 25);
            const bool need_l = below && (flags & 2u) && ((left_sym >> 24) & 1u);
            uint32_t rr = kNoRank, rl = kNoRank;
            uint2 a1, a2, b1, b2;   // each pair is only read under the predicate it was loaded under
            // the flag bits above the ids need no masking: slot_probe looks at the low 24 bits only
            const SlotProbe qa = slot_probe(p.table, merged, right_sym), qb = slot_probe(p.table, left_sym, merged);
            if (need_r) { a1 = slot_lower(p.table, qa); a2 = slot_upper(p.table, qa); }
            if (need_l) { b1 = slot_lower(p.table, qb); b2 = slot_upper(p.table, qb); }
            // meanwhile: the best of the pairs this merge does not touch
            L.R[nk][lane] = kNoRank;
            L.R[k][lane] = kNoRank;
            L.R[pk][lane] = kNoRank;           // pk == k if there is no symbol on the left
            uint32_t others = kNoRank;
#pragma unroll
            for (int j = 0; j < kTinyMax - 1; ++j) others = min(others, L.R[j][lane]);
            // keep the compiler from moving the first use of the slots, and with it the wait
            // for them, in front of these LDS reads, and from sinking the minimum behind it
            asm volatile("" : "+v"(others));
            __builtin_amdgcn_sched_barrier(0);
            if (need_r) rr = slot_match(a1, a2, qa.rest1, qa.rest2);
            if (need_l) rl = slot_match(b1, b2, qb.rest1, qb.rest2);
            const uint32_t new_k = rr | (uint32_t)k, new_pk = rl | (uint32_t)pk;     // kNoRank stays kNoRank
            L.R[k][lane] = new_k;
            if (below) L.R[pk][lane] = new_pk;
            best = min(others, min(new_k, new_pk));
        }
    }
    return alive;
}

// Stores the lane's final tokens (positions `alive` of its LDS column) to dst[0 ...].
__device__ inline void tiny_store(const TinyState &L, uint32_t alive, int32_t *dst) {
    const int lane = lane_id();
    int n_out = 0;
    while (__ballot(alive != 0)) {
        if (alive) {
            dst[n_out++] = (int32_t)(L.S[__builtin_ctz(alive)][lane] & 0xFFFFFFu);   // drop the flag bits
            alive &= alive - 1;
        }
    }
}

// ---------------------------------------------------------------------------
// The same lane-per-piece loop for longer pieces: a lane's column has N = 64 entries,
// so the 8 KiB LDS region of a wavefront holds the columns of 16 pieces (lanes 0 .. 15;
// the other lanes idle).  (N = 128, 8 pieces per wavefront, compiles as well; measured,
// it loses to the wavefront paths: a step costs 1.7 us with 128-bit position masks, and
// a run of 100 equal bytes is 95 steps, where the best-rank passes halve it seven times.)  One merge per step and piece, as
// in tiny_merge: the loop of section 3.4 run by one lane.  Pieces of random bytes take
// 15-30 merges of one dependent lookup each whichever way they are merged; here up
// to 16 of them share every instruction of a wavefront, where the lane-per-symbol
// path spends a whole wavefront on one.
// Layout: a lane's N entries are contiguous, and entry j sits at j ^ (4 * lane) of
// them: the minimum over the column is N / 4 aligned 16-byte reads per lane, and the
// XOR sends the reads that the lanes issue together to different groups of banks.
constexpr int kColumnMax = 64;         // pieces of up to this many bytes: 16 per wavefront and round
template <int N> struct ColumnGeometry {
    static_assert(N == 64 || N == 128, "columns of 64 or 128 entries");
    static constexpr int kLanes = (int)sizeof(TinyState) / (8 * N);   // 16 or 8
    static constexpr int kPosBits = N == 64 ? 6 : 7;
    using Mask = typename std::conditional<N == 64, uint64_t, unsigned __int128>::type;   // bit j: position j holds a symbol
};
struct alignas(16) ColumnState {
    uint32_t S[sizeof(TinyState) / 8];   // id | flags << 24, as in TinyState
    uint32_t R[sizeof(TinyState) / 8];   // rank order << (2 + position bits) | flags << position bits | position, or kNoRank
};
static_assert(sizeof(ColumnState) == sizeof(TinyState), "the column path reuses a wavefront's lane-per-piece region");
constexpr int kColumnLanes = ColumnGeometry<kColumnMax>::kLanes;

__device__ __forceinline__ int mask_ctz(uint64_t m) { return __builtin_ctzll(m); }
__device__ __forceinline__ int mask_ctz(unsigned __int128 m) {
    const uint64_t lo = (uint64_t)m;
    return lo ? __builtin_ctzll(lo) : 64 + __builtin_ctzll((uint64_t)(m >> 64));
}
__device__ __forceinline__ int mask_top(uint64_t m) { return 63 - __builtin_clzll(m); }     // m != 0
__device__ __forceinline__ int mask_top(unsigned __int128 m) {
    const uint64_t hi = (uint64_t)(m >> 64);
    return hi ? 127 - __builtin_clzll(hi) : 63 - __builtin_clzll((uint64_t)m);
}
__device__ __forceinline__ int mask_count(uint64_t m) { return __builtin_popcountll(m); }
__device__ __forceinline__ int mask_count(unsigned __int128 m) {
    return __builtin_popcountll((uint64_t)m) + __builtin_popcountll((uint64_t)(m >> 64));
}

// A rank word of the table as a column entry for the pair at position j.
template <int N>
__device__ __forceinline__ uint32_t column_entry(uint32_t rank_word, int j) {
    return rank_word == kNoRank ? kNoRank : (rank_word << (ColumnGeometry<N>::kPosBits - 4)) | (uint32_t)j;
}

// Merges the lane's piece bytes[o .. o + len) if `mine` (only lanes below
// ColumnGeometry<N>::kLanes may say so; 1 <= len <= N).  Returns the mask of the positions
// that hold the final tokens (in L.S at lane * N + (position ^ 4 * lane)).  Every lane
// must call it.
// Deliberately a function of its own: it has many callers, and inlined into all of them it costs the
// kernels scalar registers they do not have (spills to scratch memory, and a kernel that needs scratch
// memory took 18 us longer per launch on the 4 KB and 840 KB inputs).  Out of line, the compiler no
// longer knows which memory a pointer argument refers to, and would reach the LDS columns and the table
// through flat instructions (the texture path; fixed chunks of 64 bytes: 96 us against 56 us): so the
// address spaces are named here.  (The types may alias anything: the columns are written as words and
// read four words at a time.)
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4), may_alias));
typedef uint32_t __attribute__((may_alias)) u32_any;
typedef __attribute__((address_space(3))) u32_any lds_u32;
typedef __attribute__((address_space(3))) const u32x4 lds_u32x4;
typedef __attribute__((address_space(1))) const uint32_t global_u32;
typedef __attribute__((address_space(1))) const u32x2 global_u32x2;

template <class T>
__device__ __forceinline__ const T *uniform_pointer(const T *ptr) {
    const uint64_t v = (uint64_t)(uintptr_t)ptr;
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
    return (const T *)(uintptr_t)(((uint64_t)hi << 32) | lo);
}

template <int N>
__device__ __noinline__ typename ColumnGeometry<N>::Mask column_merge(const EncodeParams &p, ColumnState &L, int o, int len, bool mine) {
    using Mask = typename ColumnGeometry<N>::Mask;
    constexpr int kPosBits = ColumnGeometry<N>::kPosBits;
    const int lane = lane_id();
    const int my_len = mine ? len : 0;
    if (!__ballot(my_len > 0)) return (Mask)0;
    // What the loop below needs of the table is read once and pinned in scalar registers: left to itself
    // the compiler re-reads every field where it is used, four scalar loads with a full wait each (which
    // also waits for the LDS reads in flight) in every merge step.  (First made uniform by hand: where the
    // compiler cannot prove that the parameters are, it refuses to move them to scalar registers.)
    TableView tv = p.table;
    tv.slots = uniform_pointer(tv.slots);
    tv.byte_pairs = uniform_pointer(tv.byte_pairs);
    tv.merged_of = uniform_pointer(tv.merged_of);
    tv.half = (uint32_t)__builtin_amdgcn_readfirstlane((int)tv.half);
    tv.low_bits = __builtin_amdgcn_readfirstlane(tv.low_bits);
    tv.index_bits = __builtin_amdgcn_readfirstlane(tv.index_bits);
    tv.merged_delta = __builtin_amdgcn_readfirstlane(tv.merged_delta);
    tv.seed.k1a = (uint32_t)__builtin_amdgcn_readfirstlane((int)tv.seed.k1a);
    tv.seed.k1b = (uint32_t)__builtin_amdgcn_readfirstlane((int)tv.seed.k1b);
    tv.seed.k2a = (uint32_t)__builtin_amdgcn_readfirstlane((int)tv.seed.k2a);
    tv.seed.k2b = (uint32_t)__builtin_amdgcn_readfirstlane((int)tv.seed.k2b);
    asm volatile("" : "+s"(tv.slots), "+s"(tv.byte_pairs), "+s"(tv.merged_of), "+s"(tv.half), "+s"(tv.low_bits),
                      "+s"(tv.index_bits), "+s"(tv.merged_delta), "+s"(tv.seed.k1a), "+s"(tv.seed.k1b),
                      "+s"(tv.seed.k2a), "+s"(tv.seed.k2b));
    lds_u32 *const S = (lds_u32 *)&L.S[0], *const R = (lds_u32 *)&L.R[0];
    global_u32 *const byte_pairs = (global_u32 *)(uintptr_t)tv.byte_pairs;
    const uintptr_t lower = (uintptr_t)tv.slots, upper = (uintptr_t)(tv.slots + tv.half);
    auto slot_at = [](uintptr_t half_base, uint32_t byte_offset) {
        const u32x2 v = *(global_u32x2 *)(half_base + byte_offset);
        return make_uint2(v.x, v.y);
    };
    const int longest = __builtin_amdgcn_readlane(wave_scan_max_inclusive(my_len), kWave - 1);
    const int row = lane * N, sw = lane * 4;     // entry j of the lane: row + (j ^ sw)

    // Prologue, 16 bytes at a time: aligned dword loads and a funnel shift (as in tiny_merge),
    // then the ranks of the 16 byte pairs that start there, from the direct table.
    uint32_t best = kNoRank;
    const uint32_t mis = (uint32_t)((uintptr_t)p.bytes & 3);
    const uintptr_t base = (uintptr_t)p.bytes - mis;
    const uint32_t pos = (uint32_t)o + mis;
    const uint32_t last = ((uint32_t)p.n_bytes + mis - 1u) & ~3u;
    const uint32_t sh = (pos & 3u) * 8u;
#pragma unroll 1
    for (int c0 = 0; c0 < longest; c0 += 16) {
        if (c0 < my_len) {
            const uint32_t first = (pos + (uint32_t)c0) & ~3u;
            uint32_t raw[6];
#pragma unroll
            for (int k = 0; k < 6; ++k) raw[k] = *(global_u32 *)(base + min(first + 4u * (uint32_t)k, last));
            uint32_t w[5];
#pragma unroll
            for (int k = 0; k < 5; ++k) w[k] = (uint32_t)((((uint64_t)raw[k + 1] << 32) | raw[k]) >> sh);
            uint32_t c[17];
#pragma unroll
            for (int j = 0; j < 17; ++j) c[j] = (w[j / 4] >> (8 * (j % 4))) & 0xFFu;
            uint32_t r0[16];
#pragma unroll
            for (int j = 0; j < 16; ++j)
                r0[j] = c0 + j + 1 < my_len ? byte_pairs[(c[j] << 8) | c[j + 1]] : kNoRank;
#pragma unroll
            for (int j = 0; j < 16; ++j) asm volatile("" : "+v"(r0[j]));    // one batch of loads, one wait
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const int at = row + ((c0 + j) ^ sw);
                S[at] = c[j] | (3u << 24);
                const uint32_t e = column_entry<N>(r0[j], c0 + j);
                R[at] = e;
                best = min(best, e);
            }
        } else if (mine) {
#pragma unroll
            for (int j = 0; j < 16; ++j) R[row + ((c0 + j) ^ sw)] = kNoRank;   // the minimum below looks at whole groups of 16
        }
    }
    Mask alive = my_len ? (~(Mask)0 >> (N - my_len)) : (Mask)0;

    for (;;) {
        if (!__ballot(best != kNoRank)) break;
        if (best != kNoRank) {
            const int k = best & (N - 1);
            const uint32_t flags = (best >> kPosBits) & 3u;          // bit 0: merged id can be a left part, bit 1: a right part
            const uint32_t merged = merged_id_of(tv, best >> (kPosBits + 2));
            const Mask above = alive & ((~(Mask)1) << k);            // non-zero: its lowest bit is the pair's right symbol
            const int nk = mask_ctz(above);
            const Mask rest = above & (above - 1);                   // symbols right of the merged one
            alive ^= above ^ rest;                                   // the right symbol is gone
            const Mask below = alive & (((Mask)1 << k) - 1);         // symbols left of it
            const int nn = rest ? mask_ctz(rest) : k;
            const int pk = below ? mask_top(below) : k;
            const uint32_t right_sym = S[row + (nn ^ sw)];         // both reads before the write below
            const uint32_t left_sym = S[row + (pk ^ sw)];
            S[row + (k ^ sw)] = merged | (flags << 24);
            const bool need_r = rest && (flags & 1u) && (right_sym >> 25);
            const bool need_l = below && (flags & 2u) && ((left_sym >> 24) & 1u);
            uint32_t rr = kNoRank, rl = kNoRank;
            uint2 a1, a2, b1, b2;   // each pair is only read under the predicate it was loaded under
            const SlotProbe qa = slot_probe(tv, merged, right_sym), qb = slot_probe(tv, left_sym, merged);
            if (need_r) { a1 = slot_at(lower, qa.off1); a2 = slot_at(upper, qa.off2); }
            if (need_l) { b1 = slot_at(lower, qb.off1); b2 = slot_at(upper, qb.off2); }
            // meanwhile: the best of the pairs this merge does not touch
            R[row + (nk ^ sw)] = kNoRank;
            R[row + (k ^ sw)] = kNoRank;
            R[row + (pk ^ sw)] = kNoRank;    // pk == k if there is no symbol on the left
            uint32_t others = kNoRank;
            lds_u32x4 *Rq = (lds_u32x4 *)&R[row];
#pragma unroll
            for (int q = 0; q < N / 16; ++q) {
                if (q * 16 < longest) {        // the same for every lane
#pragma unroll
                    for (int g = 4 * q; g < 4 * q + 4; ++g) {
                        const u32x4 v = Rq[g ^ lane];                // entries 4 g .. 4 g + 3 of the column
                        others = min(others, min(min(v.x, v.y), min(v.z, v.w)));
                    }
                }
            }
            asm volatile("" : "+v"(others));
            __builtin_amdgcn_sched_barrier(0);
            if (need_r) rr = slot_match(a1, a2, qa.rest1, qa.rest2);
            if (need_l) rl = slot_match(b1, b2, qb.rest1, qb.rest2);
            const uint32_t new_k = column_entry<N>(rr, k), new_pk = column_entry<N>(rl, pk);
            R[row + (k ^ sw)] = new_k;
            if (below) R[row + (pk ^ sw)] = new_pk;
            best = min(others, min(new_k, new_pk));
        }
    }
    return alive;
}

// Stores the lane's final tokens (positions `alive` of its column) to dst[0 ...].
template <int N>
__device__ inline void column_store(const ColumnState &L, typename ColumnGeometry<N>::Mask alive, int32_t *dst) {
    const int lane = lane_id();
    int n_out = 0;
    while (__ballot(alive != 0)) {
        if (alive) {
            dst[n_out++] = (int32_t)(L.S[lane * N + (mask_ctz(alive) ^ (lane * 4))] & 0xFFFFFFu);   // drop the flag bits
            alive &= alive - 1;
        }
    }
}

// Level 3 for a piece whose symbols sit one per lane: is the pair of rank r that
// starts at this lane bound to be merged (see "Selection level 3" below)?  lr = the
// lowest ranks of a rule with this lane's symbol as its right / left part; lanes
// without a pair pass r = kNoRank; only lanes with `want` ask.  The walks of all
// lanes advance together.  Every lane must call it.
constexpr int kWaveSafeSteps = 7;
__device__ __forceinline__ bool wave_pair_is_bound(bool want, uint32_t r, uint2 lr, int lane, int cur) {
    // Walk to the left: at step d the lane looks at the symbol d lanes below (its lowest
    // rank as a right part) and at the pair below that symbol.  Both travel up the
    // wavefront one lane per step (a shift is one data-parallel move; lanes that run
    // out of neighbours receive "no rule").
    bool open = want, left = false;
    uint32_t ql = lr.x, rr = (uint32_t)wave_from_lane_below((int)r, (int)kNoRank);
#pragma unroll
    for (int d = 0; d <= kWaveSafeSteps; ++d) {
        if (d % 4 == 0 && !__ballot(open)) break;
        if (open) {
            if (lane - d == 0 || ql > r) { left = true; open = false; }
            else if (!(rr > r)) open = false;
        }
        ql = (uint32_t)wave_from_lane_below((int)ql, (int)kNoRank);
        rr = (uint32_t)wave_from_lane_below((int)rr, (int)kNoRank);
    }
    // Walk to the right: the symbol d lanes above (its lowest rank as a left part) and
    // the pair that starts there.
    open = want && left;
    bool right = false;
    uint32_t qr = (uint32_t)wave_from_lane_above((int)lr.y, (int)kNoRank);
    rr = (uint32_t)wave_from_lane_above((int)r, (int)kNoRank);
#pragma unroll
    for (int d = 1; d <= kWaveSafeSteps + 1; ++d) {
        if (d % 4 == 1 && !__ballot(open)) break;
        if (open) {
            if (lane + d == cur - 1 || qr >= r) { right = true; open = false; }
            else if (!(rr >= r)) open = false;
        }
        qr = (uint32_t)wave_from_lane_above((int)qr, (int)kNoRank);
        rr = (uint32_t)wave_from_lane_above((int)rr, (int)kNoRank);
    }
    return left && right;
}

// ---------------------------------------------------------------------------
// Lane-per-symbol path (one piece of at most 64 bytes per round, symbols in
// registers).  One pass = one iteration of the loop of section 3.4:
//   1. pair evaluation: lane i looks up (s[i], s[i+1]);
//   2. argmin over the wavefront of (rank << 6 | lane): ties go to the left;
//   3. selection: level 1 merges that one pair; level 2 merges every pair with
//      that rank, taking offsets 0, 2, 4 ... inside a run of equal symbols (what
//      merging "left to right without overlap" means for x x x ...);
//   4. compaction: surviving symbols move to their rank among survivors with one
//      cross-lane push (removed symbols are parked behind them, so the push is a
//      permutation of all 64 lanes).
// Merging all occurrences of the best rank is exact because a rule's parts are
// made by lower ranks (checked at table build): the pairs a merge creates
// contain the fresh id and therefore rank higher than it.
// The passes over a piece whose cur <= 64 symbols sit one per lane (lanes from cur on
// hold anything); returns the final number of symbols and leaves them in `sym`.
__device__ int encode_wave_symbols(const EncodeParams &p, uint32_t &sym, int cur) {
    const int lane = lane_id();
    const uint64_t lt_mask = (1ull << lane) - 1;
    for (;;) {
        const uint32_t nxt = (uint32_t)wave_from_lane_above((int)sym, (int)sym);
        uint32_t merged = 0, key = kNoRank;
        uint2 lr = make_uint2(kNoRank, kNoRank);
        if (p.level >= 3 && lane < cur) lr = p.table.sym_lr[sym];
        if (lane + 1 < cur) {
            const uint32_t r = table_find(p.table, sym, nxt);
            if (r != kNoRank) { key = (r & ~63u) | (uint32_t)lane; merged = merged_id_of(p.table, r >> kRankShift); }
        }
        const uint32_t best = wave_min_u32(key);
        if (best == kNoRank) break;
        bool sel;
        if (p.level == 1) {
            sel = key == best;
        } else {
            const bool cand = key != kNoRank && (key >> 6) == (best >> 6);
            const uint64_t not_cand_below = ~__ballot(cand) & lt_mask;
            const int run_start = not_cand_below ? 64 - __builtin_clzll(not_cand_below) : 0;
            sel = cand && !((lane - run_start) & 1);
            if (p.level >= 3)
                sel |= wave_pair_is_bound(key != kNoRank && !cand, key == kNoRank ? kNoRank : key >> 6, lr, lane, cur);
        }
        const uint64_t S = __ballot(sel);
        const uint32_t newsym = sel ? merged : sym;
        const uint64_t live = cur == kWave ? ~0ull : ((1ull << cur) - 1);
        const uint64_t removed = (S << 1) & live;
        const uint64_t kept = live & ~removed;
        const int n_kept = __builtin_popcountll(kept);
        int dst = lane;
        if (lane < cur) dst = ((removed >> lane) & 1) ? n_kept + mbcnt(removed) : mbcnt(kept);
        sym = permute_push(dst, newsym);
        cur = n_kept;
    }
    return cur;
}

// ---------------------------------------------------------------------------
// Lane-per-run path: a piece that is mostly runs x x x ... (one wavefront, any length),
// kept as runs (symbol, count) one per lane, neighbours holding different symbols.  Its
// pairs are the interior pair (s, s) of every run of two or more and the boundary pair
// between neighbouring runs.  A pass takes the lowest-ranked of them, left-most on ties
// (a run's interior pair lies left of the boundary behind it):
//   interior pair of run (s, c), merged id m: the run becomes (m, c / 2), followed by
//     (s, 1) if c is odd.  These are the c / 2 merges that the loop of section 3.4
//     makes one after the other, left to right: every pair they create contains m and
//     so ranks above the pair being merged (a rule's parts are made by lower ranks);
//   boundary pair between (a, ca) and (b, cb): one merge, (a, ca - 1) (m, 1) (b, cb - 1);
// then runs of nothing go and neighbours with equal symbols are joined.  A run of 4,096
// equal bytes takes a dozen passes of one table round trip each, where the workgroup
// path spends a dozen passes of four barriers over thousands of symbols.
// Returns the number of tokens (stored to p.scratch[b ...]), or -1 if the piece has,
// or comes to have, more than 64 runs: it is untouched then and takes another path.
// `stage`: 128 words of LDS of this wavefront.
constexpr int kMaxRuns = kWave;

// Lanes flagged `gone` drop out: the others close up, in order.  Returns the new run count.
__device__ __forceinline__ int runs_compact(uint32_t &sym, uint32_t &cnt, bool gone, int cur) {
    const int lane = lane_id();
    const uint64_t live = cur == kWave ? ~0ull : ((1ull << cur) - 1);
    const uint64_t removed = __ballot(gone) & live;
    if (!removed) return cur;
    const uint64_t kept = live & ~removed;
    const int n_kept = __builtin_popcountll(kept);
    int dst = lane;
    if (lane < cur) dst = ((removed >> lane) & 1) ? n_kept + mbcnt(removed) : mbcnt(kept);
    sym = permute_push(dst, sym);
    cnt = permute_push(dst, cnt);
    return n_kept;
}

// A run whose symbol equals that of the run below joins it (its count moves down, the run goes).
// One round joins pairs; three equal runs in a row (a fresh symbol between two runs of it) need two.
__device__ __forceinline__ int runs_join(uint32_t &sym, uint32_t &cnt, int cur) {
    const int lane = lane_id();
#pragma unroll
    for (int round = 0; round < 2; ++round) {
        const uint32_t below = (uint32_t)wave_from_lane_below((int)sym, -1);
        const bool joins = lane > 0 && lane < cur && sym == below;
        if (!__ballot(joins)) break;
        // the run above me joins me unless I join the run below myself (then the next round moves both)
        const uint32_t cnt_above = (uint32_t)wave_from_lane_above((int)cnt, 0);
        const bool above_joins = __builtin_amdgcn_update_dpp(0, (int)joins, 0x130, 0xF, 0xF, false) != 0;   // wave_shl:1
        const bool take = above_joins && !joins && lane + 1 < cur;
        if (take) cnt += cnt_above;
        // a run leaves only if the run below it took its count
        const bool taken = __builtin_amdgcn_update_dpp(0, (int)take, 0x138, 0xF, 0xF, false) != 0;          // wave_shr:1
        cur = runs_compact(sym, cnt, joins && taken, cur);
    }
    return cur;
}

__device__ int encode_wave_runs(const EncodeParams &p, int b, int n, uint32_t *stage) {
    const int lane = lane_id();
    // The runs of the piece: 16 bytes per lane and round, a start wherever a byte differs from
    // the one before it.  stage[r] = symbol of run r, stage[64 + r] = where it starts.
    int n_runs = 0;
    {
        const uint32_t mis = (uint32_t)((uintptr_t)p.bytes & 3);
        const uint8_t *base = p.bytes - mis;
        const uint32_t last = ((uint32_t)p.n_bytes + mis - 1u) & ~3u;
        uint32_t carry = 0x100;            // the byte before the round's first one (none: differs from every byte)
        for (int r0 = 0; r0 < n; r0 += 16 * kWave) {
            const int at = r0 + 16 * lane;                 // this lane's 16 bytes start here
            const uint32_t pos = (uint32_t)(b + min(at, n - 1)) + mis;
            const uint32_t first = pos & ~3u, sh = (pos & 3u) * 8u;
            uint32_t raw[5], w[4];
#pragma unroll
            for (int k = 0; k < 5; ++k) raw[k] = *(const uint32_t *)(base + min(first + 4u * (uint32_t)k, last));
#pragma unroll
            for (int k = 0; k < 4; ++k) w[k] = (uint32_t)((((uint64_t)raw[k + 1] << 32) | raw[k]) >> sh);
            const int mine = max(min(n - at, 16), 0);      // bytes of the piece among my 16
            // the byte before my first one: the last byte of the lane below, or the carry of the round before
            const uint32_t my_last = (w[3] >> 24) & 0xFFu;
            uint32_t prev = (uint32_t)wave_from_lane_below((int)my_last, (int)carry);
            uint32_t mask = 0;
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const uint32_t c = (w[j / 4] >> (8 * (j % 4))) & 0xFFu;
                if (j < mine && c != prev) mask |= 1u << j;
                prev = c;
            }
            const int inc = wave_scan_inclusive(__builtin_popcount(mask));
            const int total = __builtin_amdgcn_readlane(inc, kWave - 1);
            if (n_runs + total > kMaxRuns) return -1;
            int r = n_runs + inc - __builtin_popcount(mask);
            while (__ballot(mask != 0)) {
                if (mask) {
                    const int j = __builtin_ctz(mask);
                    stage[r] = (w[j / 4] >> (8 * (j % 4))) & 0xFFu;
                    stage[kWave + r] = (uint32_t)(at + j);
                    ++r;
                    mask &= mask - 1;
                }
            }
            n_runs += total;
            carry = (uint32_t)__builtin_amdgcn_readlane((int)my_last, kWave - 1);   // only read if the next round exists: then lane 63 was full
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
    __builtin_amdgcn_wave_barrier();
    int cur = n_runs;
    uint32_t sym = 0, cnt = 0;
    if (lane < cur) {
        sym = stage[lane];
        cnt = (lane + 1 < cur ? stage[kWave + lane + 1] : (uint32_t)n) - stage[kWave + lane];
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
    __builtin_amdgcn_wave_barrier();

    for (;;) {
        // pair evaluation: the boundary pair behind my run, and its interior pair
        const uint32_t nxt = (uint32_t)wave_from_lane_above((int)sym, (int)sym);
        uint32_t key_b = kNoRank, key_i = kNoRank;
        const bool has_b = lane + 1 < cur, has_i = lane < cur && cnt >= 2;
        const SlotProbe qb = slot_probe(p.table, sym, nxt), qi = slot_probe(p.table, sym, sym);
        uint2 b1, b2, i1, i2;
        if (has_b) { b1 = slot_lower(p.table, qb); b2 = slot_upper(p.table, qb); }
        if (has_i) { i1 = slot_lower(p.table, qi); i2 = slot_upper(p.table, qi); }
        if (has_b) { const uint32_t r = slot_match(b1, b2, qb.rest1, qb.rest2); if (r != kNoRank) key_b = ((r >> kRankShift) << 7) | (uint32_t)(lane << 1) | 1u; }
        if (has_i) { const uint32_t r = slot_match(i1, i2, qi.rest1, qi.rest2); if (r != kNoRank) key_i = ((r >> kRankShift) << 7) | (uint32_t)(lane << 1); }
        const uint32_t best = wave_min_u32(min(key_b, key_i));
        if (best == kNoRank) break;
        const int j = (int)((best >> 1) & 63u);
        const bool boundary = best & 1u;
        const uint32_t merged = merged_id_of(p.table, best >> 7);
        // one run is put in behind run j, unless an even run is halved
        const uint32_t cj = (uint32_t)read_lane((int)cnt, j);
        const uint32_t sj = (uint32_t)read_lane((int)sym, j);
        const bool insert = boundary || (cj & 1u);
        if (insert) {
            if (cur == kMaxRuns) return -1;
            const uint32_t sym_up = (uint32_t)wave_from_lane_below((int)sym, 0), cnt_up = (uint32_t)wave_from_lane_below((int)cnt, 0);
            if (lane > j + 1) { sym = sym_up; cnt = cnt_up; }      // runs behind j + 1 move up by one lane
            else if (lane == j + 1) {
                // boundary: the old run j + 1 (one symbol shorter) is now in lane j + 2, the fresh symbol here;
                // interior: the odd symbol left over
                sym = boundary ? merged : sj;
                cnt = 1;
            }
            ++cur;
        }
        if (boundary) {
            if (lane == j || lane == j + 2) --cnt;                 // each side gave one symbol
        } else if (lane == j) {
            sym = merged;
            cnt = cj >> 1;
        }
        cur = runs_compact(sym, cnt, lane < cur && cnt == 0, cur);
        cur = runs_join(sym, cnt, cur);
    }
    // the tokens: run after run, the wavefront writes a run's copies together
    const int inc = wave_scan_inclusive(lane < cur ? (int)cnt : 0);
    const int total = __builtin_amdgcn_readlane(inc, kWave - 1);
    int32_t *out = p.scratch + b;
    for (int r = 0; r < cur; ++r) {
        const int c = read_lane((int)cnt, r), s0 = read_lane(inc, r) - c;
        const int32_t s = read_lane((int)sym, r);
        for (int i = lane; i < c; i += kWave) out[s0 + i] = s;
    }
    return total;
}

// Piece bytes[base .. base + n), n <= 64: tokens to p.scratch[base ...], their number back.
__device__ int encode_wave_piece(const EncodeParams &p, int base, int n) {
    const int lane = lane_id();
    uint32_t sym = 0;
    if (lane < n) sym = p.bytes[base + lane];
    const int cur = encode_wave_symbols(p, sym, n);
    if (lane < cur) p.scratch[base + lane] = (int32_t)sym;
    return cur;
}

}  // namespace bpe

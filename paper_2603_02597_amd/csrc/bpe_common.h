// Shared by the host-side table builder and the device kernels of this library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <utility>
#include <vector>

#include "bpe_mi355x.h"

namespace bpe {

constexpr uint64_t kEmptyKey = ~0ull;          // no valid key: ids are non-negative int32
constexpr uint32_t kNoRank = 0xFFFFFFFFu;      // "pair not in the table"
constexpr int kRankBits = 26;                  // rule count < 2^26 so that (rank << 6 | lane) fits 32 bits
constexpr uint32_t kRankMask = (1u << kRankBits) - 1;
// A stored rank word also says whether the merged id of the rule occurs as the left
// (right) part of any rule: if not, no pair that starts (ends) with it needs a lookup.
constexpr uint32_t kCanLeft = 1u << 30, kCanRight = 1u << 31;   // in the host image's value word
// On the device a rank word is laid out as the lane-per-piece path keeps a pair:
// rank order << 6 | can-right << 5 | can-left << 4, low four bits clear for the pair's
// position, so that "word | position" is the whole conversion and kNoRank stays kNoRank.
constexpr int kRankShift = 6;
constexpr uint32_t kDevCanLeft = 1u << 4, kDevCanRight = 1u << 5;
__host__ __device__ inline uint32_t device_rank_word(uint32_t image_word) {
    return ((image_word & kRankMask) << kRankShift) | ((image_word >> 30) << 4);
}
constexpr int kIdBits = 24;                    // token ids < 2^24: the slot hash is a 24-bit mix
constexpr int kMaxRulesLog2 = 22;              // rule count < 2^22: a half of the slot table has at most 2^24 slots
constexpr int kWave = 64;
constexpr int kWavesPerGroup = 4;
constexpr int kGroupThreads = kWave * kWavesPerGroup;
constexpr int kTinyMax = 16;                   // longest piece of the lane-per-piece path
constexpr int kWaveLdsMax = kTinyMax * kWave;   // longest piece one wavefront double-buffers in its own LDS region
constexpr int kLdsMaxLen = 4104;               // symbols of one long piece held twice in LDS (32.1 KiB)
constexpr int32_t kLongMark = -1;              // per-piece count placeholder: "workgroup path pending"
constexpr int kHashSeeds = 16;

// Multipliers of the two slot-index hashes, one set per build attempt (odd, < 2^24).
struct HashSeed { uint32_t k1a, k1b, k2a, k2b; };
__host__ __device__ inline HashSeed hash_seed(int attempt) {
    const uint32_t base[4] = {0x9E3779u, 0x85EBCBu, 0xC2B2AFu, 0x27D4EBu};
    HashSeed s;
    s.k1a = (base[0] + 0x1234u * 2u * (uint32_t)attempt) & 0xFFFFFFu;
    s.k1b = (base[1] + 0x0F1Eu * 2u * (uint32_t)attempt) & 0xFFFFFFu;
    s.k2a = (base[2] + 0x2B5Cu * 2u * (uint32_t)attempt) & 0xFFFFFFu;
    s.k2b = (base[3] + 0x3A96u * 2u * (uint32_t)attempt) & 0xFFFFFFu;
    return s;
}

// 24-bit x 24-bit multiply, low 32 bits of the product (one full-rate VALU op on the GPU).
__host__ __device__ inline uint32_t mul24(uint32_t x, uint32_t k) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __umul24(x, k);
#else
    return (uint32_t)((uint64_t)(x & 0xFFFFFFu) * (uint64_t)(k & 0xFFFFFFu));
#endif
}

// Two-choice (cuckoo) open addressing: a key lives either at slot h1 of the lower
// half or at slot h2 of the upper half, so a lookup is exactly two independent
// 8-byte loads and has no probe loop.  On a 64-wide wavefront a probe loop runs
// as long as its slowest lane, which for linear probing at 38 % load is about 8
// rounds for a miss (against a mean of 1.8 per lane).
//
// A device slot is 8 bytes, {what the slot index does not say about the key, rank
// word}: the 24-bit mix m(a, b) = ((a + b * Kb) mod 2^24) * Ka mod 2^24 (Ka odd) is
// a bijection of a for a fixed b, its top log2(half) bits are the slot index, and
// the rest of m together with b names the key exactly.  Half the bytes per probe of
// a slot that holds both ids, and half the cache lines a cold L2 has to pull.
struct TableView {
    const uint2 *slots;        // {low bits of the mix | right id << 8, rank word}; empty: {0, kNoRank}
    const uint32_t *byte_pairs; // [65536] direct table for pairs of byte symbols: rank word or kNoRank
                               // rank word: see device_rank_word
    const int32_t *merged_of;  // [n_merges] merged id by rank order
    const int32_t *rank_of;    // [n_merges] caller's rank value by rank order
    const uint2 *sym_lr;       // [max_id + 1] per id: {lowest rank order of a rule with the id as its right part,
                               // ... as its left part}, kNoRank where there is none
    uint32_t half;             // slots per half (power of two, 2^16 .. 2^24)
    int low_bits;              // 24 - log2(half): bits of the mix below the slot index
    int index_bits;            // log2(half)
    int32_t merged_delta;      // >= 0: merged id = rank order + merged_delta for every rule; -1: use merged_of
    HashSeed seed;
};

// x * k + a with a 24-bit x and k, low 32 bits: one full-rate VALU op on the GPU
// (left to itself the compiler picks the quarter-rate 64-bit multiply-add).
__host__ __device__ inline uint32_t mad24(uint32_t x, uint32_t k, uint32_t a) {
#if defined(__HIP_DEVICE_COMPILE__)
    uint32_t r;
    asm("v_mad_u32_u24 %0, %1, %2, %3" : "=v"(r) : "v"(x), "s"(k), "v"(a));   // k: a multiplier of the seed, uniform
    return r;
#else
    return (uint32_t)((uint64_t)(x & 0xFFFFFFu) * (uint64_t)(k & 0xFFFFFFu)) + a;
#endif
}

// The mix of pair (a, b); only its low 24 bits count.  Two full-rate 24-bit multiplies.
__host__ __device__ inline uint32_t mix1(const HashSeed &s, uint32_t a, uint32_t b) {
    return mul24(mad24(b, s.k1b, a), s.k1a);
}
__host__ __device__ inline uint32_t mix2(const HashSeed &s, uint32_t a, uint32_t b) {
    return mul24(mad24(b, s.k2b, a), s.k2a);
}
// Slot index within a half, and the word a slot keeps of its key.
__host__ __device__ inline uint32_t slot_of(uint32_t mix, int low_bits, int index_bits) {
    return (mix >> low_bits) & ((1u << index_bits) - 1u);
}
__host__ __device__ inline uint32_t key_rest(uint32_t mix, int low_bits, uint32_t b) {
    return (mix & ((1u << low_bits) - 1u)) | (b << 8);
}

// Rank word (rank order = word >> kRankShift, 0 = merges first) of the pair whose
// two slots and key words these are, or kNoRank.  An empty slot holds kNoRank, so a
// key word that happens to equal an empty slot's changes nothing; at most one of the
// two slots holds the key, and kNoRank is the largest word.
__device__ inline uint32_t slot_match(const uint2 &s1, const uint2 &s2, uint32_t rest1, uint32_t rest2) {
    const uint32_t r1 = s1.x == rest1 ? s1.y : kNoRank;
    const uint32_t r2 = s2.x == rest2 ? s2.y : kNoRank;
    return min(r1, r2);
}
// The two slots of pair (a, b): load both, then slot_match with the same key words.
// Only the low 24 bits of a and b count (the 24-bit multiplies ignore the rest, a carry
// only travels upwards, and b << 8 drops its top byte), so callers may leave flag bits there.
// A slot is addressed by a 32-bit byte offset from the start of its half (one bit-field
// extract and one shift; the table has fewer than 2^25 slots), which lets the load take
// the base from scalar registers instead of a 64-bit address per lane.
struct SlotProbe { uint32_t off1, off2, rest1, rest2; };
__device__ inline SlotProbe slot_probe(const TableView &t, uint32_t a, uint32_t b) {
    const uint32_t m1 = mix1(t.seed, a, b), m2 = mix2(t.seed, a, b);
    SlotProbe q;
    q.off1 = __builtin_amdgcn_ubfe(m1, (uint32_t)t.low_bits, (uint32_t)t.index_bits) << 3;
    q.off2 = __builtin_amdgcn_ubfe(m2, (uint32_t)t.low_bits, (uint32_t)t.index_bits) << 3;
    q.rest1 = key_rest(m1, t.low_bits, b);
    q.rest2 = key_rest(m2, t.low_bits, b);
    return q;
}
__device__ inline uint2 slot_lower(const TableView &t, const SlotProbe &q) {
    return *(const uint2 *)((const char *)t.slots + q.off1);
}
__device__ inline uint2 slot_upper(const TableView &t, const SlotProbe &q) {
    return *(const uint2 *)((const char *)(t.slots + t.half) + q.off2);
}
__device__ inline uint32_t table_find(const TableView &t, uint32_t a, uint32_t b) {
    const SlotProbe q = slot_probe(t, a, b);
    const uint2 s1 = slot_lower(t, q), s2 = slot_upper(t, q);
    return slot_match(s1, s2, q.rest1, q.rest2);
}
__device__ inline uint32_t merged_id_of(const TableView &t, uint32_t rank) {
    return t.merged_delta >= 0 ? rank + (uint32_t)t.merged_delta : (uint32_t)t.merged_of[rank];
}

void set_error(const char *fmt, ...);
int hip_fail(hipError_t e, const char *what);
// BPE_OK if `device` (where a handle's memory lives) is the calling thread's current device.
int check_device(int device, const char *what);

// The rules of a merge table, validated and put in rank order (host side; shared
// by the table and the vocabulary builders).  Row i of the caller's arrays has
// merged id merged_row[i]; by_rank[k] = (rank value, row) of the k-th rule to
// apply; made_at[id] = k for the id that rule k makes, -1 for a byte, -2 unknown.
struct RuleOrder {
    std::vector<std::pair<int64_t, int64_t>> by_rank;
    std::vector<int64_t> merged_row;
    std::vector<int32_t> made_at;
    int64_t max_id;
};
int order_rules(const int32_t *merges, const int32_t *ranks, const int32_t *merged_ids, int64_t n, RuleOrder &ro);

// Pre-tokenizer (bpe_pretokenize.hip), as the raw encode path launches it: the
// caller supplies the status block, the tile-state array of
// pretokenize_state_bytes(n_bytes) bytes and the call id.  grid_out gets the number
// of workgroups; with `dry` nothing is launched.
int64_t pretokenize_state_bytes(int64_t n_bytes);
bool pretokenize_tile_ok(int tile_kib);
int launch_pretokenize(const uint8_t *bytes, int64_t n_bytes, const int32_t *seq_offsets, int64_t n_seqs,
                       int32_t *piece_offsets, int64_t max_pieces, int32_t *n_pieces, int32_t *seq_first_piece,
                       int32_t *status, unsigned long long *tile_state, int32_t call_id, int tile_kib,
                       hipStream_t s, int64_t *grid_out = nullptr, bool dry = false);

}  // namespace bpe

struct bpe_table {
    bpe::TableView view;
    bpe_table_info_t info;
    void *device_mem;     // one allocation: slots | byte_pairs | merged_of | rank_of | sym_lr
    int device;
};

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
constexpr uint32_t kCanLeft = 1u << 30, kCanRight = 1u << 31;
constexpr int kIdBits = 24;                    // token ids < 2^24: the hash multiplies with the 24-bit multiplier
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
// 16-byte loads and has no probe loop.  On a 64-wide wavefront a probe loop runs
// as long as its slowest lane, which for linear probing at 38 % load is about 8
// rounds for a miss (against a mean of 1.8 per lane).
struct TableView {
    const uint4 *slots;        // {key lo = right id, key hi = left id, value lo = rank word, value hi = merged id}
    const uint2 *byte_pairs;   // [65536] direct table for pairs of byte symbols: {rank word or kNoRank, merged id}
                               // rank word = rank order | kCanLeft / kCanRight of the merged id
    const int32_t *merged_of;  // [n_merges] merged id by rank order
    const int32_t *rank_of;    // [n_merges] caller's rank value by rank order
    const uint2 *sym_lr;       // [max_id + 1] per id: {lowest rank order of a rule with the id as its right part,
                               // ... as its left part}, kNoRank where there is none
    uint32_t half;             // slots per half (power of two)
    int shift;                 // 32 - log2(half)
    int32_t merged_delta;      // >= 0: merged id = rank order + merged_delta for every rule; -1: use merged_of
    HashSeed seed;
};

// x * k + a with a 24-bit x and k, low 32 bits: one full-rate VALU op on the GPU
// (left to itself the compiler picks the quarter-rate 64-bit multiply-add).
__host__ __device__ inline uint32_t mad24(uint32_t x, uint32_t k, uint32_t a) {
#if defined(__HIP_DEVICE_COMPILE__)
    uint32_t r;
    asm("v_mad_u32_u24 %0, %1, %2, %3" : "=v"(r) : "v"(x), "v"(k), "v"(a));
    return r;
#else
    return (uint32_t)((uint64_t)(x & 0xFFFFFFu) * (uint64_t)(k & 0xFFFFFFu)) + a;
#endif
}

// Slot index: fold the pair into 24 bits (a + b * Kb), multiply by Ka, keep the
// top bits of the low 32-bit word.  Two full-rate 24-bit multiplies.
__host__ __device__ inline uint32_t slot1(const HashSeed &s, int shift, uint32_t a, uint32_t b) {
    return mul24(mad24(b, s.k1b, a), s.k1a) >> shift;
}
__host__ __device__ inline uint32_t slot2(const HashSeed &s, int shift, uint32_t a, uint32_t b) {
    return mul24(mad24(b, s.k2b, a), s.k2a) >> shift;
}

// Rank word (rank order in the low kRankBits bits, 0 = merges first) and merged id of
// pair (a, b), or kNoRank.
__device__ inline uint32_t slot_match(const uint4 &s1, const uint4 &s2, uint32_t a, uint32_t b, uint32_t &merged) {
    const bool hit1 = s1.x == b && s1.y == a;
    const bool hit2 = s2.x == b && s2.y == a;
    merged = hit1 ? s1.w : s2.w;
    return hit1 ? s1.z : (hit2 ? s2.z : kNoRank);
}
__device__ inline uint32_t table_find(const TableView &t, uint32_t a, uint32_t b, uint32_t &merged) {
    const uint4 s1 = t.slots[slot1(t.seed, t.shift, a, b)];
    const uint4 s2 = t.slots[t.half + slot2(t.seed, t.shift, a, b)];
    return slot_match(s1, s2, a, b, merged);
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
// pretokenize_state_bytes(n_bytes) bytes and the call id.
int64_t pretokenize_state_bytes(int64_t n_bytes);
bool pretokenize_tile_ok(int tile_kib);
int launch_pretokenize(const uint8_t *bytes, int64_t n_bytes, const int32_t *seq_offsets, int64_t n_seqs,
                       int32_t *piece_offsets, int64_t max_pieces, int32_t *n_pieces, int32_t *seq_first_piece,
                       int32_t *status, unsigned long long *tile_state, int32_t call_id, int tile_kib,
                       hipStream_t s);

}  // namespace bpe

struct bpe_table {
    bpe::TableView view;
    bpe_table_info_t info;
    void *device_mem;     // one allocation: slots | byte_pairs | merged_of | rank_of | sym_lr
    int device;
};

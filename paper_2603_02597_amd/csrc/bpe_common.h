// Shared by the host-side table builder and the device kernels of this library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bpe_mi355x.h"

namespace bpe {

constexpr uint64_t kEmptyKey = ~0ull;          // no valid key: ids are non-negative int32
constexpr uint32_t kNoRank = 0xFFFFFFFFu;      // "pair not in the table"
constexpr int kRankBits = 26;                  // ranks < 2^26 so that (rank << 6 | lane) fits 32 bits
constexpr int kWave = 64;
constexpr int kWavesPerGroup = 4;
constexpr int kGroupThreads = kWave * kWavesPerGroup;
constexpr int kMaxPiecesPerWave = 32;
constexpr int kLdsMaxLen = 7168;               // symbols of one piece held twice in 64 KiB of LDS
constexpr int32_t kLongMark = -1;              // per-piece count placeholder: "workgroup path pending"

// Slot index of a pair: a 32-bit multiplicative mix, top `bits` bits.  The same
// function places keys on the host and finds them on the device.
__host__ __device__ inline uint32_t pair_hash(uint32_t a, uint32_t b) {
    uint32_t h = a * 0x9E3779B1u + b * 0x7FEB352Du;
    h ^= h >> 16;
    h *= 0x846CA68Bu;
    return h;
}

struct TableView {
    const uint4 *slots;   // {key lo = right id, key hi = left id, value lo = rank, value hi = merged id}
    uint32_t mask;        // capacity - 1
    int shift;            // 32 - log2(capacity)
    int max_probe;
};

// Probe the open-addressing table for pair (a, b).  Returns its rank and sets
// `merged`, or kNoRank.  Linear probing; a miss ends at the first empty slot and
// never takes more than max_probe steps (the longest chain found at build time).
__device__ inline uint32_t table_find(const TableView &t, uint32_t a, uint32_t b, uint32_t &merged) {
    uint32_t idx = pair_hash(a, b) >> t.shift;
    for (int probe = 0; probe < t.max_probe; ++probe) {
        const uint4 s = t.slots[idx];
        if (s.x == b && s.y == a) { merged = s.w; return s.z; }
        if ((s.x & s.y) == 0xFFFFFFFFu) break;
        idx = (idx + 1) & t.mask;
    }
    merged = 0xFFFFFFFFu;
    return kNoRank;
}

void set_error(const char *fmt, ...);
int hip_fail(hipError_t e, const char *what);

}  // namespace bpe

struct bpe_table {
    bpe::TableView view;
    bpe_table_info_t info;
    void *device_slots;
    int device;
};

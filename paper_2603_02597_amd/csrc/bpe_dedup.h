// Piece de-duplication (option dedup): word-like text repeats its pieces, so every
// distinct piece of at most 16 bytes is merged once and its tokens are handed to all
// its occurrences.  The paper names the idea as future work (section 6, "hybrid");
// what is built here stays on the device:
//   dedup_scatter_kernel  every piece writes its index into the slot of a hash table that
//                         its bytes hash to (plain stores: one of the pieces that share a
//                         slot stays);
//   dedup_find_kernel     every piece reads its slot and compares bytes with the piece it
//                         finds there: equal, and that piece stands for both; different
//                         (two words in one slot), and the piece stands for itself;
//   dedup_compact_kernel  the representatives, in piece order, become a dense list;
//   merge_raw_kernel      merges the pieces of that list (bpe_encode.hip; the list's
//                         length is only known on the device, as on the raw path);
//   dedup_count_kernel    every piece takes the record {token count, first token} of its
//                         representative; token totals per tile;
//   emit kernels          as without de-duplication.
// Device code, included by bpe_encode.hip.
#pragma once
#include "bpe_encode_params.h"
#include "bpe_lookback.h"

namespace bpe {

constexpr int kDedupMaxLen = 16;         // longer pieces are never looked up: each stands for itself

struct DedupParams {
    const uint8_t *bytes;
    const int32_t *off;
    int32_t n_bytes, n_pieces;
    int32_t *set;                // [capacity] index of a piece whose bytes hash to the slot
    uint32_t set_mask;           // capacity - 1 (a power of two)
    int32_t *rep;                // [n_pieces] the piece that stands for piece q (q itself if it is the first)
    int32_t *tile_reps;          // [n_tiles] representatives per tile of 256 pieces
    int32_t *piece_map;          // [n_pieces] the representatives in piece order
    int32_t *dense_of;           // [n_pieces] position of representative q in piece_map
    int32_t *n_reps;             // [1]
    const int2 *rec;             // [n_reps] records of the representatives (written by the merge kernel)
    int2 *rec_all;               // [n_pieces] records of all pieces
    int32_t *tile_sum;           // [n_tiles] tokens per tile of 256 pieces
    int32_t *status;
    int32_t call_id;
};

// The piece's bytes as four little-endian words, zero beyond its end (len <= 16).
__device__ inline uint4 piece_words(const DedupParams &p, int o, int len) {
    const uint32_t mis = (uint32_t)((uintptr_t)p.bytes & 3);
    const uint8_t *base = p.bytes - mis;
    const uint32_t pos = (uint32_t)o + mis;
    const uint32_t first = pos & ~3u, last = ((uint32_t)p.n_bytes + mis - 1u) & ~3u;
    uint32_t raw[5];
#pragma unroll
    for (int k = 0; k < 5; ++k) raw[k] = *(const uint32_t *)(base + min(first + 4u * (uint32_t)k, last));
    const uint32_t sh = (pos & 3u) * 8u;
    uint32_t w[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        w[k] = (uint32_t)((((uint64_t)raw[k + 1] << 32) | raw[k]) >> sh);
        const int valid = len - 4 * k;             // bytes of this word that belong to the piece
        w[k] = valid >= 4 ? w[k] : valid <= 0 ? 0u : (w[k] & (0xFFFFFFFFu >> (32 - 8 * valid)));
    }
    return make_uint4(w[0], w[1], w[2], w[3]);
}

__device__ inline uint32_t hash_words(const uint4 &w, int len) {
    uint32_t h = 0x9E3779B9u * (uint32_t)len;
    h = (h ^ w.x) * 0x85EBCA6Bu; h ^= h >> 15;
    h = (h ^ w.y) * 0xC2B2AE35u; h ^= h >> 13;
    h = (h ^ w.z) * 0x27D4EB2Fu; h ^= h >> 16;
    h = (h ^ w.w) * 0x165667B1u; h ^= h >> 15;
    return h;
}

// First pass: every piece of 1 .. 16 bytes stores its index into the slot its bytes hash to.
// Plain stores, no atomics: of the pieces that share a slot, whichever store lands last stays.
__global__ void __launch_bounds__(kGroupThreads) dedup_scatter_kernel(DedupParams p) {
    const int q = blockIdx.x * kGroupThreads + threadIdx.x;
    if (q >= p.n_pieces) return;
    const int o = p.off[q], o_next = p.off[q + 1];
    const bool bad = o < 0 || o_next < o || o_next > p.n_bytes || (q == 0 && o != 0) ||
                     (q == p.n_pieces - 1 && o_next != p.n_bytes);
    if (bad) __hip_atomic_store(&p.status[kStatusBadInput], p.call_id, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int len = bad ? 0 : o_next - o;
    if (len > 0 && len <= kDedupMaxLen) p.set[hash_words(piece_words(p, o, len), len) & p.set_mask] = q;
}

// Second pass, after the first one has ended (so that every workgroup reads the same words):
// a piece looks into its slot.  If the piece it finds there has the same bytes, that piece
// stands for both (and for itself: it reads the same slot); if not (another word hashed there
// and stayed, or the slot holds something an earlier launch or nobody wrote), the piece stands
// for itself.  Whatever the slot holds is only trusted after the bytes have been compared.
__global__ void __launch_bounds__(kGroupThreads) dedup_find_kernel(DedupParams p) {
    __shared__ int wave_reps[kWavesPerGroup];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const int q = blockIdx.x * kGroupThreads + tid;
    int rep = q;
    if (q < p.n_pieces) {
        const int o = p.off[q], o_next = p.off[q + 1];
        const bool bad = o < 0 || o_next < o || o_next > p.n_bytes;
        const int len = bad ? 0 : o_next - o;
        if (len > 0 && len <= kDedupMaxLen) {
            const uint4 mine = piece_words(p, o, len);
            const int r = p.set[hash_words(mine, len) & p.set_mask];
            if (r >= 0 && r < p.n_pieces && r != q) {
                const int ro = p.off[r], rlen = p.off[r + 1] - ro;
                if (rlen == len && ro >= 0 && ro + rlen <= p.n_bytes) {
                    const uint4 theirs = piece_words(p, ro, rlen);
                    if (theirs.x == mine.x && theirs.y == mine.y && theirs.z == mine.z && theirs.w == mine.w) rep = r;
                }
            }
        }
        p.rep[q] = rep;
    }
    const int n = __builtin_popcountll(__ballot(q < p.n_pieces && rep == q));
    if (lane == 0) wave_reps[wv] = n;
    __syncthreads();
    if (tid == 0) p.tile_reps[blockIdx.x] = wave_reps[0] + wave_reps[1] + wave_reps[2] + wave_reps[3];
}

// The representatives in piece order: piece_map[k] = k-th representative, dense_of[q] = k.
__global__ void __launch_bounds__(kGroupThreads) dedup_compact_kernel(DedupParams p, int n_tiles) {
    __shared__ int before_w[kWavesPerGroup], reps_w[kWavesPerGroup];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const int tile = blockIdx.x;
    const int q = tile * kGroupThreads + tid;
    const bool is_rep = q < p.n_pieces && p.rep[q] == q;
    int before = 0;                // representatives in the tiles before this one (tile_reps is 256-byte aligned)
    for (int t = tid * 4; t < tile; t += kGroupThreads * 4) {
        const int4 a = *(const int4 *)(p.tile_reps + t);
        before += a.x + (t + 1 < tile ? a.y : 0) + (t + 2 < tile ? a.z : 0) + (t + 3 < tile ? a.w : 0);
    }
    before = __builtin_amdgcn_readlane(wave_scan_inclusive(before), kWave - 1);
    const uint64_t m = __ballot(is_rep);
    if (lane == 0) { before_w[wv] = before; reps_w[wv] = __builtin_popcountll(m); }
    __syncthreads();
    int base = 0, total = 0;
    for (int w = 0; w < kWavesPerGroup; ++w) {
        base += before_w[w];
        if (w < wv) base += reps_w[w];
        total += reps_w[w];
    }
    if (is_rep) {
        const int k = base + __builtin_popcountll(m & ((1ull << lane) - 1));
        p.piece_map[k] = q;
        p.dense_of[q] = k;
    }
    if (tile == n_tiles - 1 && tid == 0) {
        int all = total;
        for (int w = 0; w < kWavesPerGroup; ++w) all += before_w[w];
        *p.n_reps = all;
    }
}

// Every piece takes the record of its representative; token totals per tile.
__global__ void __launch_bounds__(kGroupThreads) dedup_count_kernel(DedupParams p) {
    __shared__ int wave_tokens[kWavesPerGroup];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const int q = blockIdx.x * kGroupThreads + tid;
    int c = 0;
    if (q < p.n_pieces) {
        const int r = p.rep[q];
        // (indices kept inside the arrays whatever an uninitialised workspace made of them)
        const int d = p.dense_of[min(max(r, 0), p.n_pieces - 1)];
        const int2 rec = p.rec[min(max(d, 0), p.n_pieces - 1)];
        p.rec_all[q] = rec;
        c = max(rec.x, 0);
    }
    const int wave_total = __builtin_amdgcn_readlane(wave_scan_inclusive(c), kWave - 1);
    if (lane == 0) wave_tokens[wv] = wave_total;
    __syncthreads();
    if (tid == 0) {
        p.tile_sum[blockIdx.x] = wave_tokens[0] + wave_tokens[1] + wave_tokens[2] + wave_tokens[3];
    }
}

}  // namespace bpe

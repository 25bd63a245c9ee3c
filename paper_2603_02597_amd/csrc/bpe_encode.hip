// The merge loop (paper sections 3.4 and 3.5: pair evaluation, argmin,
// compaction, repeat) and the on-device assembly of the dense output (section
// 3.1, stage 4), for gfx950.
//
// All kernels work on the same tiling of the piece array (a tile = up to 64
// pieces per wavefront x 4 wavefronts).  merge_tile merges every piece of a tile
// by length class:
//     <= 16 bytes    one lane per piece, state in LDS columns;
//     <= 64 bytes    one lane per symbol, one piece per wavefront round;
//     <= 1024 bytes  one wavefront, piece double buffered in its LDS region;
//     longer         one piece per workgroup, double buffered in LDS (in the
//                    workspace beyond the LDS budget).
// Shallow grids: encode_kernel does the merges and the ordered assembly of the
// output in one launch (tile totals chained through tagged state words).
// Deeper grids: merge_kernel, then emit_kernel (out_offsets and the dense copy
// into out_ids), with scan_tiles_kernel between them when there are too many
// tile totals for every emit tile to add them up itself.
// Raw path (bpe_encode_raw): the pre-tokenizer first, then merge_raw_kernel and
// emit_raw_kernel, which stride over the tiles that exist (the piece count is
// only known on the device), then the first token of every sequence.
// Option paper_kernel: the paper's own two kernels, one workgroup per piece.
// No kernel allocates, and the host side neither synchronises nor copies.
#include <algorithm>
#include <atomic>
#include <new>

#include "bpe_common.h"
#include "bpe_lookback.h"

namespace bpe {

struct EncodeParams {
    TableView table;
    const uint8_t *bytes;
    const int32_t *off;
    int32_t n_bytes;
    int32_t n_pieces;    // with n_pieces_dev: the capacity of the piece arrays
    const int32_t *n_pieces_dev;   // raw path: the piece count is only known on the device (else nullptr)
    const int32_t *seq_first_piece;   // raw path: [n_seqs + 1] first piece of every sequence
    int32_t *seq_token_offsets;       // raw path: [n_seqs + 1] first token of every sequence
    int32_t n_seqs;
    int32_t P;           // pieces per wavefront (<= 64)
    int32_t W;           // wavefronts of a workgroup that own pieces: 4, or 1 (with P = 1: one piece per workgroup)
    int32_t raw_auto_P;  // raw path: the kernels choose P themselves once the piece count is known
    int32_t tiny_max;    // longest piece the lane-per-piece path takes (<= 16)
    int32_t wave_max;    // longest piece the lane-per-symbol path takes (<= 64)
    int32_t wave_lds_max;  // longest piece one wavefront takes through its LDS region (<= kWaveLdsMax)
    int32_t lds_max;     // longest piece the workgroup path keeps in LDS
    int32_t level;       // selection level 1, 2 or 3
    int32_t runs_by_best_rank;   // at level 3: pieces that are mostly runs of one byte take the level-2 passes
    int32_t paper;       // 0, or the paper's kernel to run instead: 1 = section 3.4, 2 = section 3.5 (one piece per tile)
    int2 *rec;           // [n_pieces] {tokens of the piece, its first token or -1 if that is in scratch too}
    int32_t *tile_sum;   // [n_tiles]
    int32_t *tile_base;  // [n_tiles]
    int32_t *scratch;    // [n_bytes] tokens of piece q at scratch[off[q] ...]
    int32_t *scratch2;   // [n_bytes] second buffer of the workspace ping-pong
    int32_t *status;     // [0] = call id if bad offsets were seen, [2] = call id of the call that ran last,
                         // [3] = call id if a wait ran out; the host derives the verdict from them
    int32_t call_id;
    unsigned long long *tile_state;  // single-kernel path: [n_tiles] (tag << 34) | (flag << 32) | value
    int32_t *out_ids;
    int32_t *out_offsets;
};

__device__ inline int lane_id() { return threadIdx.x & (kWave - 1); }
__device__ inline int mbcnt(uint64_t m) {   // set bits of m below this lane
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0));
}
__device__ inline int read_lane(int v, int l) {   // l must be the same in every lane
    return __builtin_amdgcn_readlane(v, __builtin_amdgcn_readfirstlane(l));
}
__device__ inline uint32_t permute_push(int dst_lane, uint32_t v) {   // lane dst_lane receives v
    return (uint32_t)__builtin_amdgcn_ds_permute(dst_lane << 2, (int)v);
}

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
struct TinyState {
    uint32_t S[kTinyMax][kWave];
    uint32_t R[kTinyMax][kWave];
};

__device__ inline uint32_t merged_id_of(const TableView &t, uint32_t rank) {
    return t.merged_delta >= 0 ? rank + (uint32_t)t.merged_delta : (uint32_t)t.merged_of[rank];
}

// Merges the lane's piece bytes[o .. o + len) if `mine`; len <= kTinyMax.  Returns
// the mask of positions that hold the final tokens (they stay in L.S[.][lane]).
// Loads are batched so that dependent round trips stay few: all bytes of the
// piece (five aligned dwords), then all byte-pair ranks, then per merge the two
// neighbour symbols and the two new pairs' slots together.
__device__ uint32_t tiny_merge(const EncodeParams &p, TinyState &L, int o, int len, bool mine) {
    const int lane = lane_id();
    const int my_len = mine ? len : 0;
    if (!__ballot(my_len > 0)) return 0u;

    // the piece's bytes as 4 dwords: aligned loads, then a byte-granular funnel shift
    uint32_t w[4] = {0, 0, 0, 0};
    if (my_len) {
        const uintptr_t addr = (uintptr_t)(p.bytes + o);
        const uint32_t *src = (const uint32_t *)(addr & ~(uintptr_t)3);
        const uintptr_t end = (uintptr_t)(p.bytes + p.n_bytes);
        uint32_t raw[5];
#pragma unroll
        for (int k = 0; k < 5; ++k) raw[k] = (uintptr_t)(src + k) < end ? src[k] : 0u;
        const uint32_t sh = (uint32_t)(addr & 3) * 8;
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
        r0[j] = j + 1 < my_len ? p.table.byte_pairs[(c[j] << 8) | c[j + 1]].x : kNoRank;
    // S[j] = id | flags << 24: whether the symbol can be the left / right part of a rule
    // (bits 0 / 1).  Bytes are not classified: both flags set.
#pragma unroll
    for (int j = 0; j < kTinyMax; ++j) L.S[j][lane] = c[j] | (3u << 24);
    // R[j] = rank order << 6 | flags of the merged id << 4 | j
#pragma unroll
    for (int j = 0; j < kTinyMax - 1; ++j)
        L.R[j][lane] = r0[j] != kNoRank ? (((r0[j] & kRankMask) << 6) | ((r0[j] >> 30) << 4) | (uint32_t)j) : kNoRank;
    L.R[kTinyMax - 1][lane] = kNoRank;
    uint32_t alive = my_len ? (0xFFFFFFFFu >> (32 - my_len)) : 0u;

    for (;;) {
        uint32_t best = kNoRank;
#pragma unroll
        for (int j = 0; j < kTinyMax - 1; ++j) best = min(best, L.R[j][lane]);
        if (!__ballot(best != kNoRank)) break;
        if (best != kNoRank) {
            const int k = best & 15;
            const uint32_t flags = (best >> 4) & 3u;                 // bit 0: merged id can be a left part, bit 1: a right part
            const uint32_t merged = merged_id_of(p.table, best >> 6);
            const uint32_t after = alive >> (k + 1);                 // non-zero: the pair's right symbol
            const int nk = k + 1 + __builtin_ctz(after);
            alive &= ~(1u << nk);
            const uint32_t rest = alive >> (nk + 1);                 // symbols right of the merged one
            const uint32_t below = alive & ((1u << k) - 1);          // symbols left of it
            const int nn = rest ? nk + 1 + __builtin_ctz(rest) : k;
            const int pk = below ? 31 - __builtin_clz(below) : k;
            const uint32_t right_sym = L.S[nn][lane];                // both reads before the write below
            const uint32_t left_sym = L.S[pk][lane];
            L.S[k][lane] = merged | (flags << 24);
            L.R[nk][lane] = kNoRank;
            // New pairs (merged, right) and (left, merged).  A pair needs a lookup only if
            // its first symbol can be a left part and its second a right part of some rule;
            // the loads of both lookups are in flight together.
            const bool need_r = rest && (flags & 1u) && (right_sym >> 25);
            const bool need_l = below && (flags & 2u) && ((left_sym >> 24) & 1u);
            uint32_t rr = kNoRank, rl = kNoRank, unused;
            uint4 a1, a2, b1, b2;   // each pair is only read under the predicate it was loaded under
            const uint32_t rs = right_sym & 0xFFFFFFu, ls = left_sym & 0xFFFFFFu;
            if (need_r) {
                a1 = p.table.slots[slot1(p.table.seed, p.table.shift, merged, rs)];
                a2 = p.table.slots[p.table.half + slot2(p.table.seed, p.table.shift, merged, rs)];
            }
            if (need_l) {
                b1 = p.table.slots[slot1(p.table.seed, p.table.shift, ls, merged)];
                b2 = p.table.slots[p.table.half + slot2(p.table.seed, p.table.shift, ls, merged)];
            }
            if (need_r) rr = slot_match(a1, a2, merged, rs, unused);
            if (need_l) rl = slot_match(b1, b2, ls, merged, unused);
            L.R[k][lane] = rr != kNoRank ? (((rr & kRankMask) << 6) | ((rr >> 30) << 4) | (uint32_t)k) : kNoRank;
            if (below) L.R[pk][lane] = rl != kNoRank ? (((rl & kRankMask) << 6) | ((rl >> 30) << 4) | (uint32_t)pk) : kNoRank;
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

// Level 3 for a piece whose symbols sit one per lane: is the pair of rank r that
// starts at this lane bound to be merged (see "Selection level 3" below)?  lr = the
// lowest ranks of a rule with this lane's symbol as its right / left part; lanes
// without a pair pass r = kNoRank; only lanes with `want` ask.  The walks of all
// lanes advance together, four steps per batch of cross-lane reads.  Every lane must
// call it.
constexpr int kWaveSafeSteps = 7;
__device__ __forceinline__ bool wave_pair_is_bound(bool want, uint32_t r, uint2 lr, int lane, int cur) {
    bool open = want, left = false;
#pragma unroll
    for (int batch = 0; batch < (kWaveSafeSteps + 1) / 4; ++batch) {
        if (!__ballot(open)) break;
        uint32_t ql[4], rr[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int d = 4 * batch + k;
            ql[k] = d ? (uint32_t)__shfl_up((int)lr.x, d) : lr.x;
            rr[k] = (uint32_t)__shfl_up((int)r, d + 1);
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int j = lane - (4 * batch + k);
            if (open) {
                if (j == 0 || ql[k] > r) { left = true; open = false; }
                else if (!(rr[k] > r)) open = false;
            }
        }
    }
    open = want && left;
    bool right = false;
#pragma unroll
    for (int batch = 0; batch < (kWaveSafeSteps + 1) / 4; ++batch) {
        if (!__ballot(open)) break;
        uint32_t qr[4], rr[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int d = 4 * batch + k + 1;
            qr[k] = (uint32_t)__shfl_down((int)lr.y, d);
            rr[k] = (uint32_t)__shfl_down((int)r, d);
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int j = lane + 4 * batch + k + 1;
            if (open) {
                if (j == cur - 1 || qr[k] >= r) { right = true; open = false; }
                else if (!(rr[k] >= r)) open = false;
            }
        }
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
__device__ int encode_wave_piece(const EncodeParams &p, int base, int n) {
    const int lane = lane_id();
    const uint64_t lt_mask = (1ull << lane) - 1;
    uint32_t sym = 0;
    if (lane < n) sym = p.bytes[base + lane];
    int cur = n;
    for (;;) {
        const uint32_t nxt = (uint32_t)__shfl_down((int)sym, 1);
        uint32_t merged = 0, key = kNoRank;
        uint2 lr = make_uint2(kNoRank, kNoRank);
        if (p.level >= 3 && lane < cur) lr = p.table.sym_lr[sym];
        if (lane + 1 < cur) {
            const uint32_t r = table_find(p.table, sym, nxt, merged);
            if (r != kNoRank) key = ((r & kRankMask) << 6) | (uint32_t)lane;
        }
        uint32_t best = key;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) best = min(best, (uint32_t)__shfl_xor((int)best, d));
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
    if (lane < cur) p.scratch[base + lane] = (int32_t)sym;
    return cur;
}

// ---------------------------------------------------------------------------
// Workgroup path: one piece at a time by all 256 threads (section 3.4's
// one-block-per-chunk scheme, with the double-buffered compaction of section 3.5
// generalised to several merges per pass by a prefix count of removed symbols).

struct GroupTmp {
    uint32_t min_lo[kWavesPerGroup], min_hi[kWavesPerGroup];
    int max_w[kWavesPerGroup];
    int sum_w[kWavesPerGroup];
    int last_w[kWavesPerGroup];
    int all_w[kWavesPerGroup];
};

__device__ inline uint64_t group_min(uint64_t v, GroupTmp &tmp) {
    uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const uint32_t olo = (uint32_t)__shfl_xor((int)lo, d), ohi = (uint32_t)__shfl_xor((int)hi, d);
        if (ohi < hi || (ohi == hi && olo < lo)) { hi = ohi; lo = olo; }
    }
    const int wv = threadIdx.x / kWave;
    if (lane_id() == 0) { tmp.min_lo[wv] = lo; tmp.min_hi[wv] = hi; }
    __syncthreads();
    uint64_t best = ~0ull;
    for (int w = 0; w < kWavesPerGroup; ++w)
        best = min(best, ((uint64_t)tmp.min_hi[w] << 32) | tmp.min_lo[w]);
    return best;
}

// Exclusive max-scan over the threads of the group (identity -1).
__device__ inline int group_scan_max_excl(int v, GroupTmp &tmp) {
    const int lane = lane_id(), wv = threadIdx.x / kWave;
    int inc = v;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const int o = __shfl_up(inc, d);
        if (lane >= d) inc = max(inc, o);
    }
    if (lane == kWave - 1) tmp.max_w[wv] = inc;
    __syncthreads();
    int ex = __shfl_up(inc, 1);
    if (lane == 0) ex = -1;
    for (int w = 0; w < wv; ++w) ex = max(ex, tmp.max_w[w]);
    return ex;
}

// Exclusive sum-scan over the threads of the group; total to every thread.
__device__ inline int group_scan_sum_excl(int v, GroupTmp &tmp, int &total) {
    const int lane = lane_id(), wv = threadIdx.x / kWave;
    int inc = v;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const int o = __shfl_up(inc, d);
        if (lane >= d) inc += o;
    }
    if (lane == kWave - 1) tmp.sum_w[wv] = inc;
    __syncthreads();
    int ex = inc - v;
    total = 0;
    for (int w = 0; w < kWavesPerGroup; ++w) {
        if (w < wv) ex += tmp.sum_w[w];
        total += tmp.sum_w[w];
    }
    return ex;
}

// The threads that share one long piece: the whole workgroup, or one wavefront
// (no barriers: a wavefront runs in lockstep and its LDS operations stay in order).
struct GroupScope {
    static constexpr int kThreads = kGroupThreads;
    GroupTmp &tmp;
    __device__ int tid() const { return threadIdx.x; }
    __device__ void sync() const { __syncthreads(); }
    __device__ uint64_t min_u64(uint64_t v) const { return group_min(v, tmp); }
    __device__ int scan_max_excl(int v) const { return group_scan_max_excl(v, tmp); }
    __device__ int scan_sum_excl(int v, int &total) const { return group_scan_sum_excl(v, tmp, total); }
    // the largest v of all threads (a barrier must separate two calls)
    __device__ int max_all(int v) const {
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) v = max(v, __shfl_xor(v, d));
        if (lane_id() == 0) tmp.all_w[threadIdx.x / kWave] = v;
        __syncthreads();
        int m = tmp.all_w[0];
        for (int w = 1; w < kWavesPerGroup; ++w) m = max(m, tmp.all_w[w]);
        return m;
    }
    // v of the thread before this one (0 for the first thread)
    __device__ int from_previous_thread(int v) const {
        const int lane = lane_id(), wv = threadIdx.x / kWave;
        if (lane == kWave - 1) tmp.last_w[wv] = v;
        __syncthreads();
        const int up = __shfl_up(v, 1);
        return lane ? up : (wv ? tmp.last_w[wv - 1] : 0);
    }
};

struct WaveScope {
    static constexpr int kThreads = kWave;
    __device__ int tid() const { return lane_id(); }
    __device__ void sync() const {
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
        __builtin_amdgcn_wave_barrier();
    }
    __device__ uint64_t min_u64(uint64_t v) const {
        uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            const uint32_t olo = (uint32_t)__shfl_xor((int)lo, d), ohi = (uint32_t)__shfl_xor((int)hi, d);
            if (ohi < hi || (ohi == hi && olo < lo)) { hi = ohi; lo = olo; }
        }
        return ((uint64_t)hi << 32) | lo;
    }
    __device__ int scan_max_excl(int v) const {
        const int lane = lane_id();
        int inc = v;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            const int o = __shfl_up(inc, d);
            if (lane >= d) inc = max(inc, o);
        }
        const int ex = __shfl_up(inc, 1);
        return lane == 0 ? -1 : ex;
    }
    __device__ int scan_sum_excl(int v, int &total) const {
        const int lane = lane_id();
        int inc = v;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            const int o = __shfl_up(inc, d);
            if (lane >= d) inc += o;
        }
        total = __shfl(inc, kWave - 1);
        return inc - v;
    }
    __device__ int from_previous_thread(int v) const {
        const int up = __shfl_up(v, 1);
        return lane_id() ? up : 0;
    }
    __device__ int max_all(int v) const {
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) v = max(v, __shfl_xor(v, d));
        return v;
    }
};

// One pass of the loop of section 3.4 over the cur >= 2 symbols in A, by the threads
// of `sc`: pair evaluation, argmin, and the double-buffered compaction of section
// 3.5 generalised to several merges per pass (selection level 2: every occurrence
// of the best-ranked pair, offsets 0, 2, 4 ... inside a run of equal symbols) by a
// prefix count of the removed symbols.  Writes the new sequence to B and returns
// its length, or -1 (B untouched) if no pair is in the table.
template <typename Scope, typename Ptr>
__device__ __forceinline__ int best_rank_pass(const EncodeParams &p, Ptr A, Ptr B, int cur, const Scope &sc) {
    constexpr int T = Scope::kThreads;
    const int tid = sc.tid();
    // pair evaluation, strided over the threads (section 3.4 step 1),
    // four independent lookups in flight per thread
    uint64_t best = ~0ull;
    for (int i0 = tid; i0 + 1 < cur; i0 += 4 * T) {
        uint32_t r[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = i0 + u * T;
            uint32_t mm;
            r[u] = i + 1 < cur ? table_find(p.table, (uint32_t)A[i], (uint32_t)A[i + 1], mm) : kNoRank;
            if (r[u] != kNoRank) r[u] &= kRankMask;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (r[u] != kNoRank) best = min(best, ((uint64_t)r[u] << 32) | (uint32_t)(i0 + u * T));
    }
    best = sc.min_u64(best);                           // argmin, ties to the left (step 2)
    if (best == ~0ull) return -1;
    const int best_pos = (int)(uint32_t)best;
    const int32_t a = A[best_pos], bb = A[best_pos + 1];
    const uint32_t merged = merged_id_of(p.table, (uint32_t)(best >> 32));

    // compaction (step 3): thread t owns positions [c0, c1)
    const int chunk = (cur + T - 1) / T;
    const int c0 = min(tid * chunk, cur), c1 = min(c0 + chunk, cur);
    const bool every = p.level >= 2;
    const bool run_rule = every && a == bb;
    int carry_break = -1;          // last position before c0 whose symbol is not `a`
    if (run_rule) {
        int lb = -1;
        for (int i = c0; i < c1; ++i) if (A[i] != a) lb = i;
        carry_break = sc.scan_max_excl(lb);
    }
    // is the pair at position i merged in this pass?  last_break = last position <= i
    // holding a symbol other than `a` (only used by the run rule)
    auto selected = [&](int i, int last_break) -> bool {
        if (!every) return i == best_pos;
        if (i + 1 >= cur || A[i] != a || A[i + 1] != bb) return false;
        return !run_rule || (((i - (last_break + 1)) & 1) == 0);
    };
    int lb = carry_break;
    bool prev = c0 > 0 && c0 < cur && selected(c0 - 1, carry_break);
    const bool prev0 = prev;
    int kept = 0;
    for (int i = c0; i < c1; ++i) {
        if (run_rule && A[i] != a) lb = i;
        const bool s = selected(i, lb);
        kept += !prev;
        prev = s;
    }
    int total;
    int dst = sc.scan_sum_excl(kept, total);
    lb = carry_break;
    prev = prev0;
    for (int i = c0; i < c1; ++i) {
        if (run_rule && A[i] != a) lb = i;
        const bool s = selected(i, lb);
        if (!prev) B[dst++] = s ? (int32_t)merged : A[i];
        prev = s;
    }
    sc.sync();
    return total;
}

// Encode piece [b, b + len) by the threads of `sc`, with buffers A and B (both
// hold len symbols; LDS or workspace): the paper's one-block-per-chunk loop
// (section 3.4).  Leaves the tokens at p.scratch[b ...]; returns their number.
template <typename Scope, typename Ptr>
__device__ __forceinline__ int encode_long_piece(const EncodeParams &p, int b, int len, Ptr A, Ptr B,
                                                 const Scope &sc) {
    constexpr int T = Scope::kThreads;
    const int tid = sc.tid();
    for (int i = tid; i < len; i += T) A[i] = p.bytes[b + i];
    sc.sync();
    int cur = len;
    while (cur >= 2) {
        const int n = best_rank_pass(p, A, B, cur, sc);
        if (n < 0) break;
        Ptr t = A; A = B; B = t;
        cur = n;
    }
    int32_t *out = p.scratch + b;
    if ((const void *)A != (const void *)out) {
        for (int i = tid; i < cur; i += T) out[i] = A[i];
    }
    sc.sync();
    return cur;
}

// ---------------------------------------------------------------------------
// Selection level 3: every pair that greedy is bound to merge, in one pass.
//
// The introduction of the paper promises "non-overlapping local minima" per pass and
// section 3.5 withdraws it, because a local minimum of the ranks can lose one of its
// symbols to a neighbour before its turn comes.  The exact form used here: the pair
// (u, v) at positions (i, i+1), of rank r, is *bound to be merged* if neither u nor v
// can be taken by another merge while the pair waits.  Until the pair merges, every
// merge has a rank below r (or r itself, further left), so
//   u is safe from the left   if, walking left from u over pairs of rank > r, one
//     reaches the start of the piece or a symbol that is the right part of no rule
//     of rank <= r: that symbol stays, so do all symbols between it and u, and none
//     of the pairs between them comes before (u, v);
//   v is safe from the right  if, walking right from v over pairs of rank >= r, one
//     reaches the end of the piece or a symbol that is the left part of no rule of
//     rank < r.
// Merging such a pair early changes nothing: the pairs it creates contain the fresh
// id and so rank above r (a rule's parts are made by lower ranks), greedy would not
// touch them before this pair's turn either.  Two such pairs never overlap: for
// neighbours (u, v) and (v, z) the right test of the first needs r1 <= r2 and the
// left test of the second needs r1 > r2.  A walk that would leave what is in LDS is
// given up (the pair waits for a later pass): inside a window it goes kSafeSteps
// symbols at most, in a resident piece as far as it needs.  The occurrences of the
// piece's best rank are still taken by the level-2 rule, which is what guarantees
// progress and halves runs x x x ... per pass.  The per-id lowest ranks come from
// the table (TableView::sym_lr).
constexpr int kSafeSteps = 127;
static_assert((kSafeSteps + 1) % 4 == 0, "whole batches of four steps");
constexpr int kSafeHalo = kSafeSteps + 2;     // symbols a window holds on either side of the ones it decides
// Level 3 keeps four words per symbol in LDS (symbol, pair rank, the two lowest ranks of
// the symbol), so the LDS that holds a piece twice at levels 1-2 holds half as many symbols.
constexpr int kWaveBoundMax = kWaveLdsMax / 2;     // one wavefront, its own LDS region
constexpr int kWaveBoundHandOn = kWaveBoundMax + kWaveBoundMax / 4;   // longer pieces go to the workgroup
constexpr int kGroupBoundMax = kLdsMaxLen / 2;     // the workgroup
constexpr int kGroupBoundMin = 320;                // smallest window (small values exercise the windowed passes)
static_assert(kWaveBoundMax <= 32 * kWave && kGroupBoundMax <= 32 * kGroupThreads, "a thread's chunk fits a 32-bit mask");
static_assert(kGroupBoundMin > 2 * kSafeHalo, "a window decides at least one symbol");

// first / last: index of the piece's first / last symbol in these arrays (far outside
// the window if it is not in it); n: entries the arrays hold.  A walk looks at up to
// kSafeSteps + 1 symbols; the LDS reads of four steps are issued together and the
// steps then resolved in registers, so that a walk costs one or two LDS round trips
// instead of one per step (reads past the end of a walk are clamped into the arrays
// and ignored).
__device__ inline bool pair_is_bound(const uint32_t *R, const uint32_t *QL, const uint32_t *QR, int i, uint32_t r,
                                     int first, int last, int n, int max_batches) {
    bool open = true, safe = false;
#pragma nounroll
    for (int batch = 0; batch < max_batches && open; ++batch) {
        uint32_t ql[4], rr[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int j = i - (4 * batch + k);
            ql[k] = QL[max(j, 0)];
            rr[k] = R[max(j - 1, 0)];
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int j = i - (4 * batch + k);
            if (open) {
                if (j == first || ql[k] > r) { safe = true; open = false; }
                else if (!(rr[k] > r)) open = false;
            }
        }
    }
    if (!safe) return false;
    open = true;
    safe = false;
#pragma nounroll
    for (int batch = 0; batch < max_batches && open; ++batch) {
        uint32_t qr[4], rr[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int j = min(i + 1 + 4 * batch + k, n - 1);
            qr[k] = QR[j];
            rr[k] = R[j];
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int j = i + 1 + 4 * batch + k;
            if (open) {
                if (j == last || qr[k] >= r) { safe = true; open = false; }
                else if (!(rr[k] >= r)) open = false;
            }
        }
    }
    return safe;
}

// Pair evaluation for the n symbols in S (LDS): R[i] = rank order of (S[i], S[i+1]) or
// kNoRank (also for i = n - 1), QL[i] / QR[i] = lowest rank of a rule with S[i] as its
// right / left part.  Returns the thread's best (rank << 32 | i).
template <typename Scope>
__device__ __forceinline__ uint64_t evaluate_pairs(const EncodeParams &p, const int32_t *S, uint32_t *R, uint32_t *QL,
                                                   uint32_t *QR, int n, const Scope &sc) {
    constexpr int T = Scope::kThreads;
    uint64_t best = ~0ull;
    for (int i0 = sc.tid(); i0 < n; i0 += 4 * T) {
        uint32_t r[4];
        uint2 q[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = i0 + u * T;
            r[u] = kNoRank;
            q[u] = make_uint2(kNoRank, kNoRank);
            if (i < n) {
                const uint32_t sym = (uint32_t)S[i];
                q[u] = p.table.sym_lr[sym];
                uint32_t mm;
                if (i + 1 < n) r[u] = table_find(p.table, sym, (uint32_t)S[i + 1], mm);
                if (r[u] != kNoRank) r[u] &= kRankMask;
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = i0 + u * T;
            if (i < n) {
                R[i] = r[u];
                QL[i] = q[u].x;
                QR[i] = q[u].y;
                if (r[u] != kNoRank) best = min(best, ((uint64_t)r[u] << 32) | (uint32_t)i);
            }
        }
    }
    return best;
}

// One level-3 pass over a piece whose cur >= 2 symbols are in S (LDS).  The new
// sequence goes to S2, which may be the QL array (it is dead by then); returns its
// length, or -1 if no pair is in the table.
template <typename Scope>
__device__ __forceinline__ int bound_pairs_pass_lds(const EncodeParams &p, const int32_t *S, uint32_t *R, uint32_t *QL,
                                                    uint32_t *QR, int32_t *S2, int cur, const Scope &sc) {
    constexpr int T = Scope::kThreads;
    const int tid = sc.tid();
    uint64_t best = evaluate_pairs(p, S, R, QL, QR, cur, sc);
    best = sc.min_u64(best);
    sc.sync();
    if (best == ~0ull) return -1;
    const uint32_t rho = (uint32_t)(best >> 32);
    const int best_pos = (int)(uint32_t)best;
    const int32_t a = S[best_pos];
    const bool run_rule = a == S[best_pos + 1];

    const int chunk = (cur + T - 1) / T;       // at most 32: the selection of a chunk is kept as a bit mask
    const int c0 = min(tid * chunk, cur), c1 = min(c0 + chunk, cur);
    int carry_break = -1;          // last position before c0 whose symbol is not `a`
    if (run_rule) {
        int lb = -1;
        for (int i = c0; i < c1; ++i) if (S[i] != a) lb = i;
        carry_break = sc.scan_max_excl(lb);
    }
    // pair (i, i+1), i + 1 < cur; last_break = last position <= i holding a symbol other than `a`
    auto selected = [&](int i, int last_break) -> bool {
        const uint32_t r = R[i];
        if (r == kNoRank) return false;
        if (r == rho) return !run_rule || (((i - (last_break + 1)) & 1) == 0);
        return pair_is_bound(R, QL, QR, i, r, 0, cur - 1, cur, cur);       // the whole piece is here: no limit
    };
    int lb = carry_break;
    uint32_t mask = 0;             // bit k: the pair that starts at c0 + k merges
    for (int i = c0; i < c1; ++i) {
        if (run_rule && S[i] != a) lb = i;
        const bool sel = i + 1 < cur && selected(i, lb);
        mask |= (uint32_t)sel << (i - c0);
    }
    // a symbol goes unless the pair before it merges; for the first symbol of a chunk
    // that pair is the last one of the thread before
    const bool prev0 = sc.from_previous_thread(c1 > c0 ? (int)((mask >> (c1 - c0 - 1)) & 1u) : 0) != 0;
    const int kept = (c1 - c0) - __builtin_popcount(((mask << 1) | (uint32_t)prev0) & ((1u << (c1 - c0)) - 1u));
    int total;
    int dst = sc.scan_sum_excl(kept, total);   // every walk over R, QL, QR has ended when this returns
    bool prev = prev0;
    for (int i = c0; i < c1; ++i) {
        const bool sel = (mask >> (i - c0)) & 1u;
        if (!prev) S2[dst++] = sel ? (int32_t)merged_id_of(p.table, R[i]) : S[i];
        prev = sel;
    }
    sc.sync();
    return total;
}

// The best rank of a piece as the previous windowed pass saw it (before its merges),
// and the left symbol of that pair; run: both symbols of the pair are equal.
struct CarriedRank {
    uint32_t rho;      // kNoRank: none known (first pass) or no pair was in the table
    int32_t a;
    bool run;
};

// One pass over a piece too long for the LDS arrays: its cur symbols are in A
// (workspace), the new sequence goes to B (workspace).  The piece passes through the
// LDS arrays in windows of `cap` symbols, of which the inner ones are decided and the
// kSafeHalo on either side only looked at.  A pass sees a pair's rank only while
// its window is in LDS, so it cannot know the piece's best rank before it decides;
// it uses the one the previous pass found (`carried`).  If a pair of that rank is
// still there, it is the best rank now as well (every pair is an old one or contains
// a fresh id, which ranks above the merge that made it), so its occurrences take
// the best-rank rule and all other pairs the walks, as in a resident pass; if none is
// left, the rule selects nothing.  Either this pass or the next one merges something
// as long as any pair is in the table.  Returns the new length and leaves the best
// rank it saw in `carried`.
template <typename Scope>
__device__ __forceinline__ int bound_pairs_pass_windows(const EncodeParams &p, const int32_t *A, int32_t *B, int cur,
                                                        int32_t *S, uint32_t *R, uint32_t *QL, uint32_t *QR, int cap,
                                                        CarriedRank &carried, const Scope &sc) {
    constexpr int T = Scope::kThreads;
    const int tid = sc.tid();
    const int span = cap - 2 * kSafeHalo;
    const uint32_t rho = carried.rho;
    const int32_t a = carried.a;
    const bool run_rule = rho != kNoRank && carried.run;
    uint64_t best = ~0ull;         // this thread's best (rank << 32 | position in the piece)
    int out_base = 0;
    int run_break = -1;            // last position before the window's first decided symbol that does not hold `a`
    for (int g0 = 0; g0 < cur; g0 += span) {
        const int g1 = min(g0 + span, cur);
        const int lo = max(g0 - kSafeHalo, 0), hi = min(g1 + kSafeHalo, cur);
        const int n = hi - lo;
        for (int i = tid; i < n; i += T) S[i] = A[lo + i];
        sc.sync();
        const uint64_t wbest = evaluate_pairs(p, S, R, QL, QR, n, sc);
        if (wbest != ~0ull) best = min(best, wbest + (uint32_t)lo);
        sc.sync();
        const int d0 = g0 - lo, d1 = g1 - lo;                  // the symbols this window decides
        const int first = lo == 0 ? 0 : -(1 << 30), last = hi == cur ? n - 1 : (1 << 30);
        const int chunk = (d1 - d0 + T - 1) / T;
        const int c0 = min(d0 + tid * chunk, d1), c1 = min(c0 + chunk, d1);
        int carry_break = run_break;       // last position (in the piece) before lo + c0 that does not hold `a`
        int my_break = -1;
        if (run_rule) {
            for (int i = c0; i < c1; ++i) if (S[i] != a) my_break = lo + i;
            carry_break = max(run_break, sc.scan_max_excl(my_break));
        }
        // pair (i, i+1) of the window; last_break = last position of the piece <= lo + i that does not hold `a`
        auto selected = [&](int i, int last_break) -> bool {
            const uint32_t r = R[i];
            if (r == kNoRank) return false;
            if (r == rho) return !run_rule || (((lo + i - (last_break + 1)) & 1) == 0);
            return pair_is_bound(R, QL, QR, i, r, first, last, n, (kSafeSteps + 1) / 4);
        };
        uint32_t mask = 0;
        int lb = carry_break;
        for (int i = c0; i < c1; ++i) {
            if (run_rule && S[i] != a) lb = lo + i;
            mask |= (uint32_t)selected(i, lb) << (i - c0);
        }
        // the pair before the window's first symbol is the previous window's (or the halo's) to look at
        const int before = tid == 0 && c0 < c1 && lo + c0 > 0 && selected(c0 - 1, run_break);
        const int from_prev = sc.from_previous_thread(c1 > c0 ? (int)((mask >> (c1 - c0 - 1)) & 1u) : 0);
        const bool prev0 = tid == 0 ? before != 0 : from_prev != 0;
        const int kept = (c1 - c0) - __builtin_popcount(((mask << 1) | (uint32_t)prev0) & ((1u << (c1 - c0)) - 1u));
        int total;
        int dst = out_base + sc.scan_sum_excl(kept, total);
        bool prev = prev0;
        for (int i = c0; i < c1; ++i) {
            const bool sel = (mask >> (i - c0)) & 1u;
            if (!prev) B[dst++] = sel ? (int32_t)merged_id_of(p.table, R[i]) : S[i];
            prev = sel;
        }
        out_base += total;
        if (run_rule) run_break = max(run_break, sc.max_all(my_break));
        sc.sync();
    }
    best = sc.min_u64(best);
    sc.sync();
    carried.rho = kNoRank;
    if (best != ~0ull) {
        const int pos = (int)(uint32_t)best;
        carried.rho = (uint32_t)(best >> 32);
        carried.a = A[pos];
        carried.run = A[pos] == A[pos + 1];
    }
    return out_base;
}

// Whether at least half of the piece's adjacent bytes are equal.  Such a piece is runs
// x x x ...: the best-rank passes halve it per pass, nothing else in it can merge
// before them, and they hold twice as many symbols in the same LDS.
template <typename Scope>
__device__ __forceinline__ bool piece_is_run_like(const EncodeParams &p, int b, int n, const Scope &sc) {
    int eq = 0;
    for (int i = sc.tid(); i + 1 < n; i += Scope::kThreads) eq += p.bytes[b + i] == p.bytes[b + i + 1];
    int total;
    (void)sc.scan_sum_excl(eq, total);
    return 2 * total >= n;
}

// Encode piece [b, b + len) at selection level 3 by the threads of `sc`.  X: 4 * cap
// words of LDS.  A piece of more than cap symbols starts in the workspace and moves
// into LDS once it has shrunk to cap.  Leaves the tokens at p.scratch[b ...]; returns
// their number.
template <typename Scope>
__device__ __forceinline__ int encode_long_piece_bound(const EncodeParams &p, int b, int len, uint32_t *X, int cap,
                                                       const Scope &sc) {
    constexpr int T = Scope::kThreads;
    const int tid = sc.tid();
    int32_t *S = (int32_t *)X;
    uint32_t *R = X + cap, *QL = X + 2 * cap, *QR = X + 3 * cap;
    int32_t *out = p.scratch + b;
    int cur = len;
    if (len > cap) {
        int32_t *A = out, *B = p.scratch2 + b;
        for (int i = tid; i < len; i += T) A[i] = p.bytes[b + i];
        sc.sync();
        CarriedRank carried = {kNoRank, 0, false};
        bool done = false;
        while (cur > cap) {
            const int n = bound_pairs_pass_windows(p, A, B, cur, S, R, QL, QR, cap, carried, sc);
            { int32_t *t = A; A = B; B = t; }
            if (carried.rho == kNoRank) { done = true; cur = n; break; }    // no pair anywhere: n == cur
            cur = n;
        }
        if (done) {
            if (A != out) for (int i = tid; i < cur; i += T) out[i] = A[i];
            sc.sync();
            return cur;
        }
        for (int i = tid; i < cur; i += T) S[i] = A[i];
    } else {
        for (int i = tid; i < len; i += T) S[i] = p.bytes[b + i];
    }
    sc.sync();
    while (cur >= 2) {
        const int n = bound_pairs_pass_lds(p, S, R, QL, QR, (int32_t *)QL, cur, sc);
        if (n < 0) break;
        int32_t *t = S; S = (int32_t *)QL; QL = (uint32_t *)t;
        cur = n;
    }
    for (int i = tid; i < cur; i += T) out[i] = S[i];
    sc.sync();
    return cur;
}

template <typename Ptr>
__device__ __forceinline__ int encode_group_piece(const EncodeParams &p, int b, int len, Ptr A, Ptr B,
                                                  GroupTmp &tmp) {
    return encode_long_piece(p, b, len, A, B, GroupScope{tmp});
}

// One wavefront, buffers in its own LDS region (the 8 KiB of its lane-per-piece
// state, whose tokens must have been stored before): pieces of up to kWaveLdsMax symbols.
__device__ __forceinline__ int encode_wave_lds_piece(const EncodeParams &p, int b, int len, TinyState &L) {
    return encode_long_piece(p, b, len, (int32_t *)&L.S[0][0], (int32_t *)&L.R[0][0], WaveScope{});
}

// The paper's two kernels, kept for comparison (option paper_kernel): one
// workgroup per chunk, thread-strided pair evaluation with one lookup at a time,
// workgroup argmin, exactly one merge per pass, double-buffered compaction.
// variant 1 (section 3.4, baseline): chunks of at most one symbol per thread
// compact by a 0/1 "removed" flag and an exclusive prefix sum over the threads,
// longer ones by the shift; variant 2 (section 3.5, optimized): always the shift,
// i.e. symbols right of the merged pair move one slot to the left.
template <typename Ptr>
__device__ __forceinline__ int encode_chunk_paper(const EncodeParams &p, int b, int len, Ptr A, Ptr B, GroupTmp &tmp) {
    constexpr int T = kGroupThreads;
    const int tid = threadIdx.x;
    for (int i = tid; i < len; i += T) A[i] = p.bytes[b + i];
    __syncthreads();
    int cur = len;
    while (cur >= 2) {
        uint64_t best = ~0ull;
        for (int i = tid; i + 1 < cur; i += T) {
            uint32_t mm;
            const uint32_t r = table_find(p.table, (uint32_t)A[i], (uint32_t)A[i + 1], mm);
            if (r != kNoRank) best = min(best, ((uint64_t)(r & kRankMask) << 32) | (uint32_t)i);
        }
        best = group_min(best, tmp);
        if (best == ~0ull) break;
        const int best_pos = (int)(uint32_t)best;
        const int32_t merged = (int32_t)merged_id_of(p.table, (uint32_t)(best >> 32));
        if (p.paper == 1 && cur <= T) {
            const int removed = tid == best_pos + 1;
            int n_removed;
            const int before = group_scan_sum_excl(removed, tmp, n_removed);
            if (tid < cur && !removed) B[tid - before] = tid == best_pos ? merged : A[tid];
        } else {
            for (int i = tid; i < cur - 1; i += T)           // i = position in the new sequence
                B[i] = i == best_pos ? merged : A[i + (i > best_pos)];
        }
        __syncthreads();
        Ptr t = A; A = B; B = t;
        --cur;
    }
    int32_t *out = p.scratch + b;
    if ((const void *)A != (const void *)out) {
        for (int i = tid; i < cur; i += T) out[i] = A[i];
    }
    __syncthreads();
    return cur;
}

// LDS of a tile: the lane-per-piece state of the four wavefronts and the double
// buffer of the workgroup path share the same bytes; a barrier separates the two
// uses, and the lane-per-piece tokens are in the workspace by then.
union MergeLds {
    TinyState tiny[kWavesPerGroup];
    struct { int32_t A[kLdsMaxLen]; int32_t B[kLdsMaxLen]; } group;
};

struct TileShared {
    MergeLds lds;
    GroupTmp tmp;
    int list[kGroupThreads];       // threads whose piece waits for the wavefront paths, then for the workgroup path
    int list_n;
    int cnt_back[kGroupThreads];   // token counts handed back to the owning thread
};

struct TilePiece {                 // what a thread knows about its piece after merge_tile
    int64_t q;
    int o, len, cnt;
    int tok0;                      // several-kernel path: first token if known here, else -1 (it is in scratch)
    bool has_piece, is_tiny, parked;
    bool long_path;                // the workgroup path took the piece (its thread is on TileShared::list)
    uint32_t alive;                // lane-per-piece: positions of its LDS column that hold the tokens (unless parked)
};

// Merges every piece of tile `tile`.  Tokens of a piece end up at
// p.scratch[off[q] ...], except lane-per-piece tokens when `keep_in_lds` and no
// other path of this tile needed the LDS (then TilePiece::parked is false and
// they are still in the thread's LDS column).  Sets p.status[0] on bad offsets.
__device__ __forceinline__ const EncodeParams &kernel_params();
__device__ __forceinline__ TilePiece merge_tile_long_pieces(const EncodeParams &p, TileShared &sh, TilePiece t,
                                                            int64_t tile_q0, int P, bool is_wave, bool is_long);

// n_pieces, P: the piece count and the pieces per wavefront of this launch (p's own
// values, except on the raw path, where the kernel finds them out).
__device__ __forceinline__ TilePiece merge_tile(const EncodeParams &p, TileShared &sh, int tile, bool keep_in_lds,
                                                int n_pieces, int P) {
    const int tid = threadIdx.x, lane = lane_id(), wv = tid / kWave;
    if (p.paper) {                 // the tile is piece number `tile`, merged by the paper's kernel
        TilePiece t = {};
        t.q = tile;
        t.parked = true;
        int o = 0, len = 0;
        if (tile < n_pieces) {
            o = p.off[tile];
            const int o_next = p.off[tile + 1];
            const bool bad = o < 0 || o_next < o || o_next > p.n_bytes || (tile == 0 && o != 0) ||
                             (tile == n_pieces - 1 && o_next != p.n_bytes);
            if (bad && tid == 0)
                __hip_atomic_store(&p.status[0], p.call_id, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            len = bad ? 0 : o_next - o;
        }
        o = __builtin_amdgcn_readfirstlane(o);
        len = __builtin_amdgcn_readfirstlane(len);
        int c = 0;
        if (len > 0 && len <= p.lds_max) c = encode_chunk_paper<int32_t *>(p, o, len, sh.lds.group.A, sh.lds.group.B, sh.tmp);
        else if (len > 0) c = encode_chunk_paper<int32_t *>(p, o, len, p.scratch + o, p.scratch2 + o, sh.tmp);
        t.has_piece = tid == 0 && tile < n_pieces;
        t.o = o;
        t.len = len;
        t.cnt = tid == 0 ? c : 0;
        t.tok0 = -1;
        return t;
    }
    if (tid == 0) sh.list_n = 0;
    TilePiece t;
    const int64_t tile_q0 = (int64_t)tile * p.W * P;
    t.q = tile_q0 + (int64_t)wv * P + lane;
    t.has_piece = lane < P && wv < p.W && t.q < n_pieces;
    t.o = 0;
    t.len = 0;
    bool bad = false;
    if (t.has_piece) {
        t.o = p.off[t.q];
        const int o_next = p.off[t.q + 1];
        bad = t.o < 0 || o_next < t.o || o_next > p.n_bytes;
        bad |= (t.q == 0 && t.o != 0) || (t.q == n_pieces - 1 && o_next != p.n_bytes);
        t.len = bad ? 0 : o_next - t.o;
    }
    if (__ballot(bad) && lane == 0)
        __hip_atomic_store(&p.status[0], p.call_id, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    t.is_tiny = t.has_piece && t.len > 0 && t.len <= p.tiny_max;
    t.long_path = false;
    const bool is_wave = t.has_piece && t.len > p.tiny_max && t.len <= p.wave_lds_max;
    const bool is_long = t.has_piece && t.len > p.wave_lds_max;

    // lane-per-piece path
    t.alive = tiny_merge(p, sh.lds.tiny[wv], t.o, t.len, t.is_tiny);
    t.cnt = __builtin_popcount(t.alive);
    t.parked = !keep_in_lds;
    t.tok0 = -1;
    if (t.parked) {
        // The first token travels with the count (one coalesced 8-byte record per piece);
        // only the pieces of two or more tokens, few in word-like text, touch scratch.
        if (t.alive) t.tok0 = (int)(sh.lds.tiny[wv].S[__builtin_ctz(t.alive)][lane] & 0xFFFFFFu);
        tiny_store(sh.lds.tiny[wv], t.alive & (t.alive - 1), p.scratch + t.o + 1);
    }

    // Everything else is rare in word-like text: one barrier finds out whether the tile has any.
    if (__syncthreads_count(is_wave || is_long) == 0) return t;
    return merge_tile_long_pieces(kernel_params(), sh, t, tile_q0, P, is_wave, is_long);
}

// The kernel's parameter block as it lies in the kernel-argument segment (every kernel
// that merges takes EncodeParams as its first parameter).  The rare paths read their
// parameters from there when they get to them, so that the registers of the common
// path above do not have to hold them: with the parameters passed down by reference the
// compiler kept them all live from the start of the kernel and spilled dozens of them.
__device__ __forceinline__ const EncodeParams &kernel_params() {
    return *(const EncodeParams *)__builtin_amdgcn_kernarg_segment_ptr();
}

// Second half of merge_tile: the wavefront and workgroup paths of the tile's longer pieces.
// P: pieces per wavefront of this launch (on the raw path the kernel may have chosen it).
__device__ __forceinline__ TilePiece merge_tile_long_pieces(const EncodeParams &p, TileShared &sh, TilePiece t,
                                                            int64_t tile_q0, int P, bool is_wave, bool is_long) {
    const int tid = threadIdx.x, lane = lane_id(), wv = tid / kWave;
    if (!t.parked) {               // the other paths reuse the LDS of the lane-per-piece state
        tiny_store(sh.lds.tiny[wv], t.alive, p.scratch + t.o);
        t.parked = true;
    }

    // Wavefront paths.  The tile's wavefronts share these pieces through a list in
    // LDS, so that a wavefront that owns several of them does not become the tail.
    if (is_wave) sh.list[atomicAdd(&sh.list_n, 1)] = tid;
    __syncthreads();
    // Entry e goes to wavefront e mod 4.  Everything that steers the loop is made
    // wave-uniform explicitly: a lane-0-only atomic ticket followed by readfirstlane
    // compiled into a loop in which the other 63 lanes kept re-reading their own
    // initial value of the ticket and never left.
    const int n_work = __builtin_amdgcn_readfirstlane(sh.list_n);
    for (int e = __builtin_amdgcn_readfirstlane(wv); e < n_work; e += kWavesPerGroup) {
        const int owner = __builtin_amdgcn_readfirstlane(sh.list[e]);
        const int64_t wq = tile_q0 + (int64_t)(owner / kWave) * P + (owner % kWave);
        const int b = __builtin_amdgcn_readfirstlane(p.off[wq]);      // validated by the owner
        const int n = __builtin_amdgcn_readfirstlane(p.off[wq + 1]) - b;
        int c;
        if (n <= p.wave_max) c = encode_wave_piece(p, b, n);
        else if (p.level >= 3 && !(p.runs_by_best_rank && piece_is_run_like(p, b, n, WaveScope{})))
            // well beyond what a wavefront keeps resident the whole workgroup is quicker (1,024 bytes
            // of text: 148 us against 272 us for one wavefront working through windows; even at 600)
            // (and at once when the piece has the workgroup to itself)
            c = n <= (p.W == 1 ? kWaveBoundMax : kWaveBoundHandOn)
                    ? encode_long_piece_bound(p, b, n, &sh.lds.tiny[wv].S[0][0], kWaveBoundMax, WaveScope{})
                    : kLongMark;
        else c = encode_wave_lds_piece(p, b, n, sh.lds.tiny[wv]);
        if (lane == 0) sh.cnt_back[owner] = c;
    }
    __syncthreads();
    if (is_wave) {
        t.cnt = sh.cnt_back[tid];
        if (t.cnt == kLongMark) { t.cnt = 0; is_long = true; }     // handed on to the workgroup path
    }
    t.long_path = is_long;

    // Workgroup path, one piece at a time by all threads.
    if (tid == 0) sh.list_n = 0;
    __syncthreads();
    if (is_long) sh.list[atomicAdd(&sh.list_n, 1)] = tid;
    __syncthreads();
    const int n_long = __builtin_amdgcn_readfirstlane(sh.list_n);
    for (int e = 0; e < n_long; ++e) {
        const int owner = __builtin_amdgcn_readfirstlane(sh.list[e]);
        const int64_t lq = tile_q0 + (int64_t)(owner / kWave) * P + (owner % kWave);
        const int b = __builtin_amdgcn_readfirstlane(p.off[lq]);      // validated by the owner
        const int n = __builtin_amdgcn_readfirstlane(p.off[lq + 1]) - b;
        int c;
        if (p.level >= 3 && !(p.runs_by_best_rank && piece_is_run_like(p, b, n, GroupScope{sh.tmp})))
            c = encode_long_piece_bound(p, b, n, (uint32_t *)sh.lds.group.A,
                                        min(max(p.lds_max, kGroupBoundMin), kGroupBoundMax), GroupScope{sh.tmp});
        else if (n <= p.lds_max) c = encode_group_piece<int32_t *>(p, b, n, sh.lds.group.A, sh.lds.group.B, sh.tmp);
        else c = encode_group_piece<int32_t *>(p, b, n, p.scratch + b, p.scratch2 + b, sh.tmp);
        if (tid == owner) t.cnt = c;
    }
    return t;
}

// Raw path: the piece count the pre-tokenizer left on the device, kept within the
// capacity the grid and the workspace were sized for.
__device__ inline int device_piece_count(const EncodeParams &p) {
    return min(max(__builtin_amdgcn_readfirstlane(*p.n_pieces_dev), 0), p.n_pieces);
}

// Raw path, at the start of every kernel that works by tiles: the piece count the
// pre-tokenizer found, and, if the caller left it open, the pieces per wavefront: 64
// for word-sized pieces, as few as the host's choice for longer ones (as many tiles as
// possible: pieces that take a wavefront each hide each other's latency), but never
// more tiles than the capacity-sized grids and arrays of the host provide for.  Every
// kernel of a call derives the same values from the same two numbers.
__device__ inline void raw_geometry(EncodeParams &p) {
    const int tiles_bound = max((p.n_pieces + p.W * p.P - 1) / (p.W * p.P), 1);
    p.n_pieces = device_piece_count(p);
    if (!p.raw_auto_P) return;
    const int avg = p.n_pieces > 0 ? p.n_bytes / p.n_pieces : 1;
    if (avg <= kTinyMax) return;
    const int wanted = max(min(p.n_pieces / 4096, (kWave * kTinyMax) / avg), 1);
    const int needed = (p.n_pieces + p.W * tiles_bound - 1) / (p.W * tiles_bound);
    p.P = min(max(wanted, needed), kWave);
}

__device__ inline int tiles_of(const EncodeParams &p) {
    const int per_tile = p.W * p.P;
    return (p.n_pieces + per_tile - 1) / per_tile;
}

// Several-kernel path, first kernel: tokens and counts of every piece to the
// workspace, the tile's token total to tile_sum.
__device__ __forceinline__ void merge_and_count_tile(const EncodeParams &p, TileShared &sh, int *wave_tokens, int tile,
                                                     int n_pieces, int P) {
    const TilePiece t = merge_tile(p, sh, tile, false, n_pieces, P);
    if (t.has_piece) p.rec[t.q] = make_int2(t.cnt, t.tok0);
    int wave_total = t.cnt;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) wave_total += __shfl_xor(wave_total, d);
    if (lane_id() == 0) wave_tokens[threadIdx.x / kWave] = wave_total;
    __syncthreads();
    if (threadIdx.x == 0) {
        int sum = 0;
        for (int w = 0; w < kWavesPerGroup; ++w) sum += wave_tokens[w];
        p.tile_sum[tile] = sum;
    }
}

__global__ void __launch_bounds__(kGroupThreads) merge_kernel(EncodeParams p) {
    __shared__ TileShared sh;
    __shared__ int wave_tokens[kWavesPerGroup];
    merge_and_count_tile(p, sh, wave_tokens, blockIdx.x, p.n_pieces, p.P);
}

// Raw path: the grids are sized on the host without knowing the piece count.  This
// kernel takes the first gridDim.x tiles, one per workgroup (a workgroup beyond the
// tiles that exist returns at once); merge_raw_rest_kernel strides over the others.
// Two kernels because the loop around the tile costs the common path a tenth of its
// speed (its registers must survive the loop: 90 spilled scalar registers).
__global__ void __launch_bounds__(kGroupThreads) merge_raw_kernel(EncodeParams p) {
    __shared__ TileShared sh;
    __shared__ int wave_tokens[kWavesPerGroup];
    raw_geometry(p);
    if ((int)blockIdx.x < tiles_of(p)) merge_and_count_tile(p, sh, wave_tokens, blockIdx.x, p.n_pieces, p.P);
}

__global__ void __launch_bounds__(kGroupThreads) merge_raw_rest_kernel(EncodeParams p, int first_tile) {
    __shared__ TileShared sh;
    __shared__ int wave_tokens[kWavesPerGroup];
    raw_geometry(p);
    const int n_tiles = tiles_of(p);
    for (int tile = first_tile + blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        merge_and_count_tile(p, sh, wave_tokens, tile, p.n_pieces, p.P);
        __syncthreads();   // the next tile reuses the LDS
    }
}

// ---------------------------------------------------------------------------
// Single-kernel path: the merge phase of merge_kernel followed, in the same
// workgroup, by the ordered assembly of the output.  A tile publishes its token
// total, finds the number of tokens of all tiles before it by decoupled
// look-back over the published totals, and stores its tokens straight from LDS
// to their final place.
constexpr int kFusedMaxTiles = 256;

__global__ void __launch_bounds__(kGroupThreads) encode_kernel(EncodeParams p, int n_tiles) {
    __shared__ TileShared sh;
    __shared__ LookbackTmp lb;
    __shared__ int long_src, long_dst, long_cnt;
    const int tid = threadIdx.x, lane = lane_id(), wv = tid / kWave;
    const int tile = blockIdx.x;
    if (tile == 0 && tid == 0) p.status[2] = p.call_id;    // the call the other status words refer to

    const TilePiece t = merge_tile(p, sh, tile, true, p.n_pieces, p.P);
    const bool has_piece = t.has_piece, is_tiny = t.is_tiny, parked = t.parked;
    const int o = t.o, my_cnt = t.cnt;
    const int64_t q = t.q;
    const uint32_t alive = t.alive;
    const bool is_long = t.long_path;
    const bool is_wave = has_piece && t.len > p.tiny_max && !is_long;

    // position of every piece's tokens in the output
    int total;
    const int ex = group_scan_sum_excl(my_cnt, sh.tmp, total);
    const int base = total_before_tile(p.tile_state, p.status, p.call_id, p.status + kStatusEpochEncode, tile, n_tiles,
                                       total, lb);
    const int first = base + ex;
    if (has_piece) p.out_offsets[q] = first;
    if (tid == 0 && tile == n_tiles - 1) p.out_offsets[p.n_pieces] = base + total;
    // bad offsets can make pieces overlap and the total exceed the capacity of out_ids
    const int room = first >= 0 && first < p.n_bytes ? p.n_bytes - first : 0;
    const int n_store = min(my_cnt, room);

    if (!parked) {
        tiny_store(sh.lds.tiny[wv], is_tiny && n_store == my_cnt ? alive : 0u, p.out_ids + first);
    } else if (is_tiny) {
        for (int i = 0; i < n_store; ++i) p.out_ids[first + i] = p.scratch[o + i];
    }
    for (uint64_t m = __ballot(is_wave); m;) {             // tokens of the wavefront paths: from the workspace
        const int w = __builtin_ctzll(m);
        m &= m - 1;
        const int src = read_lane(o, w), dst = read_lane(first, w), c = read_lane(n_store, w);
        for (int i = lane; i < c; i += kWave) p.out_ids[dst + i] = p.scratch[src + i];
    }
    const int any_long = __syncthreads_count(is_long);
    for (int e = 0; e < any_long; ++e) {                   // tokens of workgroup-path pieces: all threads copy
        __syncthreads();
        if (is_long && tid == sh.list[e]) { long_src = o; long_dst = first; long_cnt = n_store; }
        __syncthreads();
        const int src = long_src, dst = long_dst, c = long_cnt;
        for (int i = tid; i < c; i += kGroupThreads) p.out_ids[dst + i] = p.scratch[src + i];
    }
}

// ---------------------------------------------------------------------------
// Assembly on the device: exclusive scan of the tile totals by one workgroup.
constexpr int kScanThreads = 1024;
constexpr int kScanSpan = 8192;        // tile totals per workgroup of scan_tiles_kernel
constexpr int kSelfScanTiles = 2048;   // up to here emit_kernel adds up the tile totals itself

__global__ void __launch_bounds__(kScanThreads) scan_tiles_kernel(EncodeParams p, int64_t n_tiles) {
    __shared__ LookbackTmp lb;
    __shared__ int wave_sum[kScanThreads / kWave];
    const int tid = threadIdx.x, lane = lane_id(), wv = tid / kWave;
    if (p.n_pieces_dev) {          // raw path: only the tiles that exist; small grids add up by themselves in emit_kernel
        raw_geometry(p);
        n_tiles = tiles_of(p);
        if (n_tiles <= kSelfScanTiles) return;
    }
    // A workgroup of 1024 threads covers kScanSpan totals: a thread adds up 8
    // consecutive ones (two 16-byte loads), the thread sums are scanned, the
    // workgroups hand their totals on by look-back, and the thread writes its 8 bases.
    const int n_groups = max((int)((n_tiles + kScanSpan - 1) / kScanSpan), 1);
    const int group = blockIdx.x;
    if (group >= n_groups) return;                // raw path: the grid was sized for the capacity
    constexpr int kPerThread = kScanSpan / kScanThreads;
    const int64_t i0 = (int64_t)group * kScanSpan + (int64_t)tid * kPerThread;
    int v[kPerThread];
    if (i0 + kPerThread <= n_tiles) {             // tile_sum is 256-byte aligned and i0 a multiple of 8
#pragma unroll
        for (int j = 0; j < kPerThread; j += 4) {
            const int4 a = *(const int4 *)(p.tile_sum + i0 + j);
            v[j] = a.x; v[j + 1] = a.y; v[j + 2] = a.z; v[j + 3] = a.w;
        }
    } else {
#pragma unroll
        for (int j = 0; j < kPerThread; ++j) v[j] = i0 + j < n_tiles ? p.tile_sum[i0 + j] : 0;
    }
    int mine = 0;
#pragma unroll
    for (int j = 0; j < kPerThread; ++j) mine += v[j];
    int inc = mine;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const int o = __shfl_up(inc, d);
        if (lane >= d) inc += o;
    }
    if (lane == kWave - 1) wave_sum[wv] = inc;
    __syncthreads();
    int ex = inc - mine, total = 0;
    for (int w = 0; w < kScanThreads / kWave; ++w) {
        if (w < wv) ex += wave_sum[w];
        total += wave_sum[w];
    }
    // tile_state and the launch counter of the single-kernel path are free: that path is not taken in this call
    int before = 0;
    if (n_groups > 1)
        before = total_before_tile<1, kGroupThreads, kScanThreads / kWave>(
            p.tile_state, p.status, p.call_id, p.status + kStatusEpochEncode, group, n_groups, total, lb);
    ex += before;
#pragma unroll
    for (int j = 0; j < kPerThread; ++j) {
        if (i0 + j < n_tiles) p.tile_base[i0 + j] = ex;
        ex += v[j];
    }
    if (tid == 0 && group == n_groups - 1) {
        p.out_offsets[p.n_pieces] = before + total;
        p.status[2] = p.call_id;
    }
}

// out_offsets of the tile's pieces and the dense copy of their tokens.  With
// self_scan the tile adds up the totals of all tiles before it by itself (for a
// grid of up to kSelfScanTiles tiles that costs less than a scan kernel launch).

__device__ __forceinline__ void emit_tile(const EncodeParams &p, GroupTmp &tmp, int *before_w, int tile, int last_tile,
                                          int self_scan) {
    const int tid = threadIdx.x, lane = lane_id(), wv = tid / kWave;
    int base;
    if (self_scan) {
        int before = 0;
        for (int t = tid; t < tile; t += kGroupThreads) before += p.tile_sum[t];
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) before += __shfl_xor(before, d);
        if (lane == 0) before_w[wv] = before;
        __syncthreads();
        base = 0;
        for (int w = 0; w < kWavesPerGroup; ++w) base += before_w[w];
    } else {
        base = p.tile_base[tile];
    }
    // pieces of the tile; the paper's kernels have one piece per tile
    const int64_t q = p.paper ? tile : ((int64_t)tile * p.W + wv) * p.P + lane;
    const bool has_piece = (p.paper ? tid == 0 : (lane < p.P && wv < p.W)) && q < p.n_pieces;
    int c = 0, o = 0, tok0 = -1;
    if (has_piece) { const int2 r = p.rec[q]; c = r.x; tok0 = r.y; }
    if (c < 0) c = 0;
    if (c > 1 || (c == 1 && tok0 < 0)) o = p.off[q];     // only then is anything of the piece in scratch
    int total;
    const int ex = group_scan_sum_excl(c, tmp, total);
    const int first = base + ex;
    if (has_piece) p.out_offsets[q] = first;
    if (self_scan && tid == 0) {
        if (tile == last_tile) p.out_offsets[p.n_pieces] = base + total;
        if (tile == 0) p.status[2] = p.call_id;
    }
    // bad offsets can make pieces overlap and the total exceed the capacity of out_ids;
    // then they must still not become bad addresses
    const int room = first >= 0 && first < p.n_bytes ? p.n_bytes - first : 0;
    const int src_room = o >= 0 && o < p.n_bytes ? p.n_bytes - o : 0;
    const int n_copy = min(c, min(room, src_room));
    // most pieces are one or two tokens: each thread copies the first 8 of its own
    // piece, the wavefront shares the rest of the rare longer ones
    if (n_copy > 0) p.out_ids[first] = tok0 >= 0 ? tok0 : p.scratch[o];
    for (int i = 1; i < 8; ++i) {
        if (!__ballot(i < n_copy)) break;
        if (i < n_copy) p.out_ids[first + i] = p.scratch[o + i];
    }
    for (uint64_t m = __ballot(n_copy > 8); m;) {
        const int t = __builtin_ctzll(m);
        m &= m - 1;
        const int src = read_lane(o, t), dst = read_lane(first, t), n = read_lane(n_copy, t);
        for (int i = 8 + lane; i < n; i += kWave) p.out_ids[dst + i] = p.scratch[src + i];
    }
}

__global__ void __launch_bounds__(kGroupThreads) emit_kernel(EncodeParams p, int self_scan) {
    __shared__ GroupTmp tmp;
    __shared__ int before_w[kWavesPerGroup];
    emit_tile(p, tmp, before_w, blockIdx.x, gridDim.x - 1, self_scan);
}

// Raw path: workgroups stride over the tiles that exist (tile 0 always does: it
// also reports "no piece at all").
__global__ void __launch_bounds__(kGroupThreads) emit_raw_kernel(EncodeParams p) {
    __shared__ GroupTmp tmp;
    __shared__ int before_w[kWavesPerGroup];
    raw_geometry(p);
    const int n_tiles = tiles_of(p);
    const int last_tile = max(n_tiles, 1) - 1;
    const int self_scan = n_tiles <= kSelfScanTiles;
    for (int tile = blockIdx.x; tile <= last_tile; tile += gridDim.x) {
        emit_tile(p, tmp, before_w, tile, last_tile, self_scan);
        __syncthreads();   // the next tile reuses the LDS
    }
}

// Raw path, last kernel: the first token of every sequence.
__global__ void __launch_bounds__(kGroupThreads) seq_token_offsets_kernel(EncodeParams p) {
    const int n_pieces = device_piece_count(p);
    const int k = blockIdx.x * kGroupThreads + threadIdx.x;
    if (k <= p.n_seqs) p.seq_token_offsets[k] = p.out_offsets[min(max(p.seq_first_piece[k], 0), n_pieces)];
}

struct Layout {
    int64_t status, rec, tile_sum, tile_base, tile_state, scratch, scratch2, total;
};

static int64_t align256(int64_t v) { return (v + 255) & ~255ll; }

static Layout workspace_layout(int64_t n_bytes, int64_t n_pieces) {
    Layout l;
    const int64_t max_tiles = n_pieces + 1;      // a tile can be a single piece
    int64_t at = 0;
    l.status = at;    at += 256;
    l.rec = at;       at += align256(8 * (n_pieces + 1));
    l.tile_sum = at;  at += align256(4 * (n_pieces + 1));   // the paper's kernels have one piece per tile
    l.tile_base = at; at += align256(4 * (n_pieces + 1));
    l.tile_state = at; at += align256(8 * max_tiles);
    l.scratch = at;   at += align256(4 * (n_bytes + 1));
    l.scratch2 = at;  at += align256(4 * (n_bytes + 1));
    l.total = at;
    return l;
}

// Raw path: the encode layout for max_pieces pieces, then what the pre-tokenizer
// needs and the piece arrays the caller did not bring.
struct RawLayout {
    Layout enc;
    int64_t pretok_state, seq_first_piece, piece_offsets, out_offsets, n_pieces, total;
};

static RawLayout raw_layout(int64_t n_bytes, int64_t max_pieces, int64_t n_seqs) {
    RawLayout r;
    r.enc = workspace_layout(n_bytes, max_pieces);
    int64_t at = r.enc.total;
    r.pretok_state = at;    at += align256(pretokenize_state_bytes(n_bytes));
    r.seq_first_piece = at; at += align256(4 * (n_seqs + 2));
    r.piece_offsets = at;   at += align256(4 * (max_pieces + 1));
    r.out_offsets = at;     at += align256(4 * (max_pieces + 1));
    r.n_pieces = at;        at += 256;
    r.total = at;
    return r;
}

static std::atomic<int32_t> g_call_id{1};

int32_t next_call_id() {
    int32_t id;
    do {
        const uint32_t n = (uint32_t)g_call_id.fetch_add(1);
        id = (int32_t)((n * 0x9E3779B1u) ^ 0x7F4A7C15u);
    } while ((id & 0x3FFFFFFF) == 0);
    return id;
}

}  // namespace bpe

using namespace bpe;

extern "C" int64_t bpe_workspace_bytes(int64_t n_bytes, int64_t n_pieces) {
    if (n_bytes < 0 || n_pieces < 0 || n_bytes >= 0x7FFFFFFFll || n_pieces >= 0x7FFFFFFFll) {
        set_error("sizes out of range (n_bytes %lld, n_pieces %lld)", (long long)n_bytes, (long long)n_pieces);
        return BPE_ERR_SIZE;
    }
    return workspace_layout(n_bytes, n_pieces).total;
}

extern "C" int64_t bpe_encode_raw_workspace_bytes(int64_t n_bytes, int64_t max_pieces, int64_t n_seqs) {
    if (max_pieces == 0) max_pieces = n_bytes;
    if (n_bytes < 0 || max_pieces < 0 || n_seqs < 0 || n_bytes >= 0x7FFFFFFFll || max_pieces >= 0x7FFFFFFFll ||
        n_seqs >= 0x7FFFFFFFll) {
        set_error("sizes out of range (n_bytes %lld, max_pieces %lld, n_seqs %lld)", (long long)n_bytes,
                  (long long)max_pieces, (long long)n_seqs);
        return BPE_ERR_SIZE;
    }
    return raw_layout(n_bytes, max_pieces, n_seqs).total;
}

// What the raw path adds to the arguments of bpe_encode: the pieces are found on
// the device first, so n_pieces of launch_encode is only their capacity.
struct RawArgs {
    const int32_t *seq_offsets;
    int64_t n_seqs;
    int32_t *seq_token_offsets;
    int32_t *piece_offsets;   // nullptr: kept in the workspace
    int32_t *out_offsets;     // nullptr: kept in the workspace
    int32_t *n_pieces;        // nullptr: kept in the workspace
};

// Validates, fills the kernel parameters and enqueues the kernels.  With `ev` an
// event is recorded before the first kernel and after each: kKernels + 1 events,
// kRawKernels + 1 on the raw path.
constexpr int kKernels = 3;
constexpr int kRawKernels = 5;
constexpr int64_t kRawMaxGrid = 8192;   // raw path: workgroups of the merge and emit kernels
constexpr int64_t kRawRestGrid = 2048;  // ... of the strided merge kernel (two rounds of the chip; mostly it finds nothing to do)

static int launch_encode(const bpe_table *table, const uint8_t *bytes, const int32_t *piece_offsets,
                         int64_t n_bytes, int64_t n_pieces, int32_t *out_ids, int32_t *out_offsets,
                         void *workspace, int64_t workspace_bytes, const bpe_encode_options *opts,
                         hipStream_t s, hipEvent_t *ev, const RawArgs *raw = nullptr) {
    if (!table || (n_bytes > 0 && (!bytes || !out_ids)) ||
        (raw ? !raw->seq_token_offsets : (!piece_offsets || !out_offsets))) {
        set_error("null pointer");
        return BPE_ERR_NULL;
    }
    const int64_t need = raw ? bpe_encode_raw_workspace_bytes(n_bytes, n_pieces, raw->n_seqs)
                             : bpe_workspace_bytes(n_bytes, n_pieces);
    if (need < 0) return (int)need;
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < need) {
        set_error("workspace must be 256-byte aligned and hold %lld bytes (got %lld)", (long long)need,
                  (long long)workspace_bytes);
        return BPE_ERR_WORKSPACE;
    }
    bpe_encode_options o = {};
    if (opts) o = *opts;
    const bool raw_auto_P = raw && o.pieces_per_wave == 0;
    if (raw_auto_P) o.pieces_per_wave = kWave;   // the average piece length is not known yet: the kernels choose
    const bool auto_level = o.selection_level == 0;
    if (auto_level) o.selection_level = 3;
    if (o.tiny_max_len == 0) o.tiny_max_len = kTinyMax;
    if (o.wave_max_len == 0) o.wave_max_len = kWave;
    if (o.wave_lds_max_len == 0) o.wave_lds_max_len = kWaveLdsMax;
    if (o.lds_max_len == 0) o.lds_max_len = kLdsMaxLen;
    if (o.pieces_per_wave == 0) {
        // One piece per lane while pieces are short on average.  Longer pieces take a
        // whole wavefront or workgroup each, one after the other: then as few pieces per
        // wavefront as still leave a few thousand workgroups (they hide each other's
        // lookup latency), and one piece per workgroup once pieces are workgroup-sized.
        const int64_t avg = n_pieces > 0 ? n_bytes / n_pieces : 1;
        int64_t ppw = kWave;
        if (avg >= (o.selection_level >= 3 ? kWaveBoundHandOn : kWaveLdsMax + 1)) ppw = -1;
        else if (avg > kTinyMax) ppw = std::max<int64_t>(std::min<int64_t>(n_pieces / 4096, (kWave * kTinyMax) / avg), 1);
        o.pieces_per_wave = (int32_t)ppw;
    }
    if (o.selection_level < 1 || o.selection_level > 3 || o.pieces_per_wave < -1 || o.pieces_per_wave == 0 || o.pieces_per_wave > kWave ||
        o.tiny_max_len < -1 || o.tiny_max_len > kTinyMax || o.wave_max_len < -1 || o.wave_max_len > kWave ||
        o.wave_lds_max_len < -1 || o.wave_lds_max_len > kWaveLdsMax ||
        o.lds_max_len < 1 || o.lds_max_len > kLdsMaxLen || o.fused < -1 || o.fused > 1 ||
        !pretokenize_tile_ok(o.pretokenize_tile_kib) || o.paper_kernel < 0 || o.paper_kernel > 2 ||
        (o.paper_kernel && raw)) {
        set_error("option out of range");
        return BPE_ERR_OPTION;
    }
    if (o.tiny_max_len < 0) o.tiny_max_len = 0;      // -1 switches a path off
    if (o.wave_max_len < 0) o.wave_max_len = 0;
    if (o.wave_lds_max_len < 0) o.wave_lds_max_len = 0;

    const int dev_rc = check_device(table->device, "the table");
    if (dev_rc != BPE_OK) return dev_rc;
    const Layout l = workspace_layout(n_bytes, n_pieces);
    char *ws = (char *)workspace;
    EncodeParams p = {};     // no kernel parameter is ever left unset
    p.call_id = next_call_id();
    int n_ev = 0;
    if (ev) (void)hipEventRecord(ev[n_ev++], s);
    if (raw) {
        const RawLayout r = raw_layout(n_bytes, n_pieces, raw->n_seqs);
        int32_t *piece_off = raw->piece_offsets ? raw->piece_offsets : (int32_t *)(ws + r.piece_offsets);
        int32_t *n_dev = raw->n_pieces ? raw->n_pieces : (int32_t *)(ws + r.n_pieces);
        int32_t *first = (int32_t *)(ws + r.seq_first_piece);
        if (!out_offsets) out_offsets = (int32_t *)(ws + r.out_offsets);
        const int rc = launch_pretokenize(bytes, n_bytes, raw->seq_offsets, raw->n_seqs, piece_off, n_pieces, n_dev,
                                          first, (int32_t *)(ws + l.status),
                                          (unsigned long long *)(ws + r.pretok_state), p.call_id,
                                          o.pretokenize_tile_kib, s);
        if (rc != BPE_OK) return rc;
        if (ev) (void)hipEventRecord(ev[n_ev++], s);
        piece_offsets = piece_off;
        p.n_pieces_dev = n_dev;
        p.seq_first_piece = first;
        p.seq_token_offsets = raw->seq_token_offsets;
        p.n_seqs = raw->seq_offsets ? (int32_t)raw->n_seqs : 1;
    }
    p.table = table->view;
    p.bytes = bytes;
    p.off = piece_offsets;
    p.n_bytes = (int32_t)n_bytes;
    p.n_pieces = (int32_t)n_pieces;
    p.P = o.pieces_per_wave > 0 ? o.pieces_per_wave : 1;
    p.W = o.pieces_per_wave > 0 ? kWavesPerGroup : 1;
    p.raw_auto_P = raw_auto_P;
    p.tiny_max = o.tiny_max_len;
    p.wave_max = std::max(o.wave_max_len, o.tiny_max_len);
    p.wave_lds_max = std::max(o.wave_lds_max_len, p.wave_max);
    p.lds_max = o.lds_max_len;
    p.level = o.selection_level;
    p.runs_by_best_rank = auto_level;
    p.paper = o.paper_kernel;
    p.rec = (int2 *)(ws + l.rec);
    p.tile_sum = (int32_t *)(ws + l.tile_sum);
    p.tile_base = (int32_t *)(ws + l.tile_base);
    p.scratch = (int32_t *)(ws + l.scratch);
    p.scratch2 = (int32_t *)(ws + l.scratch2);
    p.status = (int32_t *)(ws + l.status);
    p.tile_state = (unsigned long long *)(ws + l.tile_state);
    p.out_ids = out_ids;
    p.out_offsets = out_offsets;

    const int64_t per_tile = p.paper ? 1 : (int64_t)p.P * p.W;
    const int64_t n_tiles = (n_pieces + per_tile - 1) / per_tile;
    // One kernel while the grid is a single look-back window deep (256 tiles): it
    // saves a launch (11.2 vs 13.2 us on 3 tiles, 12.7 vs 13.7 us on 124).  Beyond
    // that the waiting costs as much as the launch (16.4 vs 16.2 us on 494 tiles),
    // and on deep grids a tile that waits keeps its LDS from the next tile (208 vs
    // 141 us on 7944 tiles).
    // ... and only while pieces are short on average: a tile that waits for its
    // predecessors gives up after a bounded time (about two seconds), and tiles that merge
    // kilobyte-long pieces one merge at a time hold their successors up for that long.
    const bool short_pieces = n_bytes <= n_pieces * (int64_t)kWave;
    const bool fused = !raw && !p.paper && n_tiles > 0 &&
                       (o.fused > 0 || (o.fused == 0 && n_tiles <= kFusedMaxTiles && short_pieces));
    if (fused) {
        hipLaunchKernelGGL(encode_kernel, dim3((unsigned)n_tiles), dim3(kGroupThreads), 0, s, p, (int)n_tiles);
        if (ev) { (void)hipEventRecord(ev[1], s); (void)hipEventRecord(ev[2], s); (void)hipEventRecord(ev[3], s); }
    } else {
        // Raw path: n_tiles only bounds the tile count.  A capped grid strides over the
        // tiles that exist (at least one workgroup, which also handles "no piece at all").
        const int64_t grid = raw ? std::min<int64_t>(std::max<int64_t>(n_tiles, 1), kRawMaxGrid) : n_tiles;
        if (raw) {
            // one tile per workgroup for as many tiles as are likely to exist (an eighth of
            // the capacity-sized bound, at least kRawMaxGrid), a strided kernel for the rest
            const int64_t direct = std::min<int64_t>(std::max<int64_t>(n_tiles, 1), std::max<int64_t>(kRawMaxGrid, n_tiles / 8));
            hipLaunchKernelGGL(merge_raw_kernel, dim3((unsigned)direct), dim3(kGroupThreads), 0, s, p);
            if (n_tiles > direct)
                hipLaunchKernelGGL(merge_raw_rest_kernel, dim3((unsigned)std::min<int64_t>(n_tiles - direct, kRawRestGrid)),
                                   dim3(kGroupThreads), 0, s, p, (int)direct);
        } else if (grid > 0) {
            hipLaunchKernelGGL(merge_kernel, dim3((unsigned)grid), dim3(kGroupThreads), 0, s, p);
        }
        if (ev) (void)hipEventRecord(ev[n_ev++], s);
        const int self_scan = n_tiles > 0 && n_tiles <= kSelfScanTiles;
        if (!self_scan && !(raw && n_tiles == 0))
            hipLaunchKernelGGL(scan_tiles_kernel, dim3((unsigned)std::max<int64_t>((n_tiles + kScanSpan - 1) / kScanSpan, 1)),
                               dim3(kScanThreads), 0, s, p, n_tiles);
        if (ev) (void)hipEventRecord(ev[n_ev++], s);
        if (raw) hipLaunchKernelGGL(emit_raw_kernel, dim3((unsigned)grid), dim3(kGroupThreads), 0, s, p);
        else if (grid > 0) hipLaunchKernelGGL(emit_kernel, dim3((unsigned)grid), dim3(kGroupThreads), 0, s, p, self_scan);
        if (ev) (void)hipEventRecord(ev[n_ev++], s);
        if (raw) {
            const unsigned g = (unsigned)((p.n_seqs + 1 + kGroupThreads - 1) / kGroupThreads);
            hipLaunchKernelGGL(seq_token_offsets_kernel, dim3(g), dim3(kGroupThreads), 0, s, p);
            if (ev) (void)hipEventRecord(ev[n_ev++], s);
        }
    }
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? BPE_OK : hip_fail(e, "bpe_encode launch");
}

extern "C" int bpe_encode(const bpe_table *table, const uint8_t *bytes, const int32_t *piece_offsets,
                          int64_t n_bytes, int64_t n_pieces, int32_t *out_ids, int32_t *out_offsets,
                          void *workspace, int64_t workspace_bytes, const bpe_encode_options *opts,
                          void *stream) {
    return launch_encode(table, bytes, piece_offsets, n_bytes, n_pieces, out_ids, out_offsets, workspace,
                         workspace_bytes, opts, (hipStream_t)stream, nullptr);
}

extern "C" int bpe_encode_timed(const bpe_table *table, const uint8_t *bytes, const int32_t *piece_offsets,
                                int64_t n_bytes, int64_t n_pieces, int32_t *out_ids, int32_t *out_offsets,
                                void *workspace, int64_t workspace_bytes, const bpe_encode_options *opts,
                                void *stream, float *kernel_ms) {
    if (!kernel_ms) { set_error("kernel_ms is NULL"); return BPE_ERR_NULL; }
    hipEvent_t ev[kKernels + 1];
    for (int i = 0; i <= kKernels; ++i) {
        hipError_t e = hipEventCreate(&ev[i]);
        if (e != hipSuccess) {
            for (int k = 0; k < i; ++k) (void)hipEventDestroy(ev[k]);
            return hip_fail(e, "hipEventCreate");
        }
    }
    int rc = launch_encode(table, bytes, piece_offsets, n_bytes, n_pieces, out_ids, out_offsets, workspace,
                           workspace_bytes, opts, (hipStream_t)stream, ev);
    if (rc == BPE_OK) {
        hipError_t e = hipEventSynchronize(ev[kKernels]);
        if (e != hipSuccess) rc = hip_fail(e, "hipEventSynchronize");
        for (int i = 0; i < kKernels && rc == BPE_OK; ++i) {
            e = hipEventElapsedTime(&kernel_ms[i], ev[i], ev[i + 1]);
            if (e != hipSuccess) rc = hip_fail(e, "hipEventElapsedTime");
        }
    }
    for (int i = 0; i <= kKernels; ++i) (void)hipEventDestroy(ev[i]);
    return rc;
}

extern "C" int bpe_encode_raw(const bpe_table *table, const uint8_t *bytes, int64_t n_bytes,
                              const int32_t *seq_offsets, int64_t n_seqs, int64_t max_pieces, int32_t *out_ids,
                              int32_t *seq_token_offsets, int32_t *piece_offsets, int32_t *out_offsets,
                              int32_t *n_pieces, void *workspace, int64_t workspace_bytes,
                              const bpe_encode_options *opts, void *stream) {
    const RawArgs raw = {seq_offsets, seq_offsets ? n_seqs : 1, seq_token_offsets, piece_offsets, out_offsets, n_pieces};
    return launch_encode(table, bytes, nullptr, n_bytes, max_pieces == 0 ? n_bytes : max_pieces, out_ids, out_offsets,
                         workspace, workspace_bytes, opts, (hipStream_t)stream, nullptr, &raw);
}

extern "C" int bpe_encode_raw_timed(const bpe_table *table, const uint8_t *bytes, int64_t n_bytes,
                                    const int32_t *seq_offsets, int64_t n_seqs, int64_t max_pieces,
                                    int32_t *out_ids, int32_t *seq_token_offsets, int32_t *piece_offsets,
                                    int32_t *out_offsets, int32_t *n_pieces, void *workspace,
                                    int64_t workspace_bytes, const bpe_encode_options *opts, void *stream,
                                    float *kernel_ms) {
    if (!kernel_ms) { set_error("kernel_ms is NULL"); return BPE_ERR_NULL; }
    hipEvent_t ev[kRawKernels + 1];
    for (int i = 0; i <= kRawKernels; ++i) {
        hipError_t e = hipEventCreate(&ev[i]);
        if (e != hipSuccess) {
            for (int k = 0; k < i; ++k) (void)hipEventDestroy(ev[k]);
            return hip_fail(e, "hipEventCreate");
        }
    }
    const RawArgs raw = {seq_offsets, seq_offsets ? n_seqs : 1, seq_token_offsets, piece_offsets, out_offsets, n_pieces};
    int rc = launch_encode(table, bytes, nullptr, n_bytes, max_pieces == 0 ? n_bytes : max_pieces, out_ids,
                           out_offsets, workspace, workspace_bytes, opts, (hipStream_t)stream, ev, &raw);
    if (rc == BPE_OK) {
        hipError_t e = hipEventSynchronize(ev[kRawKernels]);
        if (e != hipSuccess) rc = hip_fail(e, "hipEventSynchronize");
        for (int i = 0; i < kRawKernels && rc == BPE_OK; ++i) {
            e = hipEventElapsedTime(&kernel_ms[i], ev[i], ev[i + 1]);
            if (e != hipSuccess) rc = hip_fail(e, "hipEventElapsedTime");
        }
    }
    for (int i = 0; i <= kRawKernels; ++i) (void)hipEventDestroy(ev[i]);
    return rc;
}

extern "C" int bpe_encode_status(void *workspace, void *stream) {
    if (!workspace) { set_error("null workspace"); return BPE_ERR_NULL; }
    hipError_t e = hipStreamSynchronize((hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e, "hipStreamSynchronize");
    int32_t st[4] = {0, 0, 0, 0};
    e = hipMemcpy(st, workspace, sizeof(st), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return hip_fail(e, "hipMemcpy(status)");
    if (st[0] == st[2] || st[1] == st[2] || st[3] == st[2]) {
        // Reported once: a call that was recorded into a graph has the same call id at
        // every replay, and a later, clean replay must not inherit this verdict.
        const int32_t cleared[4] = {~st[2], ~st[2], st[2], ~st[2]};
        e = hipMemcpy(workspace, cleared, sizeof(cleared), hipMemcpyHostToDevice);
        if (e != hipSuccess) return hip_fail(e, "hipMemcpy(status)");
    }
    if (st[3] == st[2]) { set_error("a wait between workgroups ran out (is the workspace shared by overlapping calls?)"); return BPE_ERR_HIP; }
    if (st[0] == st[2]) { set_error("piece_offsets or seq_offsets are out of range or decreasing, or a token id is not in the vocabulary"); return BPE_ERR_INPUT; }
    if (st[1] == st[2]) { set_error("more pieces than max_pieces, or more bytes than out_capacity"); return BPE_ERR_SIZE; }
    return BPE_OK;
}

struct bpe_pool {
    void *mem;
    int64_t bytes;
};

extern "C" int bpe_pool_create(int64_t max_bytes, int64_t max_pieces, bpe_pool **out_pool) {
    if (!out_pool) { set_error("out_pool is NULL"); return BPE_ERR_NULL; }
    *out_pool = nullptr;
    // enough for bpe_encode and for bpe_encode_raw with up to max_pieces sequences; the
    // pre-tokenizer and the decoder (up to max_bytes tokens) need less
    int64_t need = bpe_workspace_bytes(max_bytes, max_pieces);
    if (need < 0) return (int)need;
    need = std::max(need, bpe_encode_raw_workspace_bytes(max_bytes, std::max<int64_t>(max_pieces, 1), max_pieces));
    bpe_pool *pool = new (std::nothrow) bpe_pool();
    if (!pool) { set_error("out of host memory"); return BPE_ERR_SIZE; }
    hipError_t e = hipMalloc(&pool->mem, (size_t)need);
    if (e != hipSuccess) { delete pool; return hip_fail(e, "hipMalloc(pool)"); }
    pool->bytes = need;
    *out_pool = pool;
    return BPE_OK;
}

extern "C" int bpe_pool_destroy(bpe_pool *pool) {
    if (!pool) return BPE_OK;
    hipError_t e = hipFree(pool->mem);
    delete pool;
    return e == hipSuccess ? BPE_OK : hip_fail(e, "hipFree(pool)");
}

extern "C" int bpe_pool_workspace(const bpe_pool *pool, void **workspace, int64_t *workspace_bytes) {
    if (!pool || !workspace || !workspace_bytes) { set_error("null pointer"); return BPE_ERR_NULL; }
    *workspace = pool->mem;
    *workspace_bytes = pool->bytes;
    return BPE_OK;
}

// Merge paths for longer pieces: one wavefront or one workgroup per piece.  The
// best-rank passes (selection levels 1 and 2), the bound-pairs passes (level 3) and,
// for comparison, the paper's own two kernels.  Device code, included by
// bpe_encode.hip.
#pragma once
#include "bpe_encode_params.h"
#include "bpe_lookback.h"
#include "bpe_short_pieces.h"

namespace bpe {

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

// Smallest (hi, lo) of the wavefront, to every lane.
__device__ inline void wave_min_pair(uint32_t &hi, uint32_t &lo) {
    const uint32_t best_hi = wave_min_u32(hi);
    lo = wave_min_u32(hi == best_hi ? lo : 0xFFFFFFFFu);
    hi = best_hi;
}

__device__ inline uint64_t group_min(uint64_t v, GroupTmp &tmp) {
    uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
    wave_min_pair(hi, lo);
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
    const int inc = wave_scan_max_inclusive(v);
    if (lane == kWave - 1) tmp.max_w[wv] = inc;
    __syncthreads();
    int ex = wave_from_lane_below(inc, -1);
    for (int w = 0; w < wv; ++w) ex = max(ex, tmp.max_w[w]);
    return ex;
}

// Exclusive sum-scan over the threads of the group; total to every thread.
__device__ inline int group_scan_sum_excl(int v, GroupTmp &tmp, int &total) {
    const int lane = lane_id(), wv = threadIdx.x / kWave;
    const int inc = wave_scan_inclusive(v);
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
        v = __builtin_amdgcn_readlane(wave_scan_max_inclusive(v), kWave - 1);
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
        const int up = wave_from_lane_below(v, 0);
        return lane ? up : (wv ? tmp.last_w[wv - 1] : 0);
    }
};

// A workgroup of 16 wavefronts that shares one piece (merge_wide_kernel: inputs of
// a few very long pieces, where a 256-thread workgroup per piece leaves the chip idle).
constexpr int kWideWaves = 16;
constexpr int kWideThreads = kWideWaves * kWave;
struct WideTmp {
    uint32_t min_lo[kWideWaves], min_hi[kWideWaves];
    int max_w[kWideWaves], sum_w[kWideWaves], last_w[kWideWaves], all_w[kWideWaves];
};

struct WideScope {
    static constexpr int kThreads = kWideThreads;
    WideTmp &tmp;
    __device__ int tid() const { return threadIdx.x; }
    __device__ void sync() const { __syncthreads(); }
    __device__ uint64_t min_u64(uint64_t v) const {
        uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
        wave_min_pair(hi, lo);
        const int wv = threadIdx.x / kWave;
        if (lane_id() == 0) { tmp.min_lo[wv] = lo; tmp.min_hi[wv] = hi; }
        __syncthreads();
        uint64_t best = ~0ull;
        for (int w = 0; w < kWideWaves; ++w) best = min(best, ((uint64_t)tmp.min_hi[w] << 32) | tmp.min_lo[w]);
        return best;
    }
    __device__ int scan_max_excl(int v) const {
        const int lane = lane_id(), wv = threadIdx.x / kWave;
        const int inc = wave_scan_max_inclusive(v);
        if (lane == kWave - 1) tmp.max_w[wv] = inc;
        __syncthreads();
        int ex = wave_from_lane_below(inc, -1);
        for (int w = 0; w < wv; ++w) ex = max(ex, tmp.max_w[w]);
        return ex;
    }
    __device__ int scan_sum_excl(int v, int &total) const {
        const int lane = lane_id(), wv = threadIdx.x / kWave;
        const int inc = wave_scan_inclusive(v);
        if (lane == kWave - 1) tmp.sum_w[wv] = inc;
        __syncthreads();
        int ex = inc - v;
        total = 0;
        for (int w = 0; w < kWideWaves; ++w) {
            if (w < wv) ex += tmp.sum_w[w];
            total += tmp.sum_w[w];
        }
        return ex;
    }
    __device__ int max_all(int v) const {
        v = __builtin_amdgcn_readlane(wave_scan_max_inclusive(v), kWave - 1);
        if (lane_id() == 0) tmp.all_w[threadIdx.x / kWave] = v;
        __syncthreads();
        int m = tmp.all_w[0];
        for (int w = 1; w < kWideWaves; ++w) m = max(m, tmp.all_w[w]);
        return m;
    }
    __device__ int from_previous_thread(int v) const {
        const int lane = lane_id(), wv = threadIdx.x / kWave;
        if (lane == kWave - 1) tmp.last_w[wv] = v;
        __syncthreads();
        const int up = wave_from_lane_below(v, 0);
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
    // All four by data-parallel primitives inside the wavefront (no LDS crossbar).
    __device__ uint64_t min_u64(uint64_t v) const {
        uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
        wave_min_pair(hi, lo);
        return ((uint64_t)hi << 32) | lo;
    }
    __device__ int scan_max_excl(int v) const {
        return wave_from_lane_below(wave_scan_max_inclusive(v), -1);
    }
    __device__ int scan_sum_excl(int v, int &total) const {
        const int inc = wave_scan_inclusive(v);
        total = __builtin_amdgcn_readlane(inc, kWave - 1);
        return inc - v;
    }
    __device__ int from_previous_thread(int v) const {
        return wave_from_lane_below(v, 0);
    }
    __device__ int max_all(int v) const {
        v = __builtin_amdgcn_readlane(wave_scan_max_inclusive(v), kWave - 1);
        return v;
    }
};

// A piece that one wavefront merges in LDS (or in the workspace) has shrunk to cur <= 64
// symbols in A: the remaining passes run on one symbol per lane in registers (a pass
// there is one table round trip and a permute; through LDS it is a dozen dependent
// round trips).  Tokens to out[0 ...]; returns their number.
template <typename Ptr>
__device__ __forceinline__ int finish_in_registers(const EncodeParams &p, Ptr A, int cur, int32_t *out) {
    const int lane = lane_id();
    uint32_t sym = lane < cur ? (uint32_t)A[lane] : 0u;
    cur = encode_wave_symbols(p, sym, cur);
    if (lane < cur) out[lane] = (int32_t)sym;
    WaveScope{}.sync();
    return cur;
}

// The same for any scope: the first wavefront finishes the piece, the others wait.
template <typename Scope, typename Ptr>
__device__ __forceinline__ int finish_small(const EncodeParams &p, Ptr A, int cur, int32_t *out, const Scope &sc) {
    if (Scope::kThreads == kWave) return finish_in_registers(p, A, cur, out);
    int c = 0;
    if (sc.tid() < kWave) c = finish_in_registers(p, A, cur, out);
    return sc.max_all(c);          // a barrier: the tokens are visible to every thread
}

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
            r[u] = i + 1 < cur ? table_find(p.table, (uint32_t)A[i], (uint32_t)A[i + 1]) : kNoRank;
            if (r[u] != kNoRank) r[u] >>= kRankShift;
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
    int32_t *out = p.scratch + b;
    while (cur >= 2) {
        if (cur <= kWave) return finish_small(p, A, cur, out, sc);
        const int n = best_rank_pass(p, A, B, cur, sc);
        if (n < 0) break;
        Ptr t = A; A = B; B = t;
        cur = n;
    }
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
constexpr int kWideBoundMax = 4032;                // a workgroup of 16 wavefronts (merge_wide_kernel): 63 KiB of LDS
static_assert(kWaveBoundMax <= 32 * kWave && kGroupBoundMax <= 32 * kGroupThreads && kWideBoundMax <= 32 * kWideThreads,
              "a thread's chunk fits a 32-bit mask");
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
                if (i + 1 < n) r[u] = table_find(p.table, sym, (uint32_t)S[i + 1]);
                if (r[u] != kNoRank) r[u] >>= kRankShift;
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

// Whether at least half of the adjacent bytes at the head of the piece (one pair per
// thread) are equal.  Such a piece is runs x x x ...: the best-rank passes halve it
// per pass, nothing else in it can merge before them, and they hold twice as many
// symbols in the same LDS.  Only a choice between two exact methods: a piece that
// is judged wrongly is merely slower.
template <typename Scope>
__device__ __forceinline__ bool piece_is_run_like(const EncodeParams &p, int b, int n, const Scope &sc) {
    const int m = min(n - 1, Scope::kThreads);      // pairs looked at
    const int i = sc.tid();
    const int eq = i < m && p.bytes[b + i] == p.bytes[b + i + 1];
    int total;
    (void)sc.scan_sum_excl(eq, total);
    return 2 * total >= m;
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
        if (cur <= kWave) return finish_small(p, S, cur, out, sc);
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
            const uint32_t r = table_find(p.table, (uint32_t)A[i], (uint32_t)A[i + 1]);
            if (r != kNoRank) best = min(best, ((uint64_t)(r >> kRankShift) << 32) | (uint32_t)i);
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

}  // namespace bpe

// The merge loop (paper sections 3.4 and 3.5: pair evaluation, argmin,
// compaction, repeat) and the on-device assembly of the dense output (section
// 3.1, stage 4), for gfx950.
//
// All kernels work on the same tiling of the piece array (a tile = up to 64
// pieces per wavefront x 4 wavefronts).  merge_tile merges every piece of a tile
// by length class:
//     <= 16 bytes    one lane per piece, state in 16-entry LDS columns (bpe_short_pieces.h);
//     <= 64 bytes    one lane per piece, 64-entry columns, 16 pieces per wavefront and round;
//     runs x x x ... one lane per run of equal symbols, one wavefront per piece, any length;
//     <= 640 bytes   one wavefront, the piece in its LDS region        (bpe_long_pieces.h);
//     longer         one piece per workgroup, in LDS (in windows through the workspace
//                    beyond the LDS budget);
// and whatever has shrunk to 64 symbols finishes in registers, one lane per symbol.
// Grids of up to 256 tiles: encode_kernel does the merges and the ordered assembly of
// the output in one launch (tile totals chained through tagged state words).
// Up to 1024 tiles (what the chip holds at once): merge_tiles_kernel, then emit_kernel
// (out_offsets and the dense copy into out_ids).
// Deeper grids: merge_kernel, whose first workgroups take the pieces beyond 16 bytes of
// four tiles each while the others merge the short pieces of one tile; then emit_kernel,
// from 4096 tiles on emit_deep_kernel (four tiles per workgroup), with scan_tiles_kernel
// in between when there are too many tile totals for the emit workgroups to add up.
// Raw path (bpe_encode_raw): token-only calls on inputs the chip holds at once find the
// pieces inside the merge kernel (merge_bytes_kernel, emit_bytes_kernel: tiles of 1280
// bytes); otherwise the pre-tokenizer first, then merge_raw_kernel and emit_raw_kernel,
// which stride over the tiles that exist (the piece count is only known on the device),
// then the first token of every sequence.
// Option paper_kernel: the paper's own two kernels, one workgroup per piece.
// Option dedup: every distinct piece of up to 16 bytes is merged once (bpe_dedup.h).
// No kernel allocates, and the host side neither synchronises nor copies.
#include <algorithm>
#include <atomic>
#include <cstdio>
#include <new>
#include <tuple>
#include <utility>

#include "bpe_common.h"
#include "bpe_dedup.h"
#include "bpe_encode_params.h"
#include "bpe_long_pieces.h"
#include "bpe_lookback.h"
#include "bpe_short_pieces.h"

namespace bpe {

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
    int cnt_back[kGroupThreads];   // token counts handed back to the owning thread (long-piece workgroups: more list)
    int list_n, list_back;
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
// Where the pieces of a tile come from: the caller's (or the pre-tokenizer's) offsets array; the
// offsets array through a list of pieces (de-duplication); or the piece starts that the workgroup
// found itself in its share of the bytes (bpe_encode_raw without a pre-tokenizer launch).
enum PieceSource { kFromOffsets = 0, kFromList = 1, kFromBytes = 2 };

// kFromBytes: the starts of the tile's pieces as the workgroup holds them in LDS.
struct ByteTile {
    const uint16_t *starts;   // [n_t] start of piece k, counted from the tile's first byte
    int lo;                   // index of the tile's first byte
    int k0;                   // the 256 pieces being merged are k0 ... of the tile
    int n_t;                  // pieces that start in the tile
    int end_rel;              // where the tile's last piece ends, counted from lo (may lie far behind the tile)
};

template <int SRC>
__device__ __forceinline__ TilePiece merge_tile_long_pieces(const EncodeParams &p, TileShared &sh, TilePiece t,
                                                            int64_t tile_q0, int P, bool is_wave, bool is_long,
                                                            const ByteTile &bt);

// The piece whose offsets entry number q of the launch reads: q itself, or, with a list
// (de-duplication), the q-th piece of the list of pieces to merge.
template <int SRC>
__device__ __forceinline__ int64_t piece_of(const EncodeParams &p, int64_t q) {
    return SRC == kFromList ? (int64_t)p.piece_map[q] : q;
}

// First byte and length of the piece that thread `owner` of the tile holds.
template <int SRC>
__device__ __forceinline__ void piece_bounds(const EncodeParams &p, const ByteTile &bt, int64_t tile_q0, int P, int owner,
                                             int &b, int &n) {
    if (SRC == kFromBytes) {
        const int k = bt.k0 + owner;
        const int s0 = bt.starts[k], s1 = k + 1 < bt.n_t ? (int)bt.starts[k + 1] : bt.end_rel;
        b = bt.lo + s0;
        n = s1 - s0;
    } else {
        const int64_t q = piece_of<SRC>(p, tile_q0 + (int64_t)(owner / kWave) * P + (owner % kWave));
        b = p.off[q];                                  // validated by the owner
        n = p.off[q + 1] - b;
    }
}

// n_pieces, P: the piece count and the pieces per wavefront of this launch (p's own
// values, except on the raw path, where the kernel finds them out).
// SKIP_LONG: the pieces beyond tiny_max are somebody else's (merge_kernel's long-piece
// workgroups): they count as no tokens here and get no record from this tile.
// SRC == kFromBytes: `tile` and n_pieces are not used; the thread's piece is number bt.k0 + threadIdx.x of
// the tile (if that is below bt.n_t), and its record goes to slot bt_q0 + that number.
template <int SRC = kFromOffsets, bool SKIP_LONG = false>
__device__ __forceinline__ TilePiece merge_tile(const EncodeParams &p, TileShared &sh, int tile, bool keep_in_lds,
                                                int n_pieces, int P, const ByteTile &bt = ByteTile{}, int64_t bt_q0 = 0) {
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
    if (tid == 0) { sh.list_n = 0; sh.list_back = 0; }
    TilePiece t;
    const int64_t tile_q0 = SRC == kFromBytes ? bt_q0 + bt.k0 : (int64_t)tile * p.W * P;
    t.q = SRC == kFromBytes ? tile_q0 + tid : tile_q0 + (int64_t)wv * P + lane;
    t.has_piece = SRC == kFromBytes ? bt.k0 + tid < bt.n_t : lane < P && wv < p.W && t.q < n_pieces;
    t.o = 0;
    t.len = 0;
    bool bad = false;
    if (SRC == kFromBytes) {
        if (t.has_piece) piece_bounds<SRC>(p, bt, tile_q0, P, tid, t.o, t.len);    // the workgroup's own findings
    } else if (t.has_piece) {
        const int64_t pq = piece_of<SRC>(p, t.q);
        t.o = p.off[pq];
        const int o_next = p.off[pq + 1];
        bad = t.o < 0 || o_next < t.o || o_next > p.n_bytes;
        // (with a list of pieces, the kernel that made the list has looked at the first and the last piece)
        if (SRC == kFromOffsets) bad |= (t.q == 0 && t.o != 0) || (t.q == n_pieces - 1 && o_next != p.n_bytes);
        t.len = bad ? 0 : o_next - t.o;
    }
    if (__ballot(bad) && lane == 0)
        __hip_atomic_store(&p.status[0], p.call_id, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    t.is_tiny = t.has_piece && t.len > 0 && t.len <= p.tiny_max;
    t.long_path = false;
    // (with the default selection level every longer piece visits a wavefront first: it may be runs)
    const bool is_wave = t.has_piece && t.len > p.tiny_max && (t.len <= p.wave_lds_max || p.runs_by_best_rank);
    const bool is_long = t.has_piece && t.len > p.wave_lds_max && !p.runs_by_best_rank;

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

    if (SKIP_LONG) {
        t.has_piece = t.has_piece && !is_wave && !is_long;     // whoever merges a piece writes its record
        return t;
    }
    // Everything else is rare in word-like text: one barrier finds out whether the tile has any.
    if (__syncthreads_count(is_wave || is_long) == 0) return t;
    return merge_tile_long_pieces<SRC>(kernel_params(), sh, t, tile_q0, P, is_wave, is_long, bt);
}

// The kernel's parameter block as it lies in the kernel-argument segment (every kernel
// that merges takes EncodeParams as its first parameter).  The rare paths read their
// parameters from there when they get to them, so that the registers of the common
// path above do not have to hold them: with the parameters passed down by reference the
// compiler kept them all live from the start of the kernel and spilled dozens of them.
__device__ __forceinline__ const EncodeParams &kernel_params() {
    return *(const EncodeParams *)__builtin_amdgcn_kernarg_segment_ptr();
}

// Which entries of the list of pieces for the wavefront paths wavefront wv takes: first, first + stride, ...
// The columns keep the wavefronts they fill busy for as long as their longest piece merges (up to 64 merges of
// one dependent lookup each), so the other pieces go to the wavefronts without columns, from the last one
// down, while there are any (a round of columns fills the first wavefront first); otherwise to all four.
// Wave-uniform by construction: every value that steers a loop comes through readfirstlane.
struct WaveDeal { int first, stride; };
__device__ __forceinline__ WaveDeal wave_deal(int n_col, int n_entries, int wv) {
    const int with_columns = min((n_col + kColumnLanes - 1) / kColumnLanes, kWavesPerGroup);
    WaveDeal d;
    if (with_columns < kWavesPerGroup) {
        d.stride = kWavesPerGroup - with_columns;
        d.first = wv >= with_columns ? kWavesPerGroup - 1 - wv : n_entries;      // n_entries: none
    } else {
        d.stride = kWavesPerGroup;
        d.first = kWavesPerGroup - 1 - wv;
    }
    d.first = __builtin_amdgcn_readfirstlane(d.first);
    d.stride = __builtin_amdgcn_readfirstlane(d.stride);
    return d;
}

// Second half of merge_tile: the wavefront and workgroup paths of the tile's longer pieces.
// P: pieces per wavefront of this launch (on the raw path the kernel may have chosen it).
template <int SRC>
__device__ __forceinline__ TilePiece merge_tile_long_pieces(const EncodeParams &p, TileShared &sh, TilePiece t,
                                                            int64_t tile_q0, int P, bool is_wave, bool is_long,
                                                            const ByteTile &bt) {
    const int tid = threadIdx.x, lane = lane_id(), wv = tid / kWave;
    if (!t.parked) {               // the other paths reuse the LDS of the lane-per-piece state
        tiny_store(sh.lds.tiny[wv], t.alive, p.scratch + t.o);
        t.parked = true;
    }

    // Wavefront paths.  The tile's wavefronts share these pieces through lists in
    // LDS, so that a wavefront that owns several of them does not become the tail:
    // pieces for the 64-entry columns from the front of the list, the longer ones
    // from its back.
    const bool is_col = is_wave && t.len <= p.col_max;
    if (is_col) sh.list[atomicAdd(&sh.list_n, 1)] = tid;
    else if (is_wave) sh.list[kGroupThreads - 1 - atomicAdd(&sh.list_back, 1)] = tid;
    __syncthreads();
    // Columns: 16 pieces per wavefront and round, entry 64 r + 16 w + l to lane l of wavefront w.
    // The first wavefront fills up first: a step costs a wavefront the same instructions
    // for one piece as for 16, and the compute unit's other tiles want the issue slots.
    const int n_col = __builtin_amdgcn_readfirstlane(sh.list_n);
    for (int e0 = 0; e0 < n_col; e0 += kWavesPerGroup * kColumnLanes) {
        const int e = e0 + kColumnLanes * wv + lane;
        const bool mine = lane < kColumnLanes && e < n_col;
        int owner = 0, b = 0, n = 0;
        if (mine) {
            owner = sh.list[e];
            piece_bounds<SRC>(p, bt, tile_q0, P, owner, b, n);
        }
        ColumnState &cs = *(ColumnState *)&sh.lds.tiny[wv];
        const uint64_t alive = column_merge<kColumnMax>(p, cs, b, n, mine);
        column_store<kColumnMax>(cs, alive, p.scratch + b);
        if (mine) sh.cnt_back[owner] = mask_count(alive);
    }
    // Entry e goes to wavefront e mod 4.  Everything that steers the loop is made
    // wave-uniform explicitly: a lane-0-only atomic ticket followed by readfirstlane
    // compiled into a loop in which the other 63 lanes kept re-reading their own
    // initial value of the ticket and never left.
    // (dealt to the wavefronts that have no columns: see wave_deal)
    const int n_work = __builtin_amdgcn_readfirstlane(sh.list_back);
    const WaveDeal deal = wave_deal(n_col, n_work, wv);
    for (int e = deal.first; e < n_work; e += deal.stride) {
        const int owner = __builtin_amdgcn_readfirstlane(sh.list[kGroupThreads - 1 - e]);
        int b, n;
        piece_bounds<SRC>(p, bt, tile_q0, P, owner, b, n);
        b = __builtin_amdgcn_readfirstlane(b);
        n = __builtin_amdgcn_readfirstlane(n);
        int c = -1;
        // mostly runs of one byte: one run per lane, whatever the length (-1: too many runs after all)
        if (p.runs_by_best_rank && n > p.wave_max && piece_is_run_like(p, b, n, WaveScope{}))
            c = encode_wave_runs(p, b, n, &sh.lds.tiny[wv].S[0][0]);
        if (c >= 0) {}
        else if (n > p.wave_lds_max) c = kLongMark;
        else if (n <= p.wave_max) c = encode_wave_piece(p, b, n);
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
        int b, n;
        piece_bounds<SRC>(p, bt, tile_q0, P, owner, b, n);
        b = __builtin_amdgcn_readfirstlane(b);
        n = __builtin_amdgcn_readfirstlane(n);
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
template <int SRC = kFromOffsets, bool SKIP_LONG = false>
__device__ __forceinline__ void merge_and_count_tile(const EncodeParams &p, TileShared &sh, int *wave_tokens, int tile,
                                                     int n_pieces, int P) {
    const TilePiece t = merge_tile<SRC, SKIP_LONG>(p, sh, tile, false, n_pieces, P);
    if (t.has_piece) p.rec[t.q] = make_int2(t.cnt, t.tok0);
    const int wave_total = __builtin_amdgcn_readlane(wave_scan_inclusive(t.cnt), kWave - 1);
    if (lane_id() == 0) wave_tokens[threadIdx.x / kWave] = wave_total;
    __syncthreads();
    if (threadIdx.x == 0) {
        int sum = 0;
        for (int w = 0; w < kWavesPerGroup; ++w) sum += wave_tokens[w];
        p.tile_sum[tile] = sum;
    }
}

// ---------------------------------------------------------------------------
// The pieces beyond tiny_max of p.tiles_per_long_group consecutive tiles (of 256 pieces),
// by one workgroup.  In word-like text they are few, and each is a chain of dependent
// steps ten times as long as a word's.  Merged inside their tiles they made every tile
// that held one wait for it, tile after tile; here they start first (these workgroups
// lead the grid), many of them share a round of the column path, and the tiles of short
// pieces flow past them.  Lists in LDS: pieces for the 64-entry columns from the front,
// pieces for the wavefront paths from the back, then the ones for the whole workgroup;
// an entry is the piece's index counted from the group's first piece.
constexpr int kLongListMax = 2 * kGroupThreads;       // entries: TileShared::list and ::cnt_back together
constexpr int kLongGroupsMinTilesDevice = 1025;       // more tiles than the chip holds at a time (see kLongGroupsMinTiles)

struct LongLists {
    int *entry;        // [kLongListMax]
    int n_col, n_back;
};

__device__ __forceinline__ void long_pieces_flush(const EncodeParams &p, TileShared &sh, int *entry, int *acc,
                                              int64_t q_base) {
    const int tid = threadIdx.x, lane = lane_id(), wv = tid / kWave;
    __syncthreads();               // the lists are complete
    // what a finished piece leaves: its record, and its tokens in its tile's total
    auto done = [&](int rel, int c) {
        p.rec[q_base + rel] = make_int2(c, -1);
        atomicAdd(&acc[rel / kGroupThreads], c);
    };
    // Columns: 16 pieces per wavefront and round, the first wavefront fills up first.
    const int n_col = __builtin_amdgcn_readfirstlane(sh.list_n);
    for (int e0 = 0; e0 < n_col; e0 += kWavesPerGroup * kColumnLanes) {
        const int e = e0 + kColumnLanes * wv + lane;
        const bool mine = lane < kColumnLanes && e < n_col;
        int rel = 0, b = 0, n = 0;
        if (mine) {
            rel = entry[e];
            b = p.off[q_base + rel];                     // validated when the piece was listed
            n = p.off[q_base + rel + 1] - b;
        }
        ColumnState &cs = *(ColumnState *)&sh.lds.tiny[wv];
        const uint64_t alive = column_merge<kColumnMax>(p, cs, b, n, mine);
        column_store<kColumnMax>(cs, alive, p.scratch + b);
        if (mine) done(rel, mask_count(alive));
    }
    // Wavefront paths, dealt to the wavefronts that have no columns (see wave_deal).
    // What a wavefront hands on to the workgroup goes to the front of the list, which the
    // columns are done with... once every wavefront has left them: hence its own counter.
    const int n_back = __builtin_amdgcn_readfirstlane(sh.list_back);
    const WaveDeal deal = wave_deal(n_col, n_back, wv);
    for (int e = deal.first; e < n_back; e += deal.stride) {
        const int rel = __builtin_amdgcn_readfirstlane(entry[kLongListMax - 1 - e]);
        const int b = __builtin_amdgcn_readfirstlane(p.off[q_base + rel]);
        const int n = __builtin_amdgcn_readfirstlane(p.off[q_base + rel + 1]) - b;
        int c = -1;
        if (p.runs_by_best_rank && n > p.wave_max && piece_is_run_like(p, b, n, WaveScope{}))
            c = encode_wave_runs(p, b, n, &sh.lds.tiny[wv].S[0][0]);
        if (c >= 0) {}
        else if (n > p.wave_lds_max) c = kLongMark;
        else if (n <= p.wave_max) c = encode_wave_piece(p, b, n);
        else if (p.level >= 3 && !(p.runs_by_best_rank && piece_is_run_like(p, b, n, WaveScope{})))
            c = n <= kWaveBoundHandOn ? encode_long_piece_bound(p, b, n, &sh.lds.tiny[wv].S[0][0], kWaveBoundMax, WaveScope{})
                                      : kLongMark;
        else c = encode_wave_lds_piece(p, b, n, sh.lds.tiny[wv]);
        if (lane == 0) {
            if (c == kLongMark) entry[kLongListMax - 1 - e] = ~rel;      // for the workgroup
            else done(rel, c);
        }
    }
    __syncthreads();
    // Workgroup path, one piece at a time by all threads: the marked entries of the back list.
    for (int e = 0; e < n_back; ++e) {
        const int rel = ~__builtin_amdgcn_readfirstlane(entry[kLongListMax - 1 - e]);
        if (rel < 0) continue;     // a wavefront has merged it
        const int b = __builtin_amdgcn_readfirstlane(p.off[q_base + rel]);
        const int n = __builtin_amdgcn_readfirstlane(p.off[q_base + rel + 1]) - b;
        int c;
        if (p.level >= 3 && !(p.runs_by_best_rank && piece_is_run_like(p, b, n, GroupScope{sh.tmp})))
            c = encode_long_piece_bound(p, b, n, (uint32_t *)sh.lds.group.A,
                                        min(max(p.lds_max, kGroupBoundMin), kGroupBoundMax), GroupScope{sh.tmp});
        else if (n <= p.lds_max) c = encode_group_piece<int32_t *>(p, b, n, sh.lds.group.A, sh.lds.group.B, sh.tmp);
        else c = encode_group_piece<int32_t *>(p, b, n, p.scratch + b, p.scratch2 + b, sh.tmp);
        if (tid == 0) done(rel, c);
    }
    __syncthreads();
    if (tid == 0) {
        sh.list_n = 0;
        sh.list_back = 0;
        // some piece of this call went through these workgroups: the emit kernels add long_sum to tile_sum
        p.status[kStatusLongPieces] = p.call_id;
    }
    __syncthreads();
}

// n_pieces, n_tiles: the pieces there are, and the tiles whose long pieces these workgroups take.
__device__ __forceinline__ void long_pieces_group(const EncodeParams &p, TileShared &sh, int *acc, int group,
                                                  int n_pieces, int n_tiles) {
    const int tid = threadIdx.x;
    // the two arrays are adjacent members of TileShared: one list of kLongListMax entries
    static_assert(offsetof(TileShared, cnt_back) == offsetof(TileShared, list) + sizeof(int) * kGroupThreads,
                  "list and cnt_back form one array");
    int *entry = sh.list;
    const int tile0 = group * p.tiles_per_long_group;
    const int tile1 = min(tile0 + p.tiles_per_long_group, n_tiles);
    const int64_t q_base = (int64_t)tile0 * kGroupThreads;
    acc[tid] = 0;
    if (tid == 0) { sh.list_n = 0; sh.list_back = 0; }
    __syncthreads();
    // First a look at all the group's pieces with every load in flight at once: in word-like text
    // there is usually nothing to do, and then that is all this workgroup costs.
    {
        bool any = false;
        for (int t0 = tile0; t0 < tile1; t0 += 8) {
            int len[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int64_t q = (int64_t)(t0 + i) * kGroupThreads + tid;
                len[i] = t0 + i < tile1 && q < n_pieces ? p.off[q + 1] - p.off[q] : 0;
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) any |= len[i] > p.tiny_max;      // (bad offsets may look long: the loop below looks closer)
        }
        if (__syncthreads_count(any) == 0) {
            if (tile0 + tid < tile1) p.long_sum[tile0 + tid] = 0;
            return;
        }
    }
    // Two tiles at a time (as many entries as the lists hold at most); the lists are worked off when
    // the next two might not fit, and at the end.
    constexpr int kScanBatch = kLongListMax / kGroupThreads;
    for (int t0 = tile0;; t0 += kScanBatch) {
        const bool end = t0 >= tile1;
        int len[kScanBatch];
        int mine = 0;
#pragma unroll
        for (int i = 0; i < kScanBatch; ++i) {
            const int64_t q = (int64_t)(t0 + i) * kGroupThreads + tid;
            len[i] = 0;
            if (t0 + i < tile1 && q < n_pieces) {
                const int o = p.off[q], o_next = p.off[q + 1];
                const bool bad = o < 0 || o_next < o || o_next > p.n_bytes || (q == 0 && o != 0) ||
                                 (q == n_pieces - 1 && o_next != p.n_bytes);
                len[i] = bad ? 0 : o_next - o;     // the tile's own workgroup reports bad offsets
            }
            mine += len[i] > p.tiny_max;
        }
        const int batch_n = kScanBatch * __syncthreads_count(mine != 0);       // at most so many long pieces in these tiles
        if (!end && batch_n == 0) continue;                    // nothing but short pieces in these tiles
        const int listed = sh.list_n + sh.list_back;
        __syncthreads();           // every thread has read the counts before anyone lists a piece
        if (end ? listed > 0 : listed + batch_n > kLongListMax) long_pieces_flush(p, sh, entry, acc, q_base);
        if (end) break;
#pragma unroll
        for (int i = 0; i < kScanBatch; ++i) {
            const int rel = (int)((int64_t)(t0 + i) * kGroupThreads + tid - q_base);
            if (len[i] > p.tiny_max && len[i] <= p.col_max) entry[atomicAdd(&sh.list_n, 1)] = rel;
            else if (len[i] > p.col_max) entry[kLongListMax - 1 - atomicAdd(&sh.list_back, 1)] = rel;
        }
        __syncthreads();
    }
    __syncthreads();
    // (by every group, zeros too: once any group has merged something, the emit kernels read all of them)
    if (tile0 + tid < tile1) p.long_sum[tile0 + tid] = acc[tid];
}

// Every workgroup merges all pieces of its tile (grids of few tiles, tiles of fewer than 256
// pieces, the paper's kernels).
__global__ void __launch_bounds__(kGroupThreads) merge_tiles_kernel(EncodeParams p) {
    __shared__ TileShared sh;
    __shared__ int wave_tokens[kWavesPerGroup];
    merge_and_count_tile(p, sh, wave_tokens, blockIdx.x, p.n_pieces, p.P);
}

// Word-sized pieces on average: the first p.n_long_groups workgroups take the long pieces (see
// above), every other one the short pieces of one tile.
// (The long-piece role has one place where it works its lists off: inlined at three, it took the kernel
// beyond 128 vector registers, and the tiles lost a workgroup per compute unit to that.)
__global__ void __launch_bounds__(kGroupThreads) merge_kernel(EncodeParams p) {
    __shared__ TileShared sh;
    __shared__ int wave_tokens[kWavesPerGroup];
    // What a tile needs of the arguments is fetched before the role is known: left alone, the compiler
    // fetches n_long_groups, waits, branches, and only then fetches the rest, a second round trip to the
    // scalar cache at the head of every tile.
    asm volatile("" :: "s"(p.table.slots), "s"(p.table.byte_pairs), "s"(p.table.merged_of), "s"(p.table.half),
                       "s"(p.table.low_bits), "s"(p.table.index_bits), "s"(p.table.merged_delta), "s"(p.table.seed.k1a),
                       "s"(p.table.seed.k1b), "s"(p.table.seed.k2a), "s"(p.table.seed.k2b), "s"(p.bytes), "s"(p.off),
                       "s"(p.n_bytes), "s"(p.n_pieces), "s"(p.tiny_max), "s"(p.rec), "s"(p.tile_sum), "s"(p.scratch),
                       "s"(p.status), "s"(p.call_id), "s"(p.n_long_groups));
    if ((int)blockIdx.x >= p.n_long_groups) {
        merge_and_count_tile<kFromOffsets, true>(p, sh, wave_tokens, blockIdx.x - p.n_long_groups, p.n_pieces, p.P);
    } else {
        __shared__ int acc[kGroupThreads];
        const EncodeParams &kp = kernel_params();
        long_pieces_group(kp, sh, acc, blockIdx.x, kp.n_pieces, (kp.n_pieces + kGroupThreads - 1) / kGroupThreads);
    }
}

// Inputs of a few very long pieces (one piece per tile, at most kWideMaxPieces of
// them, longer on average than the 2,052 symbols four wavefronts keep resident): a
// workgroup of 16 wavefronts per piece instead of 4, with twice the symbols resident
// in LDS.  With so few pieces the chip is idle either way, and a pass over a long
// piece is as quick as the threads that share it are many (4 KiB pieces: 190 against
// 282 us, 16 KiB pieces: 478 against 1,050 us; 2 KiB pieces are quicker with four
// wavefronts, 178 against 224 us: more barriers than work).
constexpr int kWideMaxPieces = 256;     // one workgroup per CU
__global__ void __launch_bounds__(kWideThreads) merge_wide_kernel(EncodeParams p) {
    __shared__ uint32_t X[4 * kWideBoundMax];
    __shared__ WideTmp tmp;
    const int tid = threadIdx.x;
    const int q = blockIdx.x;
    int o = p.off[q];
    const int o_next = p.off[q + 1];
    const bool bad = o < 0 || o_next < o || o_next > p.n_bytes || (q == 0 && o != 0) ||
                     (q == p.n_pieces - 1 && o_next != p.n_bytes);
    if (bad && tid == 0) __hip_atomic_store(&p.status[0], p.call_id, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    o = __builtin_amdgcn_readfirstlane(o);
    const int len = __builtin_amdgcn_readfirstlane(bad ? 0 : o_next - o);
    const WideScope sc{tmp};
    int c = 0;
    if (len > 0) {
        const int cap = min(max(p.lds_max, kGroupBoundMin), kWideBoundMax);
        if (p.level >= 3 && !(p.runs_by_best_rank && piece_is_run_like(p, o, len, sc)))
            c = encode_long_piece_bound(p, o, len, X, cap, sc);
        else if (len <= 2 * cap)
            c = encode_long_piece<WideScope, int32_t *>(p, o, len, (int32_t *)X, (int32_t *)X + 2 * kWideBoundMax, sc);
        else
            c = encode_long_piece<WideScope, int32_t *>(p, o, len, p.scratch + o, p.scratch2 + o, sc);
    }
    if (tid == 0) {
        p.rec[q] = make_int2(c, -1);
        p.tile_sum[q] = c;
    }
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

// The same for a caller who says that the pieces are word-sized (pieces_per_wave 64 given, not left
// to the kernels): the first p.n_long_groups workgroups take the long pieces, as in merge_kernel.
__global__ void __launch_bounds__(kGroupThreads) merge_raw_groups_kernel(EncodeParams p) {
    __shared__ TileShared sh;
    __shared__ int wave_tokens[kWavesPerGroup];
    p.n_pieces = device_piece_count(p);
    const int n_tiles = tiles_of(p);
    if ((int)blockIdx.x < p.n_long_groups) {
        __shared__ int acc[kGroupThreads];
        // (the tiles beyond this kernel's grid are merged whole by merge_raw_rest_kernel)
        const int covered = min(n_tiles, (int)gridDim.x - p.n_long_groups);
        const int n_pieces = p.n_pieces;
        const EncodeParams &kp = kernel_params();      // (as they lie in memory: this role must not keep the tiles' registers busy)
        if ((int)blockIdx.x * kp.tiles_per_long_group < covered)
            long_pieces_group(kp, sh, acc, blockIdx.x, n_pieces, covered);
        return;
    }
    const int tile = blockIdx.x - p.n_long_groups;
    if (tile < n_tiles) merge_and_count_tile<kFromOffsets, true>(p, sh, wave_tokens, tile, p.n_pieces, p.P);
}

__global__ void __launch_bounds__(kGroupThreads) merge_raw_rest_kernel(EncodeParams p, int first_tile) {
    __shared__ TileShared sh;
    __shared__ int wave_tokens[kWavesPerGroup];
    raw_geometry(p);
    const int n_tiles = tiles_of(p);
    for (int tile = first_tile + blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        if (p.long_sum && threadIdx.x == 0) p.long_sum[tile] = 0;      // nothing of this tile goes to a long-piece workgroup
        merge_and_count_tile(p, sh, wave_tokens, tile, p.n_pieces, p.P);
        __syncthreads();   // the next tile reuses the LDS
    }
}

// ---------------------------------------------------------------------------
// bpe_encode_raw for callers that want tokens only (no piece arrays back): no pre-tokenizer
// launch and no piece offsets through memory.  A workgroup takes kByteTile bytes, finds
// the pieces that start there (a piece starts at byte 0, at a space and where a sequence
// starts) and merges them, including the one that runs on behind the tile.  Piece k of
// tile t owns slot t * kByteTileStride + k of the per-piece arrays (record, first byte).
constexpr int kByteTile = 1280;                  // 192 pieces of word-like text on average, for 256 lanes: with 1536
                                                 // bytes a tenth of the tiles had more than 256 and paid for it
constexpr int kByteTileStride = kByteTile + 1;
constexpr int kByteScanThreads = kByteTile / 8;  // a thread looks at 8 bytes

// Bit j set: byte j of the 8 bytes (lo, hi little-endian words) is a space.
__device__ __forceinline__ uint32_t space_mask8(uint32_t lo, uint32_t hi) {
    uint32_t m = 0;
    const uint32_t w[2] = {lo, hi};
#pragma unroll
    for (int d = 0; d < 2; ++d) {
        const uint32_t y = w[d] ^ 0x20202020u;                       // a space byte becomes 0
        uint32_t t = (y & 0x7F7F7F7Fu) + 0x7F7F7F7Fu;                // bit 7 of a byte set iff its low 7 bits are not 0
        t = ~(t | y | 0x7F7F7F7Fu);                                  // 0x80 exactly in the bytes that are 0
        m |= (((t >> 7) | (t >> 14) | (t >> 21) | (t >> 28)) & 0xFu) << (4 * d);
    }
    return m;
}

// The 8 bytes from index `at` on as a start mask: spaces among the bytes below `limit`.
__device__ __forceinline__ uint32_t space_starts(const EncodeParams &p, int64_t at, int64_t limit) {
    if (at >= limit) return 0u;
    const uint32_t mis = (uint32_t)((uintptr_t)p.bytes & 3);
    const uint8_t *base = p.bytes - mis;
    const uint32_t pos = (uint32_t)at + mis;
    const uint32_t first = pos & ~3u, last = ((uint32_t)p.n_bytes + mis - 1u) & ~3u;
    uint32_t raw[3];
#pragma unroll
    for (int k = 0; k < 3; ++k) raw[k] = *(const uint32_t *)(base + min(first + 4u * (uint32_t)k, last));
    const uint32_t sh = (pos & 3u) * 8u;
    const uint32_t w0 = (uint32_t)((((uint64_t)raw[1] << 32) | raw[0]) >> sh);
    const uint32_t w1 = (uint32_t)((((uint64_t)raw[2] << 32) | raw[1]) >> sh);
    const int64_t valid = limit - at;
    return space_mask8(w0, w1) & (valid >= 8 ? 0xFFu : (1u << valid) - 1u);
}

// The smallest v of the workgroup's threads, to every thread (tmp: one word per wavefront).
__device__ __forceinline__ uint32_t group_min_u32(uint32_t v, uint32_t *tmp) {
    const uint32_t w = wave_min_u32(v);
    __syncthreads();
    if (lane_id() == 0) tmp[threadIdx.x / kWave] = w;
    __syncthreads();
    return min(min(tmp[0], tmp[1]), min(tmp[2], tmp[3]));
}

__global__ void __launch_bounds__(kGroupThreads) merge_bytes_kernel(EncodeParams p) {
    __shared__ TileShared sh;
    __shared__ uint16_t starts[kByteTile];
    __shared__ uint32_t extra[kByteTile / 32];       // sequence starts inside the tile, one bit per byte
    __shared__ int wave_cnt[kWavesPerGroup], wave_tokens[kWavesPerGroup];
    __shared__ uint32_t min_tmp[kWavesPerGroup];
    const int tid = threadIdx.x, lane = lane_id(), wv = tid / kWave;
    const int tile = blockIdx.x;
    const int lo = tile * kByteTile, hi = min(lo + kByteTile, p.n_bytes);

    // The tile's bytes, and the 512 behind them (by the first wavefront: the tile's last piece ends at the
    // first start there, nearly always), are asked for before anything else: what follows waits for other
    // loads, and these then arrive meanwhile.
    uint32_t mask = tid < kByteScanThreads ? space_starts(p, (int64_t)lo + 8 * tid, hi) : 0u;
    const uint32_t ahead = wv == 0 ? space_starts(p, (int64_t)hi + 8 * tid, p.n_bytes) : 0u;

    // Sequence boundaries: every tile checks a strided share of them and finds the ones in its own
    // bytes; seq_next: the first one at or behind the tile's end (a piece ends there at the latest).
    // (A single sequence has none inside the text: its two offsets are checked by the first tile.)
    int seq_next = p.n_bytes;
    bool any_seq = false;
    if (p.seq_off && p.n_seqs == 1) {
        if (tile == 0 && tid < 2 && p.seq_off[tid] != (tid ? p.n_bytes : 0))
            __hip_atomic_store(&p.status[kStatusBadInput], p.call_id, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else if (p.seq_off) {
        bool bad = false;
        for (int64_t k = (int64_t)tile * kGroupThreads + tid; k <= p.n_seqs; k += (int64_t)gridDim.x * kGroupThreads) {
            const int sv = p.seq_off[k];
            bad |= sv < 0 || sv > p.n_bytes || (k == 0 && sv != 0) || (k == p.n_seqs && sv != p.n_bytes);
            if (k < p.n_seqs) bad |= p.seq_off[k + 1] < sv;
        }
        if (bad) __hip_atomic_store(&p.status[kStatusBadInput], p.call_id, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        int a = 0, b = p.n_seqs + 1;                 // first k with seq_off[k] >= lo
        while (a < b) {
            const int m = (a + b) >> 1;
            if (p.seq_off[m] < lo) a = m + 1; else b = m;
        }
        const int k0 = a;
        bool mine = false;
        if (k0 + tid <= p.n_seqs) {
            const int sv = p.seq_off[k0 + tid];
            mine = sv >= lo && sv < hi;
        }
        any_seq = __syncthreads_or(mine);
        if (any_seq) {
            for (int i = tid; i < kByteTile / 32; i += kGroupThreads) extra[i] = 0;
            __syncthreads();
            for (int64_t k = (int64_t)k0 + tid; k <= p.n_seqs; k += kGroupThreads) {
                const int sv = p.seq_off[k];
                if (sv < lo || sv >= hi) break;
                atomicOr(&extra[(sv - lo) >> 5], 1u << ((sv - lo) & 31));
            }
            __syncthreads();
        }
        a = k0; b = p.n_seqs + 1;                    // first k with seq_off[k] >= hi
        while (a < b) {
            const int m = (a + b) >> 1;
            if (p.seq_off[m] < hi) a = m + 1; else b = m;
        }
        if (a <= p.n_seqs) seq_next = min(max(p.seq_off[a], hi), p.n_bytes);
    }

    // Piece starts among the tile's bytes: 8 per thread.
    if (tid < kByteScanThreads) {
        if (any_seq) mask |= (extra[(8 * tid) >> 5] >> ((8 * tid) & 31)) & 0xFFu;
        if (lo == 0 && tid == 0 && p.n_bytes > 0) mask |= 1u;
    }
    const int c = __builtin_popcount(mask);
    const int inc = wave_scan_inclusive(c);
    if (lane == kWave - 1) wave_cnt[wv] = inc;
    if (wv == 0) {                 // the first start in the 512 bytes behind the tile, if there is one
        const uint64_t hit = __ballot(ahead != 0);
        if (hit) {
            const int l = __builtin_ctzll(hit);
            const int at = hi + 8 * l + __builtin_ctz((uint32_t)__builtin_amdgcn_readlane((int)ahead, l));
            if (lane == 0) min_tmp[0] = (uint32_t)at;
        } else if (lane == 0) {
            min_tmp[0] = 0xFFFFFFFFu;
        }
    }
    __syncthreads();
    const uint32_t ahead_start = min_tmp[0];
    int k = inc - c, n_t = 0;
    for (int w = 0; w < kWavesPerGroup; ++w) {
        if (w < wv) k += wave_cnt[w];
        n_t += wave_cnt[w];
    }
    for (uint32_t m = mask; m; m &= m - 1) starts[k++] = (uint16_t)(8 * tid + __builtin_ctz(m));
    if (n_t == 0) {                // (the same in every thread) no piece starts here: the bytes are an earlier tile's
        if (tid == 0) { p.tile_cnt[tile] = 0; p.tile_sum[tile] = 0; }
        return;
    }
    // Where the tile's last piece ends: at the next start behind the tile.
    int end = min(seq_next, p.n_bytes);
    if (ahead_start != 0xFFFFFFFFu) end = min(end, (int)ahead_start);
    for (int64_t at = (int64_t)hi + 8 * kWave; ahead_start == 0xFFFFFFFFu && at < end; at += 8 * kGroupThreads) {
        const uint32_t m = space_starts(p, at + 8 * tid, end);
        const uint32_t found = group_min_u32(m ? (uint32_t)(at + 8 * tid + __builtin_ctz(m)) : 0xFFFFFFFFu, min_tmp);
        if (found != 0xFFFFFFFFu) { end = (int)found; break; }
    }
    __syncthreads();               // starts[] is complete

    ByteTile bt;
    bt.starts = starts;
    bt.lo = lo;
    bt.k0 = 0;
    bt.n_t = n_t;
    bt.end_rel = end - lo;
    const int64_t q0 = (int64_t)tile * kByteTileStride;
    // the first 256 pieces: as in every other merge kernel
    const TilePiece t = merge_tile<kFromBytes>(p, sh, 0, false, 0, kWave, bt, q0);
    if (t.has_piece) {
        p.rec[t.q] = make_int2(t.cnt, t.tok0);
        p.off_out[t.q] = t.o;
    }
    int wave_total = __builtin_amdgcn_readlane(wave_scan_inclusive(t.cnt), kWave - 1);
    // More than 256 pieces start in the tile: fewer than six bytes per piece, so not word-like text (runs of
    // spaces, sequences of a few bytes).  The further ones one at a time by the whole workgroup: slow, and small.
    const EncodeParams &kp = kernel_params();
    for (int k = kGroupThreads; k < n_t; ++k) {
        __syncthreads();
        const int s0 = starts[k], s1 = k + 1 < n_t ? (int)starts[k + 1] : bt.end_rel;
        const int b = lo + s0, n = s1 - s0;
        const int cnt = n <= kp.lds_max ? encode_group_piece<int32_t *>(kp, b, n, sh.lds.group.A, sh.lds.group.B, sh.tmp)
                                        : encode_group_piece<int32_t *>(kp, b, n, kp.scratch + b, kp.scratch2 + b, sh.tmp);
        if (tid == 0) {
            kp.rec[q0 + k] = make_int2(cnt, -1);
            kp.off_out[q0 + k] = b;
            wave_total += cnt;         // (thread 0 is lane 0 of the first wavefront, whose total is the one that counts)
        }
    }
    __syncthreads();
    if (lane == 0) wave_tokens[wv] = wave_total;
    __syncthreads();
    if (tid == 0) {
        kp.tile_sum[tile] = wave_tokens[0] + wave_tokens[1] + wave_tokens[2] + wave_tokens[3];
        kp.tile_cnt[tile] = n_t;
    }
}

// De-duplication: merges the pieces of the list p.piece_map, whose length *p.n_pieces_dev the
// kernel before it left on the device (a workgroup beyond the tiles that exist returns at once).
__global__ void __launch_bounds__(kGroupThreads) merge_mapped_kernel(EncodeParams p) {
    __shared__ TileShared sh;
    __shared__ int wave_tokens[kWavesPerGroup];
    p.n_pieces = device_piece_count(p);
    if ((int)blockIdx.x < tiles_of(p)) merge_and_count_tile<kFromList>(p, sh, wave_tokens, blockIdx.x, p.n_pieces, p.P);
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
    if (tile == 0 && tid == 0) mark_call(p.status, p.call_id);

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
constexpr int kSelfScanTiles = 4095;   // up to here emit_kernel adds up the tile totals itself (beyond: tile groups, see below)
// Deep grids: the workgroups of the emit kernels take kEmitTiles tiles each (emit_tile_group).
constexpr int kEmitTiles = 4;        // measured on 7,944 tiles: 2 -> 15.1 us, 4 -> 14.0 us, 8 -> 17.2 us
constexpr int kDeepMinTiles = 4096;        // below, a quarter as many workgroups leave too few wavefronts per CU
                                           // for the copies of pieces with many tokens (stress, 2,064 tiles:
                                           // 24.4 against 19.6 us)
constexpr int kDeepSelfScanTiles = 8192;   // up to here such a workgroup adds up the tile totals itself

// Whether the merge kernel of this call had long-piece workgroups that merged anything: only then
// does long_sum hold anything to add (it is not even written otherwise).
__device__ __forceinline__ bool has_long_sums(const EncodeParams &p) {
    return p.long_sum && __builtin_amdgcn_readfirstlane(p.status[kStatusLongPieces]) == p.call_id;
}

__global__ void __launch_bounds__(kScanThreads) scan_tiles_kernel(EncodeParams p, int64_t n_tiles) {
    __shared__ LookbackTmp lb;
    __shared__ int wave_sum[kScanThreads / kWave];
    const int tid = threadIdx.x, lane = lane_id(), wv = tid / kWave;
    if (p.n_pieces_dev) {          // raw path: only the tiles that exist; small grids add up by themselves in emit_kernel
        raw_geometry(p);
        n_tiles = tiles_of(p);
        if (n_tiles <= kSelfScanTiles || (n_tiles >= kDeepMinTiles && n_tiles <= kDeepSelfScanTiles)) return;
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
    if (has_long_sums(p)) {
#pragma unroll
        for (int j = 0; j < kPerThread; ++j) v[j] += i0 + j < n_tiles ? p.long_sum[i0 + j] : 0;
    }
    int mine = 0;
#pragma unroll
    for (int j = 0; j < kPerThread; ++j) mine += v[j];
    const int inc = wave_scan_inclusive(mine);
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
        if (p.out_offsets) p.out_offsets[p.n_pieces] = before + total;
        mark_call(p.status, p.call_id);
    }
}

// Dense copy of one piece's c tokens to out_ids[first ...]: the first one travels in the
// record (tok0 >= 0), the others wait in scratch at the piece's byte offset o.  Every lane of
// the wavefront must call it (c = 0 without a piece).
// How many of a piece's c tokens can be copied from scratch[o ...] to out_ids[first ...]: bad offsets can
// make pieces overlap and the total exceed the capacity of out_ids; then they must still not become
// bad addresses.
__device__ __forceinline__ int copy_count(const EncodeParams &p, int c, int o, int first) {
    const int room = first >= 0 && first < p.n_bytes ? p.n_bytes - first : 0;
    const int src_room = o >= 0 && o < p.n_bytes ? p.n_bytes - o : 0;
    return min(c, min(room, src_room));
}

// Tokens [from, n) of a piece, by the T threads of which this is number t: four loads in flight per thread.
template <int T>
__device__ __forceinline__ void copy_tokens(const EncodeParams &p, int src, int dst, int from, int n, int t) {
    for (int i = from + t; i < n; i += 4 * T) {
        int v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = i + u * T < n ? p.scratch[src + i + u * T] : 0;
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (i + u * T < n) p.out_ids[dst + i + u * T] = v[u];
    }
}

// Dense copy of one piece's c tokens to out_ids[first ...]: the first one travels in the
// record (tok0 >= 0), the others wait in scratch at the piece's byte offset o.  Every lane of
// the wavefront must call it (c = 0 without a piece).  wave_limit: the wavefront leaves the
// tokens from the eighth on to somebody else if the piece has more than this many.
__device__ __forceinline__ void emit_piece_tokens(const EncodeParams &p, int c, int tok0, int o, int first,
                                                  int wave_limit = 0x7FFFFFFF) {
    const int lane = lane_id();
    const int n_copy = copy_count(p, c, o, first);
    // most pieces are one or two tokens: each thread copies the first 8 of its own
    // piece, the wavefront shares the rest of the rare longer ones
    if (n_copy > 0) p.out_ids[first] = tok0 >= 0 ? tok0 : p.scratch[o];
    for (int i = 1; i < 8; ++i) {
        if (!__ballot(i < n_copy)) break;
        if (i < n_copy) p.out_ids[first + i] = p.scratch[o + i];
    }
    for (uint64_t m = __ballot(n_copy > 8 && n_copy <= wave_limit); m;) {
        const int t = __builtin_ctzll(m);
        m &= m - 1;
        copy_tokens<kWave>(p, read_lane(o, t), read_lane(first, t), 8, read_lane(n_copy, t), lane);
    }
}

// Pieces of a tile that keep thousands of tokens (a long run of a byte that merges little): the whole
// workgroup copies them, a few per tile at most.
constexpr int kGroupCopyMin = 1024, kGroupCopyMax = 8;
struct GroupCopies {
    int n;
    int src[kGroupCopyMax], dst[kGroupCopyMax], count[kGroupCopyMax];
};

// out_offsets of the tile's pieces and the dense copy of their tokens.  With
// self_scan the tile adds up the totals of all tiles before it by itself (for a
// grid of up to kSelfScanTiles tiles that costs less than a scan kernel launch, even an empty one).

// firsts (LDS, or nullptr): gets the first token's index of the tile's piece number i at [i];
// end: the number of tokens up to and including this tile.
// big (LDS, or nullptr): where the workgroup notes pieces of more than kGroupCopyMin tokens to copy them together.
__device__ __forceinline__ void emit_tile(const EncodeParams &p, GroupTmp &tmp, int *before_w, int tile, int last_tile,
                                          int self_scan, int *firsts, int &end, GroupCopies *big = nullptr) {
    const int tid = threadIdx.x, lane = lane_id(), wv = tid / kWave;
    // The record of the thread's piece and the totals of the tiles before this one are both
    // cold in the caches: the loads go out together, and one barrier serves both sums.
    // (pieces of the tile; the paper's kernels have one piece per tile)
    const int64_t q = p.paper ? tile : ((int64_t)tile * p.W + wv) * p.P + lane;
    const bool has_piece = (p.paper ? tid == 0 : (lane < p.P && wv < p.W)) && q < p.n_pieces;
    int c = 0, o = 0, tok0 = -1;
    if (has_piece) { const int2 r = p.rec[q]; c = r.x; tok0 = r.y; }
    int before = 0;
    const bool long_sums = self_scan && has_long_sums(p);
    if (self_scan) {               // tile_sum is 256-byte aligned and has room for a tile total per piece
        for (int t = tid * 4; t < tile; t += kGroupThreads * 4) {
            const int4 a = *(const int4 *)(p.tile_sum + t);
            before += a.x + (t + 1 < tile ? a.y : 0) + (t + 2 < tile ? a.z : 0) + (t + 3 < tile ? a.w : 0);
            if (long_sums) {
                const int4 b = *(const int4 *)(p.long_sum + t);
                before += b.x + (t + 1 < tile ? b.y : 0) + (t + 2 < tile ? b.z : 0) + (t + 3 < tile ? b.w : 0);
            }
        }
    } else if (tid == 0) {
        before = p.tile_base[tile];
    }
    if (c < 0) c = 0;
    if (c > 1 || (c == 1 && tok0 < 0)) o = p.off[p.rep_of ? p.rep_of[q] : q];     // only then is anything of the piece in scratch
    const int inc = wave_scan_inclusive(c);
    before = __builtin_amdgcn_readlane(wave_scan_inclusive(before), kWave - 1);
    if (lane == kWave - 1) tmp.sum_w[wv] = inc;
    if (lane == 0) before_w[wv] = before;
    __syncthreads();
    int base = 0, ex = inc - c, total = 0;
    for (int w = 0; w < kWavesPerGroup; ++w) {
        base += before_w[w];
        if (w < wv) ex += tmp.sum_w[w];
        total += tmp.sum_w[w];
    }
    const int first = base + ex;
    end = base + total;
    if (has_piece) p.out_offsets[q] = first;
    if (firsts && has_piece) firsts[wv * p.P + lane] = first;
    if (self_scan && tid == 0) {
        if (tile == last_tile) p.out_offsets[p.n_pieces] = base + total;
        if (tile == 0) mark_call(p.status, p.call_id);
    }
    if (!big || total <= kGroupCopyMin) {          // (the same in every thread) no piece of this tile is that large
        emit_piece_tokens(p, c, tok0, o, first);
        return;
    }
    if (tid == 0) big->n = 0;
    __syncthreads();
    const int n_copy = copy_count(p, c, o, first);
    bool handed_on = false;
    if (n_copy > kGroupCopyMin) {
        const int slot = atomicAdd(&big->n, 1);
        if (slot < kGroupCopyMax) {
            big->src[slot] = o; big->dst[slot] = first; big->count[slot] = n_copy;
            handed_on = true;
        }
    }
    emit_piece_tokens(p, c, tok0, o, first, handed_on ? 8 : 0x7FFFFFFF);
    __syncthreads();
    const int n_big = min(big->n, kGroupCopyMax);
    for (int e = 0; e < n_big; ++e) copy_tokens<kGroupThreads>(p, big->src[e], big->dst[e], 8, big->count[e], tid);
}

__global__ void __launch_bounds__(kGroupThreads) emit_kernel(EncodeParams p, int self_scan) {
    __shared__ GroupTmp tmp;
    __shared__ int before_w[kWavesPerGroup];
    __shared__ GroupCopies big;
    int end;
    emit_tile(p, tmp, before_w, blockIdx.x, gridDim.x - 1, self_scan, nullptr, end, &big);
}

// Deep grids: a workgroup takes kEmitTiles consecutive tiles.  One tile per workgroup is
// four dependent round trips for 256 pieces, and with 31 tiles per CU (7,944 in all) the
// kernel is as many rounds of that latency; here a thread has the records of its
// kEmitTiles pieces in flight together, and the whole grid is resident at once.  With
// self_scan the workgroup adds up the totals of the tiles before its own (16-byte loads that
// travel with the records), which spares the launch of scan_tiles_kernel.

struct EmitDeepTmp {
    int before_w[kWavesPerGroup];
    int sum_w[kEmitTiles][kWavesPerGroup];
};

// Tiles group * kEmitTiles ... of the n_tiles there are.
__device__ __forceinline__ void emit_tile_group(const EncodeParams &p, EmitDeepTmp &tmp, int group, int n_tiles,
                                                int self_scan) {
    int (&before_w)[kWavesPerGroup] = tmp.before_w;
    int (&sum_w)[kEmitTiles][kWavesPerGroup] = tmp.sum_w;
    const int tid = threadIdx.x, lane = lane_id(), wv = tid / kWave;
    const int tile0 = group * kEmitTiles;
    int64_t q[kEmitTiles];
    int c[kEmitTiles], tok0[kEmitTiles];
    bool has_piece[kEmitTiles];
#pragma unroll
    for (int i = 0; i < kEmitTiles; ++i) {
        q[i] = ((int64_t)(tile0 + i) * p.W + wv) * p.P + lane;
        has_piece[i] = tile0 + i < n_tiles && lane < p.P && wv < p.W && q[i] < p.n_pieces;
        c[i] = 0;
        tok0[i] = -1;
        if (has_piece[i]) { const int2 r = p.rec[q[i]]; c[i] = max(r.x, 0); tok0[i] = r.y; }
    }
    int o[kEmitTiles];
#pragma unroll
    for (int i = 0; i < kEmitTiles; ++i)       // only then is anything of the piece in scratch
        o[i] = c[i] > 1 || (c[i] == 1 && tok0[i] < 0) ? p.off[p.rep_of ? p.rep_of[q[i]] : q[i]] : 0;
    if (self_scan) {               // tile_sum is 256-byte aligned and has room for a tile total per piece
        int before = 0;
        const bool long_sums = has_long_sums(p);
        for (int t = tid * 4; t < tile0; t += kGroupThreads * 4) {
            const int4 a = *(const int4 *)(p.tile_sum + t);
            before += a.x + (t + 1 < tile0 ? a.y : 0) + (t + 2 < tile0 ? a.z : 0) + (t + 3 < tile0 ? a.w : 0);
            if (long_sums) {
                const int4 b = *(const int4 *)(p.long_sum + t);
                before += b.x + (t + 1 < tile0 ? b.y : 0) + (t + 2 < tile0 ? b.z : 0) + (t + 3 < tile0 ? b.w : 0);
            }
        }
        before = __builtin_amdgcn_readlane(wave_scan_inclusive(before), kWave - 1);
        if (lane == 0) before_w[wv] = before;
    }
    int inc[kEmitTiles];
#pragma unroll
    for (int i = 0; i < kEmitTiles; ++i) {
        inc[i] = wave_scan_inclusive(c[i]);
        if (lane == kWave - 1) sum_w[i][wv] = inc[i];
    }
    __syncthreads();
    int base = 0;
    if (self_scan) {
        for (int w = 0; w < kWavesPerGroup; ++w) base += before_w[w];
    } else {
        base = p.tile_base[tile0];
    }
#pragma unroll
    for (int i = 0; i < kEmitTiles; ++i) {
        int ex = inc[i] - c[i], total = 0;
        for (int w = 0; w < kWavesPerGroup; ++w) {
            if (w < wv) ex += sum_w[i][w];
            total += sum_w[i][w];
        }
        const int first = base + ex;
        if (has_piece[i]) p.out_offsets[q[i]] = first;
        emit_piece_tokens(p, c[i], tok0[i], o[i], first);
        base += total;
    }
    if (self_scan && tid == 0) {
        if (tile0 + kEmitTiles >= n_tiles) p.out_offsets[p.n_pieces] = base;
        if (group == 0) mark_call(p.status, p.call_id);
    }
}

__global__ void __launch_bounds__(kGroupThreads) emit_deep_kernel(EncodeParams p, int n_tiles, int self_scan) {
    __shared__ EmitDeepTmp tmp;
    emit_tile_group(p, tmp, blockIdx.x, n_tiles, self_scan);
}

// Raw path: up to this many sequences, and on grids sized for fewer than kDeepMinTiles tiles, the
// emit kernel (emit_raw_seq_kernel) also writes the first token of every sequence (a launch less: 21.0 -> 19.2 us on 131 k
// tokens); otherwise seq_token_offsets_kernel does (on 7,944 tiles and 256 sequences the two
// extra barriers per workgroup cost more than the launch: 120.8 against 119.1 us).
constexpr int kSeqFoldMax = 1023;
__device__ __host__ inline bool seq_offsets_by_emit(int n_seqs, int64_t n_tiles) {
    return n_seqs <= kSeqFoldMax && n_tiles < kDeepMinTiles;
}

// The first token of every sequence whose first piece is one of the n_here pieces from q_lo
// on; firsts[i] (LDS) = index of the first token of piece q_lo + i.  The workgroup of the last
// tile also serves the sequences that start behind the last piece (empty ones at the end, and
// the closing entry): `end` tokens in all.  Every workgroup looks through all entries; a thread
// keeps its share of them (first piece of sequence threadIdx.x + k * 256, or -1) in registers
// from the start of the kernel, so that nothing is loaded here.
constexpr int kSeqPerThread = (kSeqFoldMax + 1 + kGroupThreads - 1) / kGroupThreads;
__device__ __forceinline__ void emit_seq_offsets(const EncodeParams &p, const int *firsts, const int (&fp)[kSeqPerThread],
                                                 int64_t q_lo, int n_here, bool last, int end) {
#pragma unroll
    for (int k = 0; k < kSeqPerThread; ++k) {
        const int s = threadIdx.x + k * kGroupThreads;
        if (fp[k] >= q_lo && fp[k] < q_lo + n_here) p.seq_token_offsets[s] = firsts[fp[k] - q_lo];
        else if (last && fp[k] == p.n_pieces) p.seq_token_offsets[s] = end;
    }
}

// Raw path: workgroups stride over the tiles that exist (tile 0 always does: it
// also reports "no piece at all").
__global__ void __launch_bounds__(kGroupThreads) emit_raw_kernel(EncodeParams p) {
    __shared__ GroupTmp tmp;
    __shared__ int before_w[kWavesPerGroup];
    __shared__ GroupCopies big;
    raw_geometry(p);
    const int n_tiles = tiles_of(p);
    const int last_tile = max(n_tiles, 1) - 1;
    int end;
    if (n_tiles >= kDeepMinTiles) {        // deep grid: four tiles at a time
        __shared__ EmitDeepTmp deep_tmp;
        const int n_groups = (n_tiles + kEmitTiles - 1) / kEmitTiles;
        for (int group = blockIdx.x; group < n_groups; group += gridDim.x) {
            emit_tile_group(p, deep_tmp, group, n_tiles, n_tiles <= kDeepSelfScanTiles);
            __syncthreads();   // the next group reuses the LDS
        }
        return;
    }
    const int self_scan = n_tiles <= kSelfScanTiles;
    for (int tile = blockIdx.x; tile <= last_tile; tile += gridDim.x) {
        emit_tile(p, tmp, before_w, tile, last_tile, self_scan, nullptr, end, &big);
        __syncthreads();   // the next tile reuses the LDS
    }
}

// The same for a grid sized for fewer than kDeepMinTiles tiles and at most kSeqFoldMax
// sequences: the workgroups also write the first token of every sequence (see seq_offsets_by_emit).
__global__ void __launch_bounds__(kGroupThreads) emit_raw_seq_kernel(EncodeParams p) {
    __shared__ GroupTmp tmp;
    __shared__ int before_w[kWavesPerGroup];
    __shared__ GroupCopies big;
    __shared__ int firsts[kGroupThreads];
    raw_geometry(p);
    const int n_tiles = tiles_of(p);          // below kDeepMinTiles: the host's bound was
    const int last_tile = max(n_tiles, 1) - 1;
    const int per_tile = p.W * p.P;
    int fp[kSeqPerThread];
#pragma unroll
    for (int k = 0; k < kSeqPerThread; ++k) {
        const int s = threadIdx.x + k * kGroupThreads;
        fp[k] = s <= p.n_seqs ? min(max(p.seq_first_piece[s], 0), p.n_pieces) : -1;
    }
    const int self_scan = n_tiles <= kSelfScanTiles;
    int end = 0;
    for (int tile = blockIdx.x; tile <= last_tile; tile += gridDim.x) {
        emit_tile(p, tmp, before_w, tile, last_tile, self_scan, firsts, end, &big);
        __syncthreads();   // firsts is complete (and the next tile reuses the LDS)
        const int64_t q_lo = (int64_t)tile * per_tile;
        emit_seq_offsets(p, firsts, fp, q_lo, (int)max(min((int64_t)per_tile, (int64_t)p.n_pieces - q_lo), (int64_t)0),
                         tile == last_tile, end);
        __syncthreads();
    }
}

// Assembly for merge_bytes_kernel: the tokens of the pieces that start in a tile of bytes, and the
// first token of every sequence that starts there.  One tile per workgroup; 256 pieces at a time.
__global__ void __launch_bounds__(kGroupThreads) emit_bytes_kernel(EncodeParams p, int n_tiles, int self_scan) {
    __shared__ GroupTmp tmp;
    __shared__ int before_w[kWavesPerGroup];
    const int tid = threadIdx.x, lane = lane_id(), wv = tid / kWave;
    const int tile = blockIdx.x;
    const int lo = tile * kByteTile, hi = min(lo + kByteTile, p.n_bytes);
    const int n_t = min(max(p.tile_cnt[tile], 0), kByteTile);
    const int64_t q0 = (int64_t)tile * kByteTileStride;
    if (tile == 0 && tid == 0) mark_call(p.status, p.call_id);
    // tokens before the tile
    int before = 0;
    if (self_scan) {               // tile_sum is 256-byte aligned
        for (int t = tid * 4; t < tile; t += kGroupThreads * 4) {
            const int4 a = *(const int4 *)(p.tile_sum + t);
            before += a.x + (t + 1 < tile ? a.y : 0) + (t + 2 < tile ? a.z : 0) + (t + 3 < tile ? a.w : 0);
        }
    } else if (tid == 0) {
        before = p.tile_base[tile];
    }
    before = __builtin_amdgcn_readlane(wave_scan_inclusive(before), kWave - 1);
    // the sequences that start among the tile's bytes: seq_off[s0 .. s1)
    int s0 = 0, s1 = 0;
    if (p.seq_off) {
        int a = 0, b = p.n_seqs + 1;
        while (a < b) { const int m = (a + b) >> 1; if (p.seq_off[m] < lo) a = m + 1; else b = m; }
        s0 = a;
        b = p.n_seqs + 1;
        while (a < b) { const int m = (a + b) >> 1; if (p.seq_off[m] < hi) a = m + 1; else b = m; }
        s1 = a;
    }
    int base = 0;
    for (int k0 = 0; k0 < max(n_t, 1); k0 += kGroupThreads) {
        const bool has_piece = k0 + tid < n_t;
        int c = 0, tok0 = -1, o = -1;
        if (has_piece) { const int2 r = p.rec[q0 + k0 + tid]; c = max(r.x, 0); tok0 = r.y; }
        if (has_piece && (c > 1 || (c == 1 && tok0 < 0) || s1 > s0)) o = p.off[q0 + k0 + tid];
        const int inc = wave_scan_inclusive(c);
        __syncthreads();           // (the arrays of the round before are read)
        if (lane == kWave - 1) tmp.sum_w[wv] = inc;
        if (lane == 0 && k0 == 0) before_w[wv] = before;
        __syncthreads();
        int ex = inc - c, total = 0;
        if (k0 == 0) for (int w = 0; w < kWavesPerGroup; ++w) base += before_w[w];
        for (int w = 0; w < kWavesPerGroup; ++w) {
            if (w < wv) ex += tmp.sum_w[w];
            total += tmp.sum_w[w];
        }
        const int first = base + ex;
        emit_piece_tokens(p, c, tok0, max(o, 0), first);
        // a sequence starts where one of these pieces starts: its first token is that piece's
        for (int s = s0; s < s1; ++s)
            if (has_piece && o == p.seq_off[s]) p.seq_token_offsets[s] = first;
        base += total;
    }
    if (tile == n_tiles - 1 && tid == 0) {
        // the total, for the closing entry and for sequences that start behind the last byte
        if (!p.seq_off) { p.seq_token_offsets[0] = 0; p.seq_token_offsets[1] = base; }
        else for (int s = p.n_seqs; s >= 0 && p.seq_off[s] >= p.n_bytes; --s) p.seq_token_offsets[s] = base;
    }
}

// Raw path, last kernel: the first token of every sequence.
__global__ void __launch_bounds__(kGroupThreads) seq_token_offsets_kernel(EncodeParams p) {
    const int n_pieces = device_piece_count(p);
    const int k = blockIdx.x * kGroupThreads + threadIdx.x;
    if (k <= p.n_seqs) p.seq_token_offsets[k] = p.out_offsets[min(max(p.seq_first_piece[k], 0), n_pieces)];
}

struct Layout {
    int64_t status, rec, tile_sum, long_sum, tile_base, tile_state, scratch, scratch2, total;
};

static int64_t align256(int64_t v) { return (v + 255) & ~255ll; }

static Layout workspace_layout(int64_t n_bytes, int64_t n_pieces) {
    Layout l;
    const int64_t max_tiles = n_pieces + 1;      // a tile can be a single piece
    int64_t at = 0;
    l.status = at;    at += 256;
    l.rec = at;       at += align256(8 * (n_pieces + 1));
    l.tile_sum = at;  at += align256(4 * (n_pieces + 1));   // the paper's kernels have one piece per tile
    l.long_sum = at;  at += align256(4 * (n_pieces / kGroupThreads + 2));
    l.tile_base = at; at += align256(4 * (n_pieces + 1));
    l.tile_state = at; at += align256(8 * max_tiles);
    l.scratch = at;   at += align256(4 * (n_bytes + 1));
    l.scratch2 = at;  at += align256(4 * (n_bytes + 1));
    l.total = at;
    return l;
}

// De-duplication: the encode layout, then the set of pieces seen, the representatives and
// the records of all pieces.
struct DedupLayout {
    Layout enc;
    int64_t set, rep, tile_reps, piece_map, dense_of, n_reps, rec_all, total;
    int64_t set_slots;
};

static DedupLayout dedup_layout(int64_t n_bytes, int64_t n_pieces) {
    DedupLayout d;
    d.enc = workspace_layout(n_bytes, n_pieces);
    int64_t slots = 1024;
    while (slots < 2 * n_pieces) slots *= 2;       // at most half full
    d.set_slots = slots;
    int64_t at = d.enc.total;
    d.set = at;       at += align256(4 * slots);
    d.rep = at;       at += align256(4 * (n_pieces + 1));
    d.tile_reps = at; at += align256(4 * (n_pieces / kGroupThreads + 2));
    d.piece_map = at; at += align256(4 * (n_pieces + 1));
    d.dense_of = at;  at += align256(4 * (n_pieces + 1));
    d.n_reps = at;    at += 256;
    d.rec_all = at;   at += align256(8 * (n_pieces + 1));
    d.total = at;
    return d;
}

// Raw path: the encode layout for max_pieces pieces, then what the pre-tokenizer
// needs and the piece arrays the caller did not bring.
struct RawLayout {
    Layout enc;
    int64_t pretok_state, seq_first_piece, piece_offsets, out_offsets, n_pieces, total;
    int64_t byte_rec, byte_off, byte_cnt;     // the path without a pre-tokenizer launch (-1: no room was asked for)
};

static int64_t byte_tiles(int64_t n_bytes) { return std::max<int64_t>((n_bytes + kByteTile - 1) / kByteTile, 1); }

static RawLayout raw_layout(int64_t n_bytes, int64_t max_pieces, int64_t n_seqs) {
    RawLayout r;
    r.enc = workspace_layout(n_bytes, max_pieces);
    int64_t at = r.enc.total;
    r.pretok_state = at;    at += align256(pretokenize_state_bytes(n_bytes));
    r.seq_first_piece = at; at += align256(4 * (n_seqs + 2));
    r.piece_offsets = at;   at += align256(4 * (max_pieces + 1));
    r.out_offsets = at;     at += align256(4 * (max_pieces + 1));
    r.n_pieces = at;        at += 256;
    // Tokens only, no piece arrays (the workgroups find the pieces in their bytes): a record and a first
    // byte per slot, kByteTileStride slots per tile.  Only with the default capacity (max_pieces = n_bytes):
    // a caller who sizes the workspace for fewer pieces wants the piece arrays.
    r.byte_rec = r.byte_off = r.byte_cnt = -1;
    if (max_pieces >= n_bytes) {
        const int64_t slots = byte_tiles(n_bytes) * kByteTileStride + 1;
        r.byte_rec = at; at += align256(8 * slots);
        r.byte_off = at; at += align256(4 * slots);
        r.byte_cnt = at; at += align256(4 * byte_tiles(n_bytes));
    }
    r.total = at;
    return r;
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

extern "C" int64_t bpe_dedup_workspace_bytes(int64_t n_bytes, int64_t n_pieces) {
    const int64_t base = bpe_workspace_bytes(n_bytes, n_pieces);
    if (base < 0) return base;
    return dedup_layout(n_bytes, n_pieces).total;
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

// Every kernel of the encode paths is enqueued through this: it notes the launch in the
// caller's plan (bpe_encode_plan, the *_timed calls) and, unless the call only asks what
// would be launched, launches it.  hipLaunchKernel reports the error of this very launch;
// an earlier error of the calling thread is neither picked up nor cleared.
struct Launcher {
    bpe_encode_plan_t *plan;   // nullptr: nobody asked
    bool dry;                  // true: note only
    hipStream_t s;
    hipError_t err = hipSuccess;

    void note(const char *name, int interval, int64_t grid, int block) {
        if (!plan || plan->n_launches >= BPE_PLAN_MAX_LAUNCHES) return;
        auto &l = plan->launch[plan->n_launches++];
        snprintf(l.kernel, sizeof(l.kernel), "%s", name);
        l.grid = grid;
        l.block = block;
        l.interval = interval;
    }
    template <typename... KArgs, size_t... I>
    hipError_t call(void (*kernel)(KArgs...), int64_t grid, int block, std::tuple<KArgs...> &a, std::index_sequence<I...>) {
        void *ptrs[] = {(void *)&std::get<I>(a)...};
        return hipLaunchKernel((const void *)kernel, dim3((unsigned)grid), dim3((unsigned)block), ptrs, 0, s);
    }
    // interval: which of the *_timed intervals the launch falls into
    template <typename... KArgs, typename... Args>
    void run(const char *name, int interval, void (*kernel)(KArgs...), int64_t grid, int block, Args... args) {
        note(name, interval, grid, block);
        if (dry || err != hipSuccess) return;
        std::tuple<KArgs...> a(args...);
        err = call(kernel, grid, block, a, std::index_sequence_for<KArgs...>{});
    }
};

// Validates, fills the kernel parameters and enqueues the kernels.  With `ev` an
// event is recorded before the first kernel and after each: kKernels + 1 events,
// kRawKernels + 1 on the raw path.  With `dry` nothing is launched and no pointer is
// looked at: the call only fills `plan`.
constexpr int kKernels = 3;
constexpr int kRawKernels = 5;
constexpr int64_t kRawMaxGrid = 8192;   // raw path: workgroups of the merge and emit kernels
constexpr int64_t kRawRestGrid = 2048;  // ... of the strided merge kernel (two rounds of the chip; mostly it finds nothing to do)
// Workgroups of the merge kernels that the chip holds at a time (4 per compute unit: LDS).  The
// single-kernel path is only free of deadlock by construction while every tile is resident;
// beyond, it relies on workgroups being dispatched in index order.
constexpr int64_t kResidentGroups = 1024;
// merge_kernel: one workgroup for the long pieces of every so many tiles, from grids of so many tiles on
// (more than the chip holds at a time: below, a tile that takes long holds no other tile up),
// and at most so many of them (then each takes more tiles; at most 256, the reach of a list entry)
constexpr int64_t kTilesPerLongGroup = 4, kLongGroupsMinTiles = kLongGroupsMinTilesDevice, kMaxLongGroups = 65536;

static int launch_encode(const bpe_table *table, const uint8_t *bytes, const int32_t *piece_offsets,
                         int64_t n_bytes, int64_t n_pieces, int32_t *out_ids, int32_t *out_offsets,
                         void *workspace, int64_t workspace_bytes, const bpe_encode_options *opts,
                         hipStream_t s, hipEvent_t *ev, const RawArgs *raw = nullptr,
                         bpe_encode_plan_t *plan = nullptr, bool dry = false) {
    if (!dry && (!table || (n_bytes > 0 && (!bytes || !out_ids)) ||
                 (raw ? !raw->seq_token_offsets : (!piece_offsets || !out_offsets)))) {
        set_error("null pointer");
        return BPE_ERR_NULL;
    }
    const bool dedup = opts && opts->dedup == 1;
    const int64_t need = raw ? bpe_encode_raw_workspace_bytes(n_bytes, n_pieces, raw->n_seqs)
                       : dedup ? bpe_dedup_workspace_bytes(n_bytes, n_pieces) : bpe_workspace_bytes(n_bytes, n_pieces);
    if (need < 0) return (int)need;
    if (!dry && (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < need)) {
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
    if (o.column_max_len == 0) o.column_max_len = kColumnMax;
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
        else if (avg > kTinyMax) {
            const int64_t most = std::max<int64_t>((kWave * kTinyMax) / avg, 1);
            ppw = std::max<int64_t>(std::min<int64_t>(n_pieces / 4096, most), 1);
            // The chip holds kResidentGroups such workgroups at a time.  A grid that is
            // two or three rounds of them with only a sliver in the last one waits for
            // that sliver (64-byte pieces: 1,095 tiles 121 us, 821 tiles 109 us): then
            // a few more pieces per wavefront, one round less.
            auto tiles = [&](int64_t q) { return (n_pieces + kWavesPerGroup * q - 1) / (kWavesPerGroup * q); };
            const int64_t rounds = (tiles(ppw) + kResidentGroups - 1) / kResidentGroups;
            if (rounds >= 2 && rounds <= 3 && tiles(ppw) * 20 <= (rounds - 1) * kResidentGroups * 23)
                while (ppw < most && tiles(ppw) > (rounds - 1) * kResidentGroups) ++ppw;
        }
        o.pieces_per_wave = (int32_t)ppw;
    }
    if (o.selection_level < 1 || o.selection_level > 3 || o.pieces_per_wave < -1 || o.pieces_per_wave == 0 || o.pieces_per_wave > kWave ||
        o.tiny_max_len < -1 || o.tiny_max_len > kTinyMax || o.wave_max_len < -1 || o.wave_max_len > kWave ||
        o.column_max_len < -1 || o.column_max_len > kColumnMax ||
        o.wave_lds_max_len < -1 || o.wave_lds_max_len > kWaveLdsMax ||
        o.lds_max_len < 1 || o.lds_max_len > kLdsMaxLen || o.fused < -1 || o.fused > 2 ||
        !pretokenize_tile_ok(o.pretokenize_tile_kib) || o.paper_kernel < 0 || o.paper_kernel > 2 ||
        (o.paper_kernel && raw) || o.dedup < 0 || o.dedup > 1 || o.long_groups < -1 || o.long_groups > 256) {
        set_error("option out of range");
        return BPE_ERR_OPTION;
    }
    if (o.dedup && (raw || o.paper_kernel || o.fused > 0 || o.pieces_per_wave != kWave)) {
        set_error("dedup = 1 needs bpe_encode on word-sized pieces (pieces_per_wave 64), and neither fused > 0 nor paper_kernel");
        return BPE_ERR_OPTION;
    }
    if (o.tiny_max_len < 0) o.tiny_max_len = 0;      // -1 switches a path off
    if (o.column_max_len < 0) o.column_max_len = 0;
    if (o.wave_max_len < 0) o.wave_max_len = 0;
    if (o.wave_lds_max_len < 0) o.wave_lds_max_len = 0;

    if (!dry) {
        const int dev_rc = check_device(table->device, "the table");
        if (dev_rc != BPE_OK) return dev_rc;
    }
    const Layout l = workspace_layout(n_bytes, n_pieces);
    // (offsets into the workspace as integers: a call that only plans has no workspace)
    auto ws_at = [workspace](int64_t off) { return (char *)((uintptr_t)workspace + (uintptr_t)off); };
    EncodeParams p = {};     // no kernel parameter is ever left unset
    p.call_id = dry ? 0 : next_call_id();
    p.P = o.pieces_per_wave > 0 ? o.pieces_per_wave : 1;
    p.W = o.pieces_per_wave > 0 ? kWavesPerGroup : 1;
    p.paper = o.paper_kernel;
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
    if (o.fused == 1 && !raw && !p.paper && (n_tiles > kResidentGroups || !short_pieces)) {
        set_error("fused = 1 is limited to grids of at most %lld tiles (this call: %lld) of pieces that average at most "
                  "%d bytes: beyond, a tile may wait for one that is not resident yet, which only ends because "
                  "workgroups are dispatched in index order; fused = 2 accepts that", (long long)kResidentGroups,
                  (long long)n_tiles, kWave);
        return BPE_ERR_OPTION;
    }
    const bool fused = !raw && !p.paper && !o.dedup && n_tiles > 0 &&
                       (o.fused > 0 || (o.fused == 0 && n_tiles <= kFusedMaxTiles && short_pieces));
    if (plan) {
        *plan = {};
        plan->single_kernel = fused;
        plan->pieces_per_wave = p.P;
        plan->waves_per_tile = p.W;
        plan->n_tiles = n_tiles;
        plan->selection_level = o.selection_level;
    }
    Launcher run{plan, dry, s};
    int n_ev = 0;
    if (ev) (void)hipEventRecord(ev[n_ev++], s);
    // bpe_encode_raw for tokens only (no piece array asked for, default capacity, tiles left to the library):
    // no pre-tokenizer launch, the merge workgroups find the pieces in their bytes
    bool byte_tiles_path = false;
    if (raw) {
        const RawLayout r = raw_layout(n_bytes, n_pieces, raw->n_seqs);
        // ... while the chip holds all the tiles at once: then the call is as long as its chain of dependent
        // steps, and a launch less shortens it (840 KB: 19.6 -> 15.8 us).  A deeper grid is bound by instruction
        // issue, and tiles of a fixed number of bytes leave a quarter of the lanes idle (13.5 MB: 122 -> 154 us).
        byte_tiles_path = !raw->piece_offsets && !out_offsets && !raw->n_pieces && raw_auto_P && o.fused >= 0 &&
                          r.byte_rec >= 0 && byte_tiles(n_bytes) <= kResidentGroups;
    }
    if (byte_tiles_path) {
        if (ev) (void)hipEventRecord(ev[n_ev++], s);      // (the pre-tokenizer's interval: empty)
        p.seq_off = raw->seq_offsets;
        p.seq_token_offsets = raw->seq_token_offsets;
        p.n_seqs = raw->seq_offsets ? (int32_t)raw->n_seqs : 1;
    } else if (raw) {
        const RawLayout r = raw_layout(n_bytes, n_pieces, raw->n_seqs);
        int32_t *piece_off = raw->piece_offsets ? raw->piece_offsets : (int32_t *)ws_at(r.piece_offsets);
        int32_t *n_dev = raw->n_pieces ? raw->n_pieces : (int32_t *)ws_at(r.n_pieces);
        int32_t *first = (int32_t *)ws_at(r.seq_first_piece);
        if (!out_offsets) out_offsets = (int32_t *)ws_at(r.out_offsets);
        int64_t pre_grid = 0;
        const int rc = launch_pretokenize(bytes, n_bytes, raw->seq_offsets, raw->n_seqs, piece_off, n_pieces, n_dev,
                                          first, (int32_t *)ws_at(l.status),
                                          (unsigned long long *)ws_at(r.pretok_state), p.call_id,
                                          o.pretokenize_tile_kib, s, &pre_grid, dry);
        if (rc != BPE_OK) return rc;
        run.note("pretokenize_kernel", 0, pre_grid, kGroupThreads);
        if (ev) (void)hipEventRecord(ev[n_ev++], s);
        piece_offsets = piece_off;
        p.n_pieces_dev = n_dev;
        p.seq_first_piece = first;
        p.seq_token_offsets = raw->seq_token_offsets;
        p.n_seqs = raw->seq_offsets ? (int32_t)raw->n_seqs : 1;
    }
    if (!dry) p.table = table->view;
    p.bytes = bytes;
    p.off = piece_offsets;
    p.n_bytes = (int32_t)n_bytes;
    p.n_pieces = (int32_t)n_pieces;
    p.raw_auto_P = raw_auto_P;
    p.tiny_max = o.tiny_max_len;
    p.col_max = std::max(o.column_max_len, o.tiny_max_len);
    p.wave_max = std::max(o.wave_max_len, p.col_max);
    p.wave_lds_max = std::max(o.wave_lds_max_len, p.wave_max);
    p.lds_max = o.lds_max_len;
    p.level = o.selection_level;
    p.runs_by_best_rank = auto_level;
    p.rec = (int2 *)ws_at(l.rec);
    p.tile_sum = (int32_t *)ws_at(l.tile_sum);
    p.tile_base = (int32_t *)ws_at(l.tile_base);
    p.scratch = (int32_t *)ws_at(l.scratch);
    p.scratch2 = (int32_t *)ws_at(l.scratch2);
    p.status = (int32_t *)ws_at(l.status);
    p.tile_state = (unsigned long long *)ws_at(l.tile_state);
    p.out_ids = out_ids;
    p.out_offsets = out_offsets;

    const int i0 = raw ? 1 : 0;    // interval of the merge kernel
    if (byte_tiles_path) {
        const RawLayout r = raw_layout(n_bytes, n_pieces, raw->n_seqs);
        const int64_t nt = byte_tiles(n_bytes);
        p.rec = (int2 *)ws_at(r.byte_rec);
        p.off_out = (int32_t *)ws_at(r.byte_off);
        p.off = p.off_out;
        p.tile_cnt = (int32_t *)ws_at(r.byte_cnt);
        p.out_offsets = nullptr;
        p.P = kWave;
        p.W = kWavesPerGroup;
        p.raw_auto_P = 0;
        if (plan) { plan->n_tiles = nt; plan->pieces_per_wave = kWave; plan->waves_per_tile = kWavesPerGroup; }
        run.run("merge_bytes_kernel", 1, merge_bytes_kernel, nt, kGroupThreads, p);
        if (ev) (void)hipEventRecord(ev[n_ev++], s);
        const int self_scan = nt <= kDeepSelfScanTiles;
        if (!self_scan) run.run("scan_tiles_kernel", 2, scan_tiles_kernel, (nt + kScanSpan - 1) / kScanSpan, kScanThreads, p, nt);
        if (ev) (void)hipEventRecord(ev[n_ev++], s);
        run.run("emit_bytes_kernel", 3, emit_bytes_kernel, nt, kGroupThreads, p, (int)nt, self_scan);
        if (ev) { (void)hipEventRecord(ev[n_ev++], s); (void)hipEventRecord(ev[n_ev++], s); }
    } else if (fused) {
        run.run("encode_kernel", 0, encode_kernel, n_tiles, kGroupThreads, p, (int)n_tiles);
        if (ev) { (void)hipEventRecord(ev[1], s); (void)hipEventRecord(ev[2], s); (void)hipEventRecord(ev[3], s); }
    } else {
        // Raw path: n_tiles only bounds the tile count.  A capped grid strides over the
        // tiles that exist (at least one workgroup, which also handles "no piece at all").
        const int64_t grid = raw ? std::min<int64_t>(std::max<int64_t>(n_tiles, 1), kRawMaxGrid) : n_tiles;
        if (raw) {
            // one tile per workgroup for as many tiles as are likely to exist (an eighth of
            // the capacity-sized bound, at least kRawMaxGrid), a strided kernel for the rest
            const int64_t direct = std::min<int64_t>(std::max<int64_t>(n_tiles, 1), std::max<int64_t>(kRawMaxGrid, n_tiles / 8));
            // (the long-piece workgroups need tiles of 256 pieces: only if the caller fixed that, and from
            // as many tiles on as on the other path, or when asked for)
            if (!raw_auto_P && p.P == kWave && o.long_groups >= 0 && (o.long_groups > 0 || direct >= kLongGroupsMinTiles)) {
                p.tiles_per_long_group = (int32_t)(o.long_groups > 0 ? o.long_groups : kTilesPerLongGroup);
                p.n_long_groups = (int32_t)((direct + p.tiles_per_long_group - 1) / p.tiles_per_long_group);
                p.long_sum = (int32_t *)ws_at(l.long_sum);
                run.run("merge_raw_groups_kernel", i0, merge_raw_groups_kernel, direct + p.n_long_groups, kGroupThreads, p);
            } else {
                run.run("merge_raw_kernel", i0, merge_raw_kernel, direct, kGroupThreads, p);
            }
            if (n_tiles > direct)
                run.run("merge_raw_rest_kernel", i0, merge_raw_rest_kernel, std::min<int64_t>(n_tiles - direct, kRawRestGrid),
                        kGroupThreads, p, (int)direct);
        } else if (o.dedup && grid > 0) {
            // the distinct pieces first, then their merges, then every piece takes its representative's record
            const DedupLayout d = dedup_layout(n_bytes, n_pieces);
            DedupParams dp = {};
            dp.bytes = bytes; dp.off = piece_offsets; dp.n_bytes = (int32_t)n_bytes; dp.n_pieces = (int32_t)n_pieces;
            dp.set = (int32_t *)ws_at(d.set);
            dp.set_mask = (uint32_t)(d.set_slots - 1);
            dp.rep = (int32_t *)ws_at(d.rep);
            dp.tile_reps = (int32_t *)ws_at(d.tile_reps);
            dp.piece_map = (int32_t *)ws_at(d.piece_map);
            dp.dense_of = (int32_t *)ws_at(d.dense_of);
            dp.n_reps = (int32_t *)ws_at(d.n_reps);
            dp.rec = p.rec;
            dp.rec_all = (int2 *)ws_at(d.rec_all);
            dp.tile_sum = p.tile_sum;
            dp.status = p.status;
            dp.call_id = p.call_id;
            run.run("dedup_scatter_kernel", i0, dedup_scatter_kernel, grid, kGroupThreads, dp);
            run.run("dedup_find_kernel", i0, dedup_find_kernel, grid, kGroupThreads, dp);
            run.run("dedup_compact_kernel", i0, dedup_compact_kernel, grid, kGroupThreads, dp, (int)grid);
            EncodeParams pm = p;
            pm.piece_map = dp.piece_map;
            pm.n_pieces_dev = dp.n_reps;
            pm.tile_sum = p.tile_base;      // the totals of the list's tiles are of no use (the scan kernel, if any, overwrites them)
            run.run("merge_mapped_kernel", i0, merge_mapped_kernel, grid, kGroupThreads, pm);
            run.run("dedup_count_kernel", i0 + 1, dedup_count_kernel, grid, kGroupThreads, dp);
            p.rec = dp.rec_all;
            p.rep_of = dp.rep;
        } else if (grid > 0 && p.W == 1 && !p.paper && n_pieces <= kWideMaxPieces && n_bytes > n_pieces * (int64_t)kGroupBoundMax) {
            run.run("merge_wide_kernel", i0, merge_wide_kernel, grid, kWideThreads, p);
        } else if (grid > 0) {
            // Word-sized pieces on average (a tile is 256 pieces): the rare longer ones go to workgroups
            // of their own at the head of the grid, one for every kTilesPerLongGroup tiles.
            if (p.P == kWave && p.W == kWavesPerGroup && !p.paper && o.long_groups >= 0 &&
                (o.long_groups > 0 || n_tiles >= kLongGroupsMinTiles)) {
                const int64_t wanted = o.long_groups > 0 ? o.long_groups : kTilesPerLongGroup;
                p.tiles_per_long_group = (int32_t)std::max<int64_t>(wanted, (n_tiles + kMaxLongGroups - 1) / kMaxLongGroups);
                p.n_long_groups = (int32_t)((n_tiles + p.tiles_per_long_group - 1) / p.tiles_per_long_group);
                p.long_sum = (int32_t *)ws_at(l.long_sum);
            }
            if (p.n_long_groups) run.run("merge_kernel", i0, merge_kernel, grid + p.n_long_groups, kGroupThreads, p);
            else run.run("merge_tiles_kernel", i0, merge_tiles_kernel, grid, kGroupThreads, p);
        }
        if (ev) (void)hipEventRecord(ev[n_ev++], s);
        const bool deep = !raw && !p.paper && n_tiles >= kDeepMinTiles;
        // (raw path: n_tiles bounds the tile count, and the emit kernel adds the totals up itself
        // up to kDeepSelfScanTiles tiles whichever way it walks them)
        const int self_scan = n_tiles > 0 && n_tiles <= (deep || raw ? kDeepSelfScanTiles : kSelfScanTiles);
        if (!self_scan && !(raw && n_tiles == 0))
            run.run("scan_tiles_kernel", i0 + 1, scan_tiles_kernel, std::max<int64_t>((n_tiles + kScanSpan - 1) / kScanSpan, 1),
                    kScanThreads, p, n_tiles);
        if (ev) (void)hipEventRecord(ev[n_ev++], s);
        // (raw path: n_tiles bounds the tile count)
        const bool seq_by_emit = raw && seq_offsets_by_emit(p.n_seqs, n_tiles);
        if (seq_by_emit) run.run("emit_raw_seq_kernel", i0 + 2, emit_raw_seq_kernel, grid, kGroupThreads, p);
        else if (raw) run.run("emit_raw_kernel", i0 + 2, emit_raw_kernel, grid, kGroupThreads, p);
        else if (deep)
            run.run("emit_deep_kernel", i0 + 2, emit_deep_kernel, (n_tiles + kEmitTiles - 1) / kEmitTiles, kGroupThreads, p,
                    (int)n_tiles, self_scan);
        else if (grid > 0) run.run("emit_kernel", i0 + 2, emit_kernel, grid, kGroupThreads, p, self_scan);
        if (ev) (void)hipEventRecord(ev[n_ev++], s);
        if (raw) {
            if (!seq_by_emit)
                run.run("seq_token_offsets_kernel", i0 + 3, seq_token_offsets_kernel,
                        (p.n_seqs + 1 + kGroupThreads - 1) / kGroupThreads, kGroupThreads, p);
            if (ev) (void)hipEventRecord(ev[n_ev++], s);
        }
    }
    return run.err == hipSuccess ? BPE_OK : hip_fail(run.err, "bpe_encode launch");
}

extern "C" int bpe_encode_plan(int64_t n_bytes, int64_t n_pieces, const bpe_encode_options *opts,
                               bpe_encode_plan_t *plan) {
    if (!plan) { set_error("plan is NULL"); return BPE_ERR_NULL; }
    return launch_encode(nullptr, nullptr, nullptr, n_bytes, n_pieces, nullptr, nullptr, nullptr, 0, opts, nullptr,
                         nullptr, nullptr, plan, true);
}

extern "C" int bpe_encode_raw_plan(int64_t n_bytes, int64_t max_pieces, int64_t n_seqs, int has_seq_offsets,
                                   int wants_piece_arrays, const bpe_encode_options *opts, bpe_encode_plan_t *plan) {
    if (!plan) { set_error("plan is NULL"); return BPE_ERR_NULL; }
    int32_t dummy = 0;
    const RawArgs raw = {has_seq_offsets ? &dummy : nullptr, has_seq_offsets ? n_seqs : 1, &dummy,
                         wants_piece_arrays ? &dummy : nullptr, nullptr, nullptr};
    return launch_encode(nullptr, nullptr, nullptr, n_bytes, max_pieces == 0 ? n_bytes : max_pieces, nullptr, nullptr,
                         nullptr, 0, opts, nullptr, nullptr, &raw, plan, true);
}

extern "C" int bpe_encode(const bpe_table *table, const uint8_t *bytes, const int32_t *piece_offsets,
                          int64_t n_bytes, int64_t n_pieces, int32_t *out_ids, int32_t *out_offsets,
                          void *workspace, int64_t workspace_bytes, const bpe_encode_options *opts,
                          void *stream) {
    return launch_encode(table, bytes, piece_offsets, n_bytes, n_pieces, out_ids, out_offsets, workspace,
                         workspace_bytes, opts, (hipStream_t)stream, nullptr);
}

// ---------------------------------------------------------------------------
// bpe_encode for callers that can neither allocate nor bring a workspace: the
// workspace is this array, which every GPU the library runs on holds (at its own
// address) until the process ends.  In host code the array's name is only a
// stand-in for the symbol; the device address comes from hipGetSymbolAddress, once
// per device, and is what the kernels get.  Nothing in it needs clearing between
// calls (every cross-call word carries the call id, as in a caller's workspace).
constexpr int64_t kStaticScratchBytes = 16ll << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static std::atomic<void *> g_scratch_ptr[kMaxDevices];

// The current device's copy of `scratch` (looked up on the first call on that device).
static int static_scratch(void **out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) { set_error("device index %d out of range", dev); return BPE_ERR_HIP; }
    void *ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) return hip_fail(e, "hipGetSymbolAddress(scratch)");
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);   // two threads find the same address
    }
    *out = ptr;
    return BPE_OK;
}

extern "C" int bpe_encode_static(const bpe_table *table, const uint8_t *bytes, const int32_t *piece_offsets,
                                 int64_t n_bytes, int64_t n_pieces, int32_t *out_ids, int32_t *out_offsets,
                                 const bpe_encode_options *opts, void *stream) {
    const int64_t need = bpe_workspace_bytes(n_bytes, n_pieces);
    if (need < 0) return (int)need;
    if (need > kStaticScratchBytes) {
        set_error("bpe_encode_static: %lld bytes in %lld pieces need %lld bytes of scratch, the built-in array holds %lld "
                  "(use bpe_encode with a workspace)", (long long)n_bytes, (long long)n_pieces, (long long)need,
                  (long long)kStaticScratchBytes);
        return BPE_ERR_SIZE;
    }
    void *ws = nullptr;
    const int rc = static_scratch(&ws);
    if (rc != BPE_OK) return rc;
    return launch_encode(table, bytes, piece_offsets, n_bytes, n_pieces, out_ids, out_offsets, ws, kStaticScratchBytes,
                         opts, (hipStream_t)stream, nullptr);
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

// The verdict that the first 8 status words of a workspace (host copy) spell.
static int verdict_of(const int32_t *st) {
    // No call has finished in this workspace (fresh or zero-filled memory, or a call whose launch
    // failed before its last kernel): nothing to report.
    if (st[kStatusCallCheck] != (st[kStatusCall] ^ kCallCheck)) return BPE_OK;
    const int32_t id = st[kStatusCall];
    if (st[kStatusWait] == id) { set_error("a wait between workgroups ran out (is the workspace shared by overlapping calls?)"); return BPE_ERR_HIP; }
    if (st[kStatusBadInput] == id) { set_error("piece_offsets or seq_offsets are out of range or decreasing, or a token id is not in the vocabulary"); return BPE_ERR_INPUT; }
    if (st[kStatusOverflow] == id) { set_error("more pieces than max_pieces, or more bytes than out_capacity"); return BPE_ERR_SIZE; }
    return BPE_OK;
}

extern "C" int bpe_status_from_words(const int32_t *status_words) {
    if (!status_words) { set_error("null pointer"); return BPE_ERR_NULL; }
    return verdict_of(status_words);
}

extern "C" int bpe_encode_status(void *workspace, void *stream) {
    if (!workspace) {              // the built-in scratch of bpe_encode_static on the current device
        const int rc = static_scratch(&workspace);
        if (rc != BPE_OK) return rc;
    }
    hipError_t e = hipStreamSynchronize((hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e, "hipStreamSynchronize");
    int32_t st[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    e = hipMemcpy(st, workspace, sizeof(st), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return hip_fail(e, "hipMemcpy(status)");
    const int verdict = verdict_of(st);
    if (verdict != BPE_OK) {
        // Reported once: a call that was recorded into a graph has the same call id at
        // every replay, and a later, clean replay must not inherit this verdict.
        const int32_t id = st[kStatusCall];
        const int32_t cleared[4] = {~id, ~id, id, ~id};
        e = hipMemcpy(workspace, cleared, sizeof(cleared), hipMemcpyHostToDevice);
        if (e != hipSuccess) return hip_fail(e, "hipMemcpy(status)");
    }
    return verdict;
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

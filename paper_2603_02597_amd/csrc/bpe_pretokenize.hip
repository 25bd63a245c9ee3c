// Pre-tokenization on the device: where pieces start.  The paper's pipeline has
// no such step (section 3.1 cuts the input into fixed-size chunks, which forbids
// merges across a cut); here a piece starts at byte 0, at the first byte of every
// sequence and at every space (0x20), and the merge loop never crosses a piece
// boundary.  This is a stream compaction: flag the start bytes, count them in
// order, write their indices densely.  One pass over the bytes, one kernel.
//
// A tile is ITER x 4 KiB of input for a workgroup of 4 wavefronts.  Wavefront w
// owns the contiguous ITER KiB number w of the tile and reads it 1 KiB at a time
// (one aligned 16-byte load per lane, so every load instruction is one contiguous
// 1 KiB).  Per 16-byte group a lane keeps a 16-bit mask of piece starts; ranks
// come from a wavefront scan per KiB, the wavefront totals, and the number of
// pieces before the tile, which tiles hand on by decoupled look-back.
#include "bpe_common.h"
#include "bpe_lookback.h"

namespace bpe {
// Tiles of the staged variants (large inputs) look back over 32 tiles per round
// instead of 256: the state words of other workgroups are uncached reads, and on
// deep grids their number, not the number of rounds, is what costs (1 GiB in 64 KiB
// tiles: 427 us with 256, 397 us with 64, 381 us with 32, 377 us with 16).
constexpr int kStagedWindow = 32;
}

namespace bpe {

struct PretokParams {
    const uint8_t *bytes;
    int32_t n_bytes;
    int32_t mis;                 // bytes & 15: positions are counted from the 16-byte boundary below `bytes`
    const int32_t *seq;          // [n_seqs + 1], or nullptr for one sequence
    int32_t n_seqs;
    int32_t *piece_offsets;      // [max_pieces + 1]
    int32_t max_pieces;
    int32_t *n_pieces;           // [1]
    int32_t *seq_first_piece;    // [n_seqs + 1] or nullptr
    unsigned long long *tile_state;
    int32_t *status;
    int32_t call_id;
    int32_t n_tiles;
};

// Bit j of the result is set if byte j of the 16-byte group is a space.
__device__ inline uint32_t space_mask(const uint4 &x) {
    uint32_t m = 0;
    const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const uint32_t y = w[d] ^ 0x20202020u;                       // a space byte becomes 0
        uint32_t t = (y & 0x7F7F7F7Fu) + 0x7F7F7F7Fu;                // bit 7 of a byte set iff its low 7 bits are not 0
        t = ~(t | y | 0x7F7F7F7Fu);                                  // 0x80 exactly in the bytes that are 0
        // bits 7, 15, 23, 31 -> bits 0..3
        const uint32_t nib = ((t >> 7) | (t >> 14) | (t >> 21) | (t >> 28)) & 0xFu;
        m |= nib << (4 * d);
    }
    return m;
}

template <int ITER, bool STAGED>
__global__ void __launch_bounds__(kGroupThreads) pretokenize_kernel(PretokParams p) {
    constexpr int kWaveBytes = ITER * 1024;
    constexpr int kTileBytes = kWavesPerGroup * kWaveBytes;
    __shared__ LookbackTmp lb;
    __shared__ int wave_total[kWavesPerGroup];
    // `extra` (sequence starts inside the tile, one bit per byte) is dead before
    // `pre` is written
    __shared__ union { uint32_t extra[kTileBytes / 32]; uint32_t pre[ITER][kGroupThreads]; } sq;   // pre: (pieces of the wavefront's share before the group) << 16 | mask
    __shared__ uint16_t stage[STAGED ? kWavesPerGroup : 1][STAGED ? 1024 : 1];   // starts of the KiB a wavefront is writing out, in order
    uint32_t (&extra)[kTileBytes / 32] = sq.extra;
    uint32_t (&pre)[ITER][kGroupThreads] = sq.pre;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const int tile = blockIdx.x;
    const bool last = tile == p.n_tiles - 1;
    // v = i + mis is the position of byte i counted from the aligned base
    const int64_t v_end = (int64_t)p.n_bytes + p.mis;
    const int64_t tile_v0 = (int64_t)tile * kTileBytes;
    const uint4 *src = (const uint4 *)(p.bytes - p.mis);
    if (tile == 0 && tid == 0) mark_call(p.status, p.call_id);

    // Loads run kDepth KiB ahead of the arithmetic.  A 16-byte group that holds at
    // least one byte of the input lies in the same page as that byte, so reading all
    // of it cannot fault.  In an interior tile every group lies inside the input.
    constexpr int kDepth = ITER < 4 ? ITER : ITER < 16 ? 4 : 8;
    const bool interior = tile_v0 >= 16 && tile_v0 + kTileBytes <= v_end;
    const int64_t lane_v0 = tile_v0 + (int64_t)wv * kWaveBytes + lane * 16;
    const uint4 *lane_src = src + (lane_v0 >> 4);
    auto load_group = [&](int it) {
        uint4 g = make_uint4(0, 0, 0, 0);
        if (interior || lane_v0 + it * 1024 < v_end) g = lane_src[it * 64];
        return g;
    };
    uint4 x[kDepth];
#pragma unroll
    for (int it = 0; it < kDepth; ++it) x[it] = load_group(it);

    // Sequence boundaries: every tile checks a strided share of them, and finds the
    // ones that fall into its own byte range.
    const int64_t lo_i = tile_v0 > p.mis ? tile_v0 - p.mis : 0;
    const int64_t hi_i = min(tile_v0 + kTileBytes - p.mis, (int64_t)p.n_bytes);
    int k0 = 0;
    bool any_seq = false;
    if (p.seq) {
        bool bad = false;
        for (int64_t k = (int64_t)tile * kGroupThreads + tid; k <= p.n_seqs; k += (int64_t)p.n_tiles * kGroupThreads) {
            const int sv = p.seq[k];
            bad |= sv < 0 || sv > p.n_bytes || (k == 0 && sv != 0) || (k == p.n_seqs && sv != p.n_bytes);
            if (k < p.n_seqs) bad |= p.seq[k + 1] < sv;
        }
        if (bad) __hip_atomic_store(&p.status[kStatusBadInput], p.call_id, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        int a = 0, b = p.n_seqs + 1;                 // first k with seq[k] >= lo_i
        while (a < b) {
            const int m = (a + b) >> 1;
            if (p.seq[m] < lo_i) a = m + 1; else b = m;
        }
        k0 = a;
        bool mine = false;
        if (k0 + tid <= p.n_seqs) {
            const int sv = p.seq[k0 + tid];
            mine = sv >= lo_i && (sv < hi_i || (last && sv == p.n_bytes));
        }
        any_seq = __syncthreads_or(mine);
        if (any_seq) {
            for (int i = tid; i < kTileBytes / 32; i += kGroupThreads) extra[i] = 0;
            __syncthreads();
            for (int64_t k = (int64_t)k0 + tid; k <= p.n_seqs; k += kGroupThreads) {
                const int sv = p.seq[k];
                if (sv < lo_i || sv >= hi_i) break;
                const int at = (int)(sv + p.mis - tile_v0);
                atomicOr(&extra[at >> 5], 1u << (at & 31));
            }
            __syncthreads();
        }
    }

    // Start masks and their ranks inside the wavefront's share.
    uint32_t packed[ITER];       // (starts of this wavefront before the group) << 16 | mask
    int wave_run = 0;
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
        const uint4 cur = x[it % kDepth];
        if (it + kDepth < ITER) x[it % kDepth] = load_group(it + kDepth);
        __builtin_amdgcn_sched_barrier(0);           // keep the loads kDepth ahead, not all at the top
        uint32_t m = space_mask(cur);
        if (any_seq) {
            const int at = wv * kWaveBytes + it * 1024 + lane * 16;
            m |= (extra[at >> 5] >> (at & 31)) & 0xFFFFu;
        }
        if (!interior) {
            // byte 0 starts a piece; bytes before the input or behind its end are none
            const int64_t v = lane_v0 + it * 1024;
            const int64_t first_valid = p.mis - v, end_valid = v_end - v;
            if (first_valid >= 0 && first_valid < 16) m |= 1u << first_valid;
            const uint32_t below_end = end_valid >= 16 ? 0xFFFFu : end_valid <= 0 ? 0u : (1u << end_valid) - 1u;
            const uint32_t from_first = first_valid <= 0 ? 0xFFFFu : first_valid >= 16 ? 0u : 0xFFFFu & ~((1u << first_valid) - 1u);
            m &= below_end & from_first;
        }
        const int c = __builtin_popcount(m);
        const int inc = wave_scan_inclusive(c);
        packed[it] = ((uint32_t)(wave_run + inc - c) << 16) | m;
        wave_run += __builtin_amdgcn_readlane(inc, kWave - 1);
    }
    if (lane == 0) wave_total[wv] = wave_run;
    __syncthreads();
    int wave_before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kWavesPerGroup; ++w) {
        if (w < wv) wave_before += wave_total[w];
        total += wave_total[w];
    }
    // the same value in every lane; telling the compiler keeps the output pointer of the tile scalar
    const int base = __builtin_amdgcn_readfirstlane(total_before_tile<1, (STAGED ? kStagedWindow : kGroupThreads)>(p.tile_state, p.status, p.call_id, p.status + kStatusEpochPretokenize, tile, p.n_tiles, total, lb));

    // The indices of the start bytes, densely, in order.  The tile's pieces are
    // addressed from its own first slot, so that a 32-bit offset is enough.
    const bool fits = (int64_t)base + total <= p.max_pieces;
    char *tile_out = (char *)(p.piece_offsets + base);
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
        uint32_t m = packed[it] & 0xFFFFu;
        const int in_tile = wave_before + (int)(packed[it] >> 16);
        if (any_seq) pre[it][tid] = packed[it];
        const int i0 = (int)(lane_v0 + it * 1024 - p.mis);
        if (fits && STAGED) {
            // Through LDS, so that the wavefront stores the starts of its KiB as one
            // contiguous run: scattered directly, one store instruction touches every
            // cache line of the run and each line is written five or six times.  That
            // pays once the input is large enough for bandwidth to matter; below, the
            // extra trip through LDS only adds latency.
            const int run0 = __builtin_amdgcn_readfirstlane((int)(packed[it] >> 16));    // lane 0: starts before this KiB
            const int run1 = it + 1 < ITER ? __builtin_amdgcn_readfirstlane((int)(packed[it + 1 < ITER ? it + 1 : it] >> 16))
                                           : wave_run;
            uint32_t at = (packed[it] >> 16) - (uint32_t)run0;
            const int b0 = lane * 16;
            while (m) {
                stage[wv][at++] = (uint16_t)(b0 + __builtin_ctz(m));
                m &= m - 1;
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
            __builtin_amdgcn_wave_barrier();
            const int kib_i0 = i0 - b0;              // input index of the KiB's first byte
            int32_t *run_out = (int32_t *)tile_out + wave_before + run0;
            for (int j = lane; j < run1 - run0; j += kWave) run_out[j] = kib_i0 + stage[wv][j];
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
            __builtin_amdgcn_wave_barrier();
        } else if (fits) {
            uint32_t at = (uint32_t)in_tile << 2;
            while (m) {
                *(int32_t *)(tile_out + at) = i0 + __builtin_ctz(m);
                m &= m - 1;
                at += 4;
            }
        } else {
            int r = base + in_tile;
            while (m) {
                if (r < p.max_pieces) p.piece_offsets[r] = i0 + __builtin_ctz(m);
                m &= m - 1;
                ++r;
            }
        }
    }
    const int n_all = base + total;
    if (last && tid == 0) {
        const int n = min(n_all, p.max_pieces);
        p.piece_offsets[n] = p.n_bytes;
        *p.n_pieces = n;
        if (n_all > p.max_pieces)
            __hip_atomic_store(&p.status[kStatusOverflow], p.call_id, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (!p.seq && p.seq_first_piece) { p.seq_first_piece[0] = 0; p.seq_first_piece[1] = n; }
    }

    // First piece of every sequence that begins in this tile = number of starts before it.
    if (any_seq && p.seq_first_piece) {
        __syncthreads();
        for (int64_t k = (int64_t)k0 + tid; k <= p.n_seqs; k += kGroupThreads) {
            const int sv = p.seq[k];
            if (sv < lo_i) break;
            int r;
            if (sv < hi_i) {
                const int at = (int)(sv + p.mis - tile_v0);
                const int w = at / kWaveBytes;
                const uint32_t word = pre[(at % kWaveBytes) >> 10][w * kWave + ((at & 1023) >> 4)];
                r = base + (int)(word >> 16) + __builtin_popcount(word & ((1u << (at & 15)) - 1u));
                for (int w2 = 0; w2 < w; ++w2) r += wave_total[w2];
            } else if (last && sv == p.n_bytes) {
                r = n_all;
            } else {
                break;
            }
            p.seq_first_piece[k] = min(r, p.max_pieces);
        }
    }
}

bool pretokenize_tile_ok(int k) { return k == 0 || k == 4 || k == 16 || k == 64 || k == 128 || k == -64 || k == -128; }

struct PretokLayout { int64_t status, tile_state, total; };

static int64_t pretok_tiles(int64_t n_bytes, int tile_bytes) {
    // + 15: the tiling starts up to 15 bytes below the first byte; never zero tiles
    const int64_t t = (n_bytes + 15 + tile_bytes - 1) / tile_bytes;
    return t > 0 ? t : 1;
}

static PretokLayout pretok_layout(int64_t n_bytes) {
    PretokLayout l;
    l.status = 0;
    l.tile_state = 256;
    l.total = 256 + ((8 * pretok_tiles(n_bytes, 4096) + 255) & ~255ll);
    return l;
}

int64_t pretokenize_state_bytes(int64_t n_bytes) { return pretok_layout(n_bytes).total - 256; }

// Enqueues the kernel.  All pointers are validated by the callers.
int launch_pretokenize(const uint8_t *bytes, int64_t n_bytes, const int32_t *seq_offsets, int64_t n_seqs,
                       int32_t *piece_offsets, int64_t max_pieces, int32_t *n_pieces, int32_t *seq_first_piece,
                       int32_t *status, unsigned long long *tile_state, int32_t call_id, int tile_kib,
                       hipStream_t s, int64_t *grid_out, bool dry) {
    const int mis = n_bytes > 0 ? (int)((uintptr_t)bytes & 15) : 0;   // nothing is loaded from an empty input
    const int64_t v_end = n_bytes + mis;
    if (tile_kib == 0) {
        // Small tiles while they fit one look-back window or two (the chip has 256
        // compute units); the hand-over between windows costs 1-2 us and every tile
        // polls 256 state words of other tiles, so large inputs take large tiles.
        // From tens of MiB on, bandwidth matters and the stores go through LDS.
        tile_kib = v_end <= (2ll << 20) ? 4 : v_end <= (8ll << 20) ? 16 : v_end <= (32ll << 20) ? 64 : -64;
    }
    PretokParams p = {};
    p.bytes = bytes;
    p.n_bytes = (int32_t)n_bytes;
    p.mis = mis;
    p.seq = seq_offsets;
    p.n_seqs = seq_offsets ? (int32_t)n_seqs : 1;
    p.piece_offsets = piece_offsets;
    p.max_pieces = (int32_t)max_pieces;
    p.n_pieces = n_pieces;
    p.seq_first_piece = seq_first_piece;
    p.tile_state = tile_state;
    p.status = status;
    p.call_id = call_id;
    const int64_t tile_bytes = (int64_t)(tile_kib < 0 ? -tile_kib : tile_kib) * 1024;
    int64_t n_tiles = (v_end + tile_bytes - 1) / tile_bytes;
    if (n_tiles < 1) n_tiles = 1;
    p.n_tiles = (int32_t)n_tiles;
    if (grid_out) *grid_out = n_tiles;
    if (dry) {
        if (pretokenize_tile_ok(tile_kib) && tile_kib != 0) return BPE_OK;
        set_error("pretokenize tile size must be 0, 4, 16, 64, 128, -64 or -128 KiB");
        return BPE_ERR_OPTION;
    }
    const dim3 grid((unsigned)n_tiles), block(kGroupThreads);
    switch (tile_kib) {
    case 4:    hipLaunchKernelGGL((pretokenize_kernel<1, false>), grid, block, 0, s, p); break;
    case 16:   hipLaunchKernelGGL((pretokenize_kernel<4, false>), grid, block, 0, s, p); break;
    case 64:   hipLaunchKernelGGL((pretokenize_kernel<16, false>), grid, block, 0, s, p); break;
    case 128:  hipLaunchKernelGGL((pretokenize_kernel<32, false>), grid, block, 0, s, p); break;
    case -64:  hipLaunchKernelGGL((pretokenize_kernel<16, true>), grid, block, 0, s, p); break;
    case -128: hipLaunchKernelGGL((pretokenize_kernel<32, true>), grid, block, 0, s, p); break;
    default: set_error("pretokenize tile size must be 0, 4, 16, 64, 128, -64 or -128 KiB"); return BPE_ERR_OPTION;
    }
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? BPE_OK : hip_fail(e, "bpe_pretokenize launch");
}

}  // namespace bpe

using namespace bpe;

extern "C" int64_t bpe_pretokenize_workspace_bytes(int64_t n_bytes) {
    if (n_bytes < 0 || n_bytes >= 0x7FFFFFFFll) {
        set_error("n_bytes out of range (%lld)", (long long)n_bytes);
        return BPE_ERR_SIZE;
    }
    return pretok_layout(n_bytes).total;
}

extern "C" int bpe_pretokenize(const uint8_t *bytes, int64_t n_bytes, const int32_t *seq_offsets, int64_t n_seqs,
                               int32_t *piece_offsets, int64_t max_pieces, int32_t *n_pieces,
                               int32_t *seq_first_piece, void *workspace, int64_t workspace_bytes,
                               const bpe_encode_options *opts, void *stream) {
    if ((!bytes && n_bytes > 0) || !piece_offsets || !n_pieces) { set_error("null pointer"); return BPE_ERR_NULL; }
    if (n_bytes < 0 || n_bytes >= 0x7FFFFFFFll || n_seqs < 0 || n_seqs >= 0x7FFFFFFFll || max_pieces < 0 ||
        max_pieces >= 0x7FFFFFFFll) {
        set_error("sizes out of range (n_bytes %lld, n_seqs %lld, max_pieces %lld)", (long long)n_bytes,
                  (long long)n_seqs, (long long)max_pieces);
        return BPE_ERR_SIZE;
    }
    const int64_t need = bpe_pretokenize_workspace_bytes(n_bytes);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < need) {
        set_error("workspace missing, misaligned or too small (need %lld bytes)", (long long)need);
        return BPE_ERR_WORKSPACE;
    }
    const int tile_kib = opts ? opts->pretokenize_tile_kib : 0;
    if (!pretokenize_tile_ok(tile_kib)) {
        set_error("pretokenize_tile_kib must be 0, 4, 16, 64, 128, -64 or -128");
        return BPE_ERR_OPTION;
    }
    const PretokLayout l = pretok_layout(n_bytes);
    char *ws = (char *)workspace;
    return launch_pretokenize(bytes, n_bytes, seq_offsets, n_seqs, piece_offsets, max_pieces,
                              n_pieces, seq_first_piece, (int32_t *)(ws + l.status),
                              (unsigned long long *)(ws + l.tile_state), next_call_id(), tile_kib,
                              (hipStream_t)stream);
}

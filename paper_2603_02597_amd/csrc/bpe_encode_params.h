// Parameter block and lane helpers shared by the merge paths (device code).
#pragma once
#include "bpe_common.h"

namespace bpe {

struct EncodeParams {
    TableView table;
    const uint8_t *bytes;
    const int32_t *off;
    int32_t n_bytes;
    int32_t n_pieces;    // with n_pieces_dev: the capacity of the piece arrays
    const int32_t *n_pieces_dev;   // raw path: the piece count is only known on the device (else nullptr)
    const int32_t *piece_map;      // de-duplication: the pieces to merge, [*n_pieces_dev] indices into off (else nullptr)
    const int32_t *rep_of;         // de-duplication: [n_pieces] the piece whose tokens piece q shares (else nullptr)
    const int32_t *seq_off;        // raw path without a pre-tokenizer launch: [n_seqs + 1] the caller's sequence offsets (or nullptr)
    int32_t *tile_cnt;             // ... [byte tiles] pieces that start in a tile
    int32_t *off_out;              // ... [byte tiles x kByteTileStride] first byte of every piece (`off` points to the same array)
    const int32_t *seq_first_piece;   // raw path: [n_seqs + 1] first piece of every sequence
    int32_t *seq_token_offsets;       // raw path: [n_seqs + 1] first token of every sequence
    int32_t n_seqs;
    int32_t P;           // pieces per wavefront (<= 64)
    int32_t W;           // wavefronts of a workgroup that own pieces: 4, or 1 (with P = 1: one piece per workgroup)
    int32_t raw_auto_P;  // raw path: the kernels choose P themselves once the piece count is known
    int32_t tiny_max;    // longest piece the lane-per-piece path takes (<= 16)
    int32_t col_max;     // longest piece the lane-per-piece path with 64-entry columns takes (<= 64)
    int32_t wave_max;    // longest piece the lane-per-symbol path takes (<= 64)
    int32_t wave_lds_max;  // longest piece one wavefront takes through its LDS region (<= kWaveLdsMax)
    int32_t lds_max;     // longest piece the workgroup path keeps in LDS
    int32_t level;       // selection level 1, 2 or 3
    int32_t runs_by_best_rank;   // at level 3: pieces that are mostly runs of one byte take the level-2 passes
    int32_t paper;       // 0, or the paper's kernel to run instead: 1 = section 3.4, 2 = section 3.5 (one piece per tile)
    int2 *rec;           // [n_pieces] {tokens of the piece, its first token or -1 if that is in scratch too}
    int32_t *tile_sum;   // [n_tiles]
    int32_t *long_sum;   // [n_tiles] tokens of a tile's pieces that the long-piece workgroups merged (nullptr: there are none)
    int32_t n_long_groups;    // merge_kernel: the first so many workgroups take the pieces beyond tiny_max ...
    int32_t tiles_per_long_group;   // ... of so many consecutive tiles each; the others take one tile's short pieces
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

// The smallest v of the 64 lanes, to every lane, with data-parallel primitives: prefix
// minima by shifts of 1, 2, 4, 8 inside each row of 16 lanes, lane 15 of rows 0 and 2
// into rows 1 and 3, lane 31 into rows 2 and 3; lane 63 then holds the minimum.  (Six
// cross-lane reads through the LDS crossbar take about 0.12 us longer.)
__device__ inline uint32_t wave_min_u32(uint32_t v) {
    v = min(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x111, 0xF, 0xF, false));   // row_shr:1
    v = min(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x112, 0xF, 0xF, false));   // row_shr:2
    v = min(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x114, 0xF, 0xF, false));   // row_shr:4
    v = min(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x118, 0xF, 0xF, false));   // row_shr:8
    v = min(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x142, 0xA, 0xF, false));   // row_bcast:15
    v = min(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x143, 0xC, 0xF, false));   // row_bcast:31
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

// Inclusive prefix maximum over the 64 lanes, the same way.
__device__ inline int wave_scan_max_inclusive(int v) {
    v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x111, 0xF, 0xF, false));   // row_shr:1
    v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x112, 0xF, 0xF, false));   // row_shr:2
    v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x114, 0xF, 0xF, false));   // row_shr:4
    v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x118, 0xF, 0xF, false));   // row_shr:8
    v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x142, 0xA, 0xF, false));   // row_bcast:15
    v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x143, 0xC, 0xF, false));   // row_bcast:31
    return v;
}

// v of the lane below (lane 0 gets `first`) / of the lane above (lane 63 gets `last`).
__device__ inline int wave_from_lane_below(int v, int first) {
    return __builtin_amdgcn_update_dpp(first, v, 0x138, 0xF, 0xF, false);    // wave_shr:1
}
__device__ inline int wave_from_lane_above(int v, int last) {
    return __builtin_amdgcn_update_dpp(last, v, 0x130, 0xF, 0xF, false);     // wave_shl:1
}

}  // namespace bpe

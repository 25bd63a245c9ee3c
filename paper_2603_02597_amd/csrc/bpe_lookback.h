// Ordered hand-over of running totals between the workgroups of one launch
// (decoupled look-back): tile t publishes its own total, adds up the totals of
// the tiles before it until it meets one that already published its prefix, and
// publishes its own prefix.  Used by the single-kernel encode path (tokens
// before a tile) and by the pre-tokenizer (pieces before a tile).
//
// Every cross-workgroup word carries a tag derived from the call id and from a
// launch counter that lives next to the state array (the epoch), so the state
// array needs no clearing between calls, and a call that was recorded into a
// graph, whose call id is the same at every replay, does not mistake the words
// of the previous replay for its own.  The epoch is advanced by the launch
// itself: by the last tile, once its look-back is complete.  By then every other
// tile has published its total, and a tile derives the tag it publishes from the
// epoch it read, so every tile of the launch has read the old value.
//
// A tile only ever waits for tiles with a lower index.  Workgroups are handed to
// each XCD in increasing index order, so the lowest unfinished tile is always
// resident and waits for nobody: the waits cannot form a cycle.  Every wait is
// also bounded (kWaitTicks of the 100 MHz wall clock, about two seconds: far
// longer than any tile of a sane call takes, short enough for a test to sit
// through); running out reports BPE_ERR_HIP through the status words instead of
// hanging, and once one wait has run out nobody waits any longer.  (A shared ticket counter would make the
// order explicit, but device-wide atomics on one address complete at about one
// per 2 us here, which serialises the tiles.)
#ifndef BPE_LOOKBACK_H
#define BPE_LOOKBACK_H

#include "bpe_common.h"

namespace bpe {

constexpr uint32_t kFlagAggregate = 1, kFlagPrefix = 2;
constexpr unsigned long long kWaitTicks = 200000000ull;

// Status block at the start of a workspace (int32 words).  A word counts only
// if it equals the call id in kStatusCall.
constexpr int kStatusBadInput = 0;   // offsets out of range or decreasing
constexpr int kStatusOverflow = 1;   // more pieces than the caller's capacity
constexpr int kStatusCall = 2;       // call id of the call that ran last
constexpr int kStatusWait = 3;       // a wait between workgroups ran out
constexpr int kStatusEpochEncode = 4;       // launch counters of the three kernels that hand totals on
constexpr int kStatusEpochPretokenize = 5;
constexpr int kStatusEpochDecode = 6;
constexpr int kStatusLongPieces = 9;  // call id if the merge kernel's long-piece workgroups merged anything
constexpr int kStatusCallCheck = 7;  // call id ^ kCallCheck, written with kStatusCall: a workspace that no call has
                                     // finished in (fresh, zero-filled, or holding an older program's data) fails it
constexpr int32_t kCallCheck = 0x5AC3A53C;

// By one thread of the launch that ends a call: the call the other status words refer to.
__device__ inline void mark_call(int32_t *status, int32_t call_id) {
    status[kStatusCall] = call_id;
    status[kStatusCallCheck] = call_id ^ kCallCheck;
}

__device__ inline unsigned long long state_word(uint32_t tag, uint32_t flag, uint32_t value) {
    return ((unsigned long long)((tag << 2) | flag) << 32) | value;
}

// Inclusive prefix sum over the 64 lanes of a wavefront with data-parallel
// primitives: shifts by 1, 2, 4, 8 inside each row of 16 lanes (a lane without a
// source adds 0), then lane 15 of row 0 and 2 into rows 1 and 3, then lane 31
// into rows 2 and 3.
__device__ inline int wave_scan_inclusive(int v) {
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xF, 0xF, false);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xF, 0xF, false);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xF, 0xF, false);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xF, 0xF, false);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xA, 0xF, false);   // row_bcast:15 into rows 1, 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xC, 0xF, false);   // row_bcast:31 into rows 2, 3
    return v;
}

constexpr int kLookbackMaxWaves = 16;
struct LookbackTmp {
    int first_w[kLookbackMaxWaves];
    int sum_w[kLookbackMaxWaves];
};

// Sum of the totals of all tiles before `tile` of `n_tiles`; also publishes this
// tile's total and prefix in state[tile].  `epoch` is the launch counter of this
// kernel in the status block.  All 64 * WAVES threads of the workgroup must call
// it; the first WINDOW of them look at other tiles.  A round looks
// at kGroupThreads * LOOK tiles, LOOK per thread with their loads in flight
// together: a state word of another workgroup takes 1-2 us to arrive, so deep
// grids (where the nearest published prefix is a thousand tiles back) want few,
// wide rounds.
template <int LOOK = 1, int WINDOW = kGroupThreads, int WAVES = kWavesPerGroup>
__device__ inline int total_before_tile(unsigned long long *state, int32_t *status, int32_t call_id, int32_t *epoch,
                                        int tile, int n_tiles, int total, LookbackTmp &lb) {
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const uint32_t launch = (uint32_t)__builtin_amdgcn_readfirstlane(*epoch);
    uint32_t tag = ((uint32_t)call_id + launch) & 0x3FFFFFFFu;
    if (tag == 0) tag = 1;
    if (tid == 0)
        __hip_atomic_store(&state[tile], state_word(tag, tile == 0 ? kFlagPrefix : kFlagAggregate, (uint32_t)total),
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // the word is the whole message: no release needed
    if (tile == 0) {
        if (n_tiles == 1 && tid == 0) *epoch = (int32_t)(launch + 1);
        return 0;
    }
    int running = 0;
    for (int hi = tile;; hi -= WINDOW * LOOK) {            // this round looks at tiles [hi - WINDOW * LOOK, hi)
        // thread t owns tiles hi - 1 - (t * LOOK + l), l = 0 .. LOOK - 1: nearest first
        unsigned long long w[LOOK];
#pragma unroll
        for (int l = 0; l < LOOK; ++l) {
            const int j = hi - 1 - (tid * LOOK + l);
            w[l] = tid >= WINDOW ? state_word(tag, 0, 0)              // threads beyond the window look at nothing
                 : j >= 0 ? __hip_atomic_load(&state[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                          : state_word(tag, kFlagPrefix, 0);          // before tile 0: an empty prefix
        }
        int mine = 0;              // totals of my tiles up to and including my nearest prefix
        bool have_prefix = false;
#pragma unroll
        for (int l = 0; l < LOOK; ++l) {
            const int j = hi - 1 - (tid * LOOK + l);
            if ((uint32_t)(w[l] >> 34) != tag) {
                const unsigned long long t_start = wall_clock64();
                int polls = 0;
                for (;;) {
                    __builtin_amdgcn_s_sleep(2);
                    w[l] = __hip_atomic_load(&state[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if ((uint32_t)(w[l] >> 34) == tag) break;
                    if ((++polls & 255) == 0 &&
                        (wall_clock64() - t_start > kWaitTicks ||
                         __hip_atomic_load(&status[kStatusWait], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == call_id))
                        break;
                }
            }
            uint32_t flag = 0, value = 0;
            if ((uint32_t)(w[l] >> 34) == tag) {
                flag = (uint32_t)(w[l] >> 32) & 3u;
                value = (uint32_t)w[l];
            } else {
                // gave up waiting: reported as BPE_ERR_HIP
                __hip_atomic_store(&status[kStatusWait], call_id, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            if (!have_prefix) mine += (int)value;
            have_prefix |= flag == kFlagPrefix;
        }
        // nearest tile with a published prefix = smallest thread index that has one
        const uint64_t pm = __ballot(have_prefix);
        if (lane == 0) lb.first_w[wv] = pm ? wv * kWave + (int)__builtin_ctzll(pm) : 0x7FFFFFFF;
        __syncthreads();
        int first = 0x7FFFFFFF;
        for (int w4 = 0; w4 < WAVES; ++w4) first = min(first, lb.first_w[w4]);
        int part = tid <= first ? mine : 0;
        part = __builtin_amdgcn_readlane(wave_scan_inclusive(part), kWave - 1);
        if (lane == 0) lb.sum_w[wv] = part;
        __syncthreads();
        for (int w4 = 0; w4 < WAVES; ++w4) running += lb.sum_w[w4];
        if (first != 0x7FFFFFFF) break;
    }
    if (tid == 0) {
        __hip_atomic_store(&state[tile], state_word(tag, kFlagPrefix, (uint32_t)(running + total)),
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (tile == n_tiles - 1) *epoch = (int32_t)(launch + 1);
    }
    return running;
}

// Scrambled counter: marks the status and tile-state words of one call.  An
// uninitialised workspace holds whatever lived there before, typically small
// integers; the low 30 bits (the tile-state tag) are never zero.
int32_t next_call_id();

}  // namespace bpe
#endif

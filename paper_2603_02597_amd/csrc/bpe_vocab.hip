// Vocabulary side of the tokenizer: what every token id stands for.  The paper
// takes GPT-2's vocabulary as given (section 3.2) and decodes on the host; here
// the byte expansion of every id is derived from the merge rules themselves
// (a merged id expands to the expansions of its two parts, section 3.3), kept on
// the device, and used to turn ids back into bytes (bpe_decode).  An optional
// renumbering (internal id <-> output id) lets a caller who has a real
// vocabulary file emit and accept that file's ids (bpe_map_ids).
//
// Decoding is an expansion: length of every token, running sum, copy.  One pass,
// one kernel: tiles of 1024 tokens, the bytes before a tile by decoupled
// look-back, the tile's bytes assembled in LDS and stored as aligned words.
#include <algorithm>
#include <cstring>
#include <new>

#include "bpe_common.h"
#include "bpe_lookback.h"

struct bpe_vocab {
    bpe_vocab_info_t info;
    void *device_mem;      // one allocation: tok | out_of | int_of | pool
    const uint2 *tok;      // [n_ids] {offset of the expansion in the pool, its length; 0 = id not in use}
    const int32_t *out_of, *int_of;
    const uint8_t *pool;
    int32_t n_out;
    int device;
};

namespace bpe {

constexpr int kTokPerThread = 4;
constexpr int kTileTokens = kGroupThreads * kTokPerThread;
constexpr int kStageBytes = 16384;            // a tile whose bytes fit is assembled in LDS
constexpr int64_t kMaxTokenBytes = 1 << 20;   // longest expansion a vocabulary may hold
constexpr int64_t kMaxPoolBytes = 1ll << 30;

struct DecodeParams {
    const uint2 *tok;               // [n_ids] {offset in the pool (a multiple of 4), length (0 = id not in use)}
    const int32_t *int_of;          // output id -> internal id, or nullptr: ids are internal ids
    const uint8_t *pool;
    int32_t n_ids, n_out;
    const int32_t *ids;
    int32_t n_tokens;
    const int32_t *n_tokens_dev;    // or nullptr
    uint8_t *out;
    int32_t out_capacity;
    int32_t *token_byte_offsets;    // [n_tokens + 1] or nullptr
    int32_t *n_bytes;               // [1] or nullptr
    unsigned long long *tile_state;
    int32_t *status;
    int32_t call_id;
};

__device__ inline int token_count(const DecodeParams &p) {
    return p.n_tokens_dev ? min(max(__builtin_amdgcn_readfirstlane(*p.n_tokens_dev), 0), p.n_tokens) : p.n_tokens;
}

// A tile is ROUNDS x 1024 tokens: thread t owns tokens r * 1024 + 4 t .. + 3 of the
// tile for r = 0 .. ROUNDS - 1.  The bytes before the tile are found once per tile
// (every tile polls the state words of 256 others, so deep grids want few, large
// tiles); the bytes go out round by round through the same 16 KiB of LDS.
template <int ROUNDS, int WINDOW>
__global__ void __launch_bounds__(kGroupThreads) decode_kernel(DecodeParams p) {
    constexpr int kTile = ROUNDS * kTileTokens;
    __shared__ LookbackTmp lb;
    __shared__ int wave_total[ROUNDS][kWavesPerGroup];
    __shared__ uint32_t stage[kStageBytes / 4 + 2];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const int tile = blockIdx.x;
    const int n = token_count(p);
    const int n_tiles = max((n + kTile - 1) / kTile, 1);
    if (tile >= n_tiles) return;               // the grid was sized for the host's upper bound
    if (tile == 0 && tid == 0) mark_call(p.status, p.call_id);

    uint32_t len[ROUNDS][kTokPerThread], off[ROUNDS][kTokPerThread];
    int ex[ROUNDS];                            // bytes of the round before this thread's tokens
    bool bad = false;
#pragma unroll
    for (int r = 0; r < ROUNDS; ++r) {
        const int t0 = tile * kTile + r * kTileTokens + tid * kTokPerThread;
        int mine = 0;
#pragma unroll
        for (int j = 0; j < kTokPerThread; ++j) {
            len[r][j] = 0;
            off[r][j] = 0;
            if (t0 + j < n) {
                int id = p.ids[t0 + j];
                if (p.int_of) id = id >= 0 && id < p.n_out ? p.int_of[id] : -1;
                if (id >= 0 && id < p.n_ids) { const uint2 t = p.tok[id]; off[r][j] = t.x; len[r][j] = t.y; }
                bad |= len[r][j] == 0;         // no token is empty: the id is not in the vocabulary
            }
            mine += (int)len[r][j];
        }
        const int inc = wave_scan_inclusive(mine);
        if (lane == kWave - 1) wave_total[r][wv] = inc;
        ex[r] = inc - mine;
    }
    if (__ballot(bad) && lane == 0)
        __hip_atomic_store(&p.status[kStatusBadInput], p.call_id, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    int round_total[ROUNDS], total = 0;
#pragma unroll
    for (int r = 0; r < ROUNDS; ++r) {
        round_total[r] = 0;
#pragma unroll
        for (int w = 0; w < kWavesPerGroup; ++w) {
            if (w < wv) ex[r] += wave_total[r][w];
            round_total[r] += wave_total[r][w];
        }
        total += round_total[r];
    }
    // token lengths are at most 2^20 and a tile has at most 2^13 tokens: a tile total
    // cannot wrap, and the running total is compared against the capacity in 64 bits
    const uint32_t base = (uint32_t)__builtin_amdgcn_readfirstlane(
        total_before_tile<1, WINDOW>(p.tile_state, p.status, p.call_id, p.status + kStatusEpochDecode, tile, n_tiles,
                                     total, lb));
    const int64_t end = (int64_t)base + (uint32_t)total;
    if ((base > (uint32_t)p.out_capacity || end > p.out_capacity) && tid == 0)
        __hip_atomic_store(&p.status[kStatusOverflow], p.call_id, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (tile == n_tiles - 1 && tid == 0) {
        if (p.token_byte_offsets) p.token_byte_offsets[n] = (int)end;
        if (p.n_bytes) *p.n_bytes = (int)min(end, (int64_t)p.out_capacity);
    }

    const uint32_t *pool_w = (const uint32_t *)p.pool;       // every expansion starts at a multiple of 4
    int64_t round_base = base;
#pragma unroll
    for (int r = 0; r < ROUNDS; ++r) {
        const int t0 = tile * kTile + r * kTileTokens + tid * kTokPerThread;
        const int rt = __builtin_amdgcn_readfirstlane(round_total[r]);
        if (p.token_byte_offsets) {
            int at = (int)round_base + ex[r];
#pragma unroll
            for (int j = 0; j < kTokPerThread; ++j) {
                if (t0 + j < n) p.token_byte_offsets[t0 + j] = at;
                at += (int)len[r][j];
            }
        }
        if (round_base + rt <= p.out_capacity && rt <= kStageBytes) {
            // Assemble in LDS at the same offset from a 4-byte boundary as in the output,
            // then store whole aligned words (the first and last one byte by byte).
            uint8_t *dst = p.out + round_base;
            const int m = (int)((uintptr_t)dst & 3);
            uint8_t *sb = (uint8_t *)stage;
            int at = m + ex[r];
#pragma unroll
            for (int j = 0; j < kTokPerThread; ++j) {
                // whole words first (the compiler picks the widest LDS store the target
                // allows at an unaligned address), then the last one to three bytes
                const uint32_t l = len[r][j], o = off[r][j], full = l & ~3u;
                for (uint32_t k = 0; k < full; k += 4) {
                    const uint32_t w = pool_w[(o + k) >> 2];
                    __builtin_memcpy(sb + at + k, &w, 4);
                }
                if (l & 3u) {
                    const uint32_t w = pool_w[(o + full) >> 2];
                    for (uint32_t q = 0; q < (l & 3u); ++q) sb[at + full + q] = (uint8_t)(w >> (8 * q));
                }
                at += (int)l;
            }
            __syncthreads();
            const int n_words = (m + rt + 3) >> 2;
            uint32_t *dst_w = (uint32_t *)(dst - m);
            for (int d = tid; d < n_words; d += kGroupThreads) {
                const uint32_t w = stage[d];
                const int lo = d == 0 ? m : 0, hi = min(4, m + rt - 4 * d);
                if (lo == 0 && hi == 4) {
                    dst_w[d] = w;
                } else {
                    for (int q = lo; q < hi; ++q) ((uint8_t *)(dst_w + d))[q] = (uint8_t)(w >> (8 * q));
                }
            }
            if (r + 1 < ROUNDS) __syncthreads();             // the next round reuses the stage
        } else {
            // Long tokens (or an output that is too small): bytes straight to the output,
            // a wavefront sharing every token of more than 64 bytes.
            int64_t at = round_base + ex[r];
#pragma unroll
            for (int j = 0; j < kTokPerThread; ++j) {
                const uint32_t l = len[r][j], o = off[r][j];
                const bool is_long = l > 64;
                if (!is_long) {
                    for (uint32_t k = 0; k < l; ++k)
                        if (at + k < p.out_capacity) p.out[at + k] = p.pool[o + k];
                }
                for (uint64_t lm = __ballot(is_long); lm;) {
                    const int src_lane = __builtin_ctzll(lm);
                    lm &= lm - 1;
                    const uint32_t so = (uint32_t)__builtin_amdgcn_readlane((int)o, src_lane);
                    const uint32_t sl = (uint32_t)__builtin_amdgcn_readlane((int)l, src_lane);
                    const int64_t a = ((int64_t)(uint32_t)__builtin_amdgcn_readlane((int)(at >> 32), src_lane) << 32) |
                                      (uint32_t)__builtin_amdgcn_readlane((int)at, src_lane);
                    for (uint32_t k = lane; k < sl; k += kWave)
                        if (a + k < p.out_capacity) p.out[a + k] = p.pool[so + k];
                }
                at += l;
            }
        }
        round_base += rt;
    }
}

struct MapParams {
    const int32_t *table;   // out_of or int_of
    int32_t n_table;
    const int32_t *in;
    int32_t *out;
    int64_t n;
    const int32_t *n_dev;
};

__global__ void __launch_bounds__(kGroupThreads) map_ids_kernel(MapParams p) {
    int64_t n = p.n;
    if (p.n_dev) n = min<int64_t>(max(*p.n_dev, 0), n);
    const int64_t i = (int64_t)blockIdx.x * kGroupThreads + threadIdx.x;
    if (i >= n) return;
    const int id = p.in[i];
    p.out[i] = id >= 0 && id < p.n_table ? p.table[id] : -1;
}

static int64_t align256v(int64_t v) { return (v + 255) & ~255ll; }

}  // namespace bpe

using namespace bpe;

extern "C" int bpe_vocab_build(const int32_t *merges, const int32_t *ranks, const int32_t *merged_ids, int64_t n,
                               const int32_t *output_ids, int64_t n_output_ids, bpe_vocab **out_vocab) {
    if (!out_vocab) { set_error("out_vocab is NULL"); return BPE_ERR_NULL; }
    *out_vocab = nullptr;
    RuleOrder ro;
    int rc = order_rules(merges, ranks, merged_ids, n, ro);
    if (rc != BPE_OK) return rc;
    const int64_t n_ids = ro.max_id + 1;
    if (output_ids && n_output_ids != n_ids) {
        set_error("output_ids must have one entry per id up to the largest (%lld), got %lld", (long long)n_ids,
                  (long long)n_output_ids);
        return BPE_ERR_SIZE;
    }
    // expansions in rank order: both parts of a rule are bytes or made by earlier rules
    std::vector<uint32_t> tok_off((size_t)n_ids, 0), tok_len((size_t)n_ids, 0);
    std::vector<uint8_t> pool((size_t)256 * 4, 0);
    for (int b = 0; b < 256; ++b) { tok_off[b] = 4 * b; tok_len[b] = 1; pool[4 * b] = (uint8_t)b; }
    int64_t longest = 1;
    for (int64_t k = 0; k < n; ++k) {
        const int64_t i = ro.by_rank[k].second;
        const int64_t a = merges[2 * i], b = merges[2 * i + 1], m = ro.merged_row[i];
        const int64_t len = (int64_t)tok_len[a] + tok_len[b];
        if (len > kMaxTokenBytes || (int64_t)pool.size() + len + 4 > kMaxPoolBytes) {
            set_error("the expansions of this table are too long to keep (token of %lld bytes, pool of %lld)",
                      (long long)len, (long long)pool.size());
            return BPE_ERR_SIZE;
        }
        const size_t at = pool.size();
        pool.resize(at + (size_t)((len + 3) & ~3ll), 0);
        memcpy(pool.data() + at, pool.data() + tok_off[a], tok_len[a]);
        memcpy(pool.data() + at + tok_len[a], pool.data() + tok_off[b], tok_len[b]);
        tok_off[m] = (uint32_t)at;
        tok_len[m] = (uint32_t)len;
        longest = std::max(longest, len);
    }
    // renumbering: unique output ids in [0, 2^24) for the ids in use
    std::vector<int32_t> out_of, int_of;
    if (output_ids) {
        int64_t max_out = -1;
        for (int64_t id = 0; id < n_ids; ++id) {
            if (tok_len[id] == 0) continue;
            const int64_t o = output_ids[id];
            if (o < 0 || o >= (1ll << kIdBits)) { set_error("output id %lld of id %lld is outside [0, 2^24)", (long long)o, (long long)id); return BPE_ERR_ID_RANGE; }
            max_out = std::max(max_out, o);
        }
        out_of.assign((size_t)n_ids, -1);
        int_of.assign((size_t)(max_out + 1), -1);
        for (int64_t id = 0; id < n_ids; ++id) {
            if (tok_len[id] == 0) continue;
            const int32_t o = output_ids[id];
            if (int_of[o] != -1) { set_error("output id %d is given to ids %d and %lld", o, int_of[o], (long long)id); return BPE_ERR_DUP_MERGED; }
            int_of[o] = (int32_t)id;
            out_of[id] = o;
        }
    }
    std::vector<uint32_t> tok((size_t)(2 * n_ids));
    for (int64_t id = 0; id < n_ids; ++id) { tok[2 * id] = tok_off[id]; tok[2 * id + 1] = tok_len[id]; }
    const int64_t b_tok = 0, b_outof = b_tok + align256v(8 * n_ids),
                  b_intof = b_outof + align256v(4 * (int64_t)out_of.size()),
                  b_pool = b_intof + align256v(4 * (int64_t)int_of.size()),
                  b_total = b_pool + align256v((int64_t)pool.size());
    std::vector<char> blob((size_t)b_total, 0);
    memcpy(blob.data() + b_tok, tok.data(), tok.size() * 4);
    if (!out_of.empty()) memcpy(blob.data() + b_outof, out_of.data(), out_of.size() * 4);
    if (!int_of.empty()) memcpy(blob.data() + b_intof, int_of.data(), int_of.size() * 4);
    memcpy(blob.data() + b_pool, pool.data(), pool.size());

    bpe_vocab *v = new (std::nothrow) bpe_vocab();
    if (!v) { set_error("out of host memory"); return BPE_ERR_SIZE; }
    hipError_t e = hipGetDevice(&v->device);
    if (e != hipSuccess) { delete v; return hip_fail(e, "hipGetDevice"); }
    e = hipMalloc(&v->device_mem, blob.size());
    if (e != hipSuccess) { delete v; return hip_fail(e, "hipMalloc(vocab)"); }
    e = hipMemcpy(v->device_mem, blob.data(), blob.size(), hipMemcpyHostToDevice);
    if (e != hipSuccess) { (void)hipFree(v->device_mem); delete v; return hip_fail(e, "hipMemcpy(vocab)"); }
    char *d = (char *)v->device_mem;
    v->tok = (const uint2 *)(d + b_tok);
    v->out_of = out_of.empty() ? nullptr : (const int32_t *)(d + b_outof);
    v->int_of = int_of.empty() ? nullptr : (const int32_t *)(d + b_intof);
    v->pool = (const uint8_t *)(d + b_pool);
    v->n_out = (int32_t)int_of.size();
    v->info.n_ids = n_ids;
    v->info.n_output_ids = (int64_t)int_of.size();
    v->info.pool_bytes = (int64_t)pool.size();
    v->info.device_bytes = b_total;
    v->info.max_token_bytes = (int32_t)longest;
    v->info.has_output_ids = output_ids ? 1 : 0;
    *out_vocab = v;
    return BPE_OK;
}

extern "C" int bpe_vocab_free(bpe_vocab *v) {
    if (!v) return BPE_OK;
    hipError_t e = hipFree(v->device_mem);
    delete v;
    return e == hipSuccess ? BPE_OK : hip_fail(e, "hipFree(vocab)");
}

extern "C" int bpe_vocab_info(const bpe_vocab *v, bpe_vocab_info_t *info) {
    if (!v || !info) { set_error("null pointer"); return BPE_ERR_NULL; }
    *info = v->info;
    return BPE_OK;
}

extern "C" int bpe_map_ids(const bpe_vocab *v, const int32_t *ids_in, int32_t *ids_out, int64_t n,
                           const int32_t *n_device, int to_output_ids, void *stream) {
    if (!v || (n > 0 && (!ids_in || !ids_out))) { set_error("null pointer"); return BPE_ERR_NULL; }
    if (n < 0 || n >= 0x7FFFFFFFll * kGroupThreads) { set_error("n out of range"); return BPE_ERR_SIZE; }
    if (!v->out_of) { set_error("the vocabulary was built without output ids"); return BPE_ERR_OPTION; }
    if (n == 0) return BPE_OK;
    const int dev_rc = check_device(v->device, "the vocabulary");
    if (dev_rc != BPE_OK) return dev_rc;
    MapParams p = {};
    p.table = to_output_ids ? v->out_of : v->int_of;
    p.n_table = to_output_ids ? (int32_t)v->info.n_ids : v->n_out;
    p.in = ids_in;
    p.out = ids_out;
    p.n = n;
    p.n_dev = n_device;
    hipLaunchKernelGGL(map_ids_kernel, dim3((unsigned)((n + kGroupThreads - 1) / kGroupThreads)), dim3(kGroupThreads),
                       0, (hipStream_t)stream, p);
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? BPE_OK : hip_fail(e, "bpe_map_ids launch");
}

extern "C" int64_t bpe_decode_workspace_bytes(int64_t n_tokens) {
    if (n_tokens < 0 || n_tokens >= 0x7FFFFFFFll) { set_error("n_tokens out of range (%lld)", (long long)n_tokens); return BPE_ERR_SIZE; }
    const int64_t n_tiles = std::max<int64_t>((n_tokens + kTileTokens - 1) / kTileTokens, 1);
    return 256 + align256v(8 * n_tiles);
}

extern "C" int bpe_decode(const bpe_vocab *v, const int32_t *ids, int64_t n_tokens, const int32_t *n_tokens_device,
                          int ids_are_output_ids, uint8_t *out_bytes, int64_t out_capacity,
                          int32_t *token_byte_offsets, int32_t *n_bytes, void *workspace, int64_t workspace_bytes,
                          void *stream) {
    if (!v || (n_tokens > 0 && !ids) || (out_capacity > 0 && !out_bytes)) { set_error("null pointer"); return BPE_ERR_NULL; }
    if (out_capacity < 0 || out_capacity >= 0x7FFFFFFFll) { set_error("out_capacity out of range (%lld)", (long long)out_capacity); return BPE_ERR_SIZE; }
    const int64_t need = bpe_decode_workspace_bytes(n_tokens);
    if (need < 0) return (int)need;
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < need) {
        set_error("workspace must be 256-byte aligned and hold %lld bytes (got %lld)", (long long)need,
                  (long long)workspace_bytes);
        return BPE_ERR_WORKSPACE;
    }
    if (ids_are_output_ids && !v->int_of) { set_error("the vocabulary was built without output ids"); return BPE_ERR_OPTION; }
    const int dev_rc = check_device(v->device, "the vocabulary");
    if (dev_rc != BPE_OK) return dev_rc;
    DecodeParams p = {};
    p.tok = v->tok;
    p.int_of = ids_are_output_ids ? v->int_of : nullptr;
    p.pool = v->pool;
    p.n_ids = (int32_t)v->info.n_ids;
    p.n_out = v->n_out;
    p.ids = ids;
    p.n_tokens = (int32_t)n_tokens;
    p.n_tokens_dev = n_tokens_device;
    p.out = out_bytes;
    p.out_capacity = (int32_t)out_capacity;
    p.token_byte_offsets = token_byte_offsets;
    p.n_bytes = n_bytes;
    p.status = (int32_t *)workspace;
    p.tile_state = (unsigned long long *)((char *)workspace + 256);
    p.call_id = next_call_id();
    // Deep grids want fewer, larger tiles and a narrow look-back (every state word of
    // another workgroup is an uncached read), but the registers of a round cost
    // occupancy: 40 M tokens take 643 us with (1 round, 256 tiles looked at per round),
    // 558 with (1, 32), 434 with (2, 32), 393 with (4, 32), 519 with (8, 256: 224 VGPRs);
    // 2.1 M tokens take 33 us with (1, 256), 25 with (2, 64), 29 with (4, 32).
    const dim3 block(kGroupThreads);
    auto tiles = [&](int rounds) { return (unsigned)std::max<int64_t>((n_tokens + rounds * kTileTokens - 1) / (rounds * kTileTokens), 1); };
    const hipStream_t st = (hipStream_t)stream;
    if (n_tokens <= 512 * kTileTokens) hipLaunchKernelGGL((decode_kernel<1, kGroupThreads>), dim3(tiles(1)), block, 0, st, p);
    else if (n_tokens <= 4096 * kTileTokens) hipLaunchKernelGGL((decode_kernel<2, 64>), dim3(tiles(2)), block, 0, st, p);
    else hipLaunchKernelGGL((decode_kernel<4, 32>), dim3(tiles(4)), block, 0, st, p);
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? BPE_OK : hip_fail(e, "bpe_decode launch");
}

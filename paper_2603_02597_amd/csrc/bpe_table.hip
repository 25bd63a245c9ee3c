// Merge-table validation, host slot image, device upload and the stand-alone
// pair-lookup kernel.  In the host image keys and values are the packed 64-bit
// words of the paper's section 3.3; the placement is two-choice instead of linear
// probing, and the device copy keeps 8 bytes per slot (see TableView).
#include <algorithm>
#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "bpe_common.h"

namespace bpe {

static thread_local char g_error[512] = "";

// Identifier of one call of the library, never 0 in its low 30 bits: the kernels of a call stamp the flags
// they leave in a workspace with it, so that flags of earlier calls read as unset without any clearing.
static std::atomic<int32_t> g_call_id{1};

int32_t next_call_id() {
    int32_t id;
    do {
        const uint32_t n = (uint32_t)g_call_id.fetch_add(1);
        id = (int32_t)((n * 0x9E3779B1u) ^ 0x7F4A7C15u);
    } while ((id & 0x3FFFFFFF) == 0);
    return id;
}

void set_error(const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
}

int hip_fail(hipError_t e, const char *what) {
    set_error("%s: %s", what, hipGetErrorString(e));
    return BPE_ERR_HIP;
}

__global__ void __launch_bounds__(256) lookup_kernel(TableView t, int32_t max_id, const int32_t *pairs,
                                                    int64_t n, int32_t *out_rank, int32_t *out_merged) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int32_t a = pairs[2 * i], b = pairs[2 * i + 1];
    int32_t rank = -1, merged = -1;
    if (a >= 0 && b >= 0 && a <= max_id && b <= max_id) {
        const uint32_t r = table_find(t, (uint32_t)a, (uint32_t)b);
        if (r != kNoRank) { rank = t.rank_of[r >> kRankShift]; merged = (int32_t)merged_id_of(t, r >> kRankShift); }
    }
    out_rank[i] = rank;
    out_merged[i] = merged;
}

static int log2_exact(int64_t v) {
    int l = 0;
    while ((1ll << l) < v) ++l;
    return l;
}

struct HostImage {
    std::vector<uint64_t> slots;        // 2 words per slot
    std::vector<uint32_t> byte_pairs;   // rank word per pair of bytes
    std::vector<int32_t> merged_of, rank_of;
    std::vector<uint32_t> sym_lr;       // 2 words per id: lowest rank order of a rule with the id as right / left part
    bpe_table_info_t info;
    int32_t merged_delta;
};

// Place every key at one of its two slots; evict and re-place along the way.
static bool place_all(const std::vector<uint64_t> &keys, const std::vector<uint64_t> &vals, int64_t half,
                      int index_bits, const HashSeed &seed, std::vector<uint64_t> &slots) {
    const int low_bits = 24 - index_bits;
    std::fill(slots.begin(), slots.end(), ~0ull);
    for (size_t i = 0; i < keys.size(); ++i) {
        uint64_t key = keys[i], val = vals[i];
        int side = 0;
        bool placed = false;
        for (int kick = 0; kick < 1000; ++kick) {
            const uint32_t a = (uint32_t)(key >> 32), b = (uint32_t)key;
            const uint64_t p1 = slot_of(mix1(seed, a, b), low_bits, index_bits);
            const uint64_t p2 = (uint64_t)half + slot_of(mix2(seed, a, b), low_bits, index_bits);
            if (kick == 0 && slots[2 * p1] == kEmptyKey) { slots[2 * p1] = key; slots[2 * p1 + 1] = val; placed = true; break; }
            if (kick == 0 && slots[2 * p2] == kEmptyKey) { slots[2 * p2] = key; slots[2 * p2 + 1] = val; placed = true; break; }
            const uint64_t p = side == 0 ? p1 : p2;
            std::swap(key, slots[2 * p]);
            std::swap(val, slots[2 * p + 1]);
            if (key == kEmptyKey) { placed = true; break; }
            side ^= 1;     // the evicted key goes to its slot in the other half
        }
        if (!placed) return false;
    }
    return true;
}

int check_device(int device, const char *what) {
    int cur = -1;
    const hipError_t e = hipGetDevice(&cur);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (cur != device) {
        set_error("%s lives on device %d but the current device is %d", what, device, cur);
        return BPE_ERR_HIP;
    }
    return BPE_OK;
}

int order_rules(const int32_t *merges, const int32_t *ranks, const int32_t *merged_ids, int64_t n, RuleOrder &ro) {
    if (n < 0 || n >= (1ll << kMaxRulesLog2)) { set_error("n_merges %lld out of range", (long long)n); return BPE_ERR_SIZE; }
    if (n > 0 && !merges) { set_error("null pointer"); return BPE_ERR_NULL; }
    // rows in rank order; ranks unique and non-negative
    std::vector<std::pair<int64_t, int64_t>> &by_rank = ro.by_rank;
    by_rank.assign((size_t)n, {0, 0});
    for (int64_t i = 0; i < n; ++i) {
        const int64_t r = ranks ? ranks[i] : i;
        if (r < 0) { set_error("rank %lld of rule %lld is negative", (long long)r, (long long)i); return BPE_ERR_DUP_RANK; }
        by_rank[i] = {r, i};
    }
    std::sort(by_rank.begin(), by_rank.end());
    for (int64_t i = 1; i < n; ++i)
        if (by_rank[i].first == by_rank[i - 1].first) { set_error("rank %lld appears twice", (long long)by_rank[i].first); return BPE_ERR_DUP_RANK; }

    // merged ids: >= 256, < 2^24, unique; remember the rank order that makes each id
    int64_t max_id = 255;
    std::vector<int64_t> &merged_row = ro.merged_row;
    merged_row.assign((size_t)n, 0);
    for (int64_t i = 0; i < n; ++i) {
        const int64_t m = merged_ids ? (int64_t)merged_ids[i] : 256 + (ranks ? (int64_t)ranks[i] : i);
        if (m < 256 || m >= (1ll << kIdBits)) { set_error("merged id %lld of rule %lld is outside [256, 2^24)", (long long)m, (long long)i); return BPE_ERR_ID_RANGE; }
        merged_row[i] = m;
        if (m > max_id) max_id = m;
    }
    ro.max_id = max_id;
    std::vector<int32_t> &made_at = ro.made_at;   // -2 unknown id, -1 byte, else rank order
    made_at.assign((size_t)(max_id + 1), -2);
    for (int b = 0; b < 256; ++b) made_at[b] = -1;
    for (int64_t k = 0; k < n; ++k) {
        const int64_t m = merged_row[by_rank[k].second];
        if (made_at[m] != -2) { set_error("merged id %lld is produced twice", (long long)m); return BPE_ERR_DUP_MERGED; }
        made_at[m] = (int32_t)k;
    }
    // parts must exist and be made by strictly earlier ranks
    for (int64_t k = 0; k < n; ++k) {
        const int64_t i = by_rank[k].second;
        for (int s = 0; s < 2; ++s) {
            const int64_t part = merges[2 * i + s];
            if (part < 0 || part > max_id || made_at[part] == -2) { set_error("rule %lld uses unknown id %lld", (long long)i, (long long)part); return BPE_ERR_ID_RANGE; }
            if (made_at[part] >= k) { set_error("rule %lld (rank %lld) uses id %lld that an equal or later rank makes", (long long)i, (long long)by_rank[k].first, (long long)part); return BPE_ERR_ORDER; }
        }
    }
    return BPE_OK;
}

static int build_image(const int32_t *merges, const int32_t *ranks, const int32_t *merged_ids, int64_t n,
                       HostImage &img) {
    RuleOrder ro;
    const int rc = order_rules(merges, ranks, merged_ids, n, ro);
    if (rc != BPE_OK) return rc;
    const std::vector<std::pair<int64_t, int64_t>> &by_rank = ro.by_rank;
    const std::vector<int64_t> &merged_row = ro.merged_row;
    const int64_t max_id = ro.max_id;
    const int64_t cap = bpe_table_capacity(n);
    // keys and values in rank order; duplicates show up as equal neighbours after sorting
    std::vector<uint64_t> keys((size_t)n), vals((size_t)n);
    img.merged_of.assign((size_t)std::max<int64_t>(n, 1), 0);
    img.rank_of.assign((size_t)std::max<int64_t>(n, 1), 0);
    img.byte_pairs.assign(65536, kNoRank);
    img.merged_delta = n > 0 ? (int32_t)merged_row[by_rank[0].second] : 256;
    std::vector<uint8_t> is_left((size_t)(max_id + 1), 0), is_right((size_t)(max_id + 1), 0);
    for (int64_t i = 0; i < n; ++i) { is_left[merges[2 * i]] = 1; is_right[merges[2 * i + 1]] = 1; }
    img.sym_lr.assign(2 * (size_t)(max_id + 1), kNoRank);
    for (int64_t k = 0; k < n; ++k) {
        const int64_t i = by_rank[k].second;
        const uint32_t a = (uint32_t)merges[2 * i], b = (uint32_t)merges[2 * i + 1];
        if (img.sym_lr[2 * (size_t)b] == kNoRank) img.sym_lr[2 * (size_t)b] = (uint32_t)k;          // b as right part
        if (img.sym_lr[2 * (size_t)a + 1] == kNoRank) img.sym_lr[2 * (size_t)a + 1] = (uint32_t)k;  // a as left part
        const uint32_t word = (uint32_t)k | (is_left[merged_row[i]] ? kCanLeft : 0u) |
                              (is_right[merged_row[i]] ? kCanRight : 0u);
        keys[k] = ((uint64_t)a << 32) | b;
        vals[k] = ((uint64_t)merged_row[i] << 32) | (uint64_t)word;
        img.merged_of[k] = (int32_t)merged_row[i];
        img.rank_of[k] = (int32_t)by_rank[k].first;
        if (merged_row[i] != (int64_t)img.merged_delta + k) img.merged_delta = -1;
        if (a < 256 && b < 256) img.byte_pairs[(a << 8) | b] = device_rank_word(word);
    }
    {
        std::vector<uint64_t> sorted(keys);
        std::sort(sorted.begin(), sorted.end());
        for (int64_t k = 1; k < n; ++k)
            if (sorted[k] == sorted[k - 1]) { set_error("pair (%u, %u) appears twice", (uint32_t)(sorted[k] >> 32), (uint32_t)sorted[k]); return BPE_ERR_DUP_PAIR; }
    }
    img.slots.assign((size_t)cap * 2, ~0ull);
    const int64_t half = cap / 2;
    const int index_bits = log2_exact(half);
    int attempt = 0;
    for (; attempt < kHashSeeds; ++attempt)
        if (place_all(keys, vals, half, index_bits, hash_seed(attempt), img.slots)) break;
    if (attempt == kHashSeeds) { set_error("could not place the keys with any of the %d hash seeds", kHashSeeds); return BPE_ERR_SIZE; }
    img.info.n_merges = n;
    img.info.capacity = cap;
    img.info.device_bytes = cap * 8 + 65536 * 4 + 2 * 4 * std::max<int64_t>(n, 1) + 8 * (max_id + 1);
    img.info.hash_attempt = attempt;
    img.info.max_id = (int32_t)max_id;
    return BPE_OK;
}

}  // namespace bpe

using namespace bpe;

extern "C" const char *bpe_last_error(void) { return g_error; }

extern "C" int64_t bpe_table_capacity(int64_t n_merges) {
    if (n_merges < 0 || n_merges >= (1ll << kMaxRulesLog2)) return BPE_ERR_SIZE;
    // Two-choice placement needs a load factor safely below 1/2: at most 0.4.  Never
    // fewer than 2^16 slots per half (1 MiB on the device in all): a device slot keeps
    // 32 bits of its key, the right id (24 bits) and the 24 - log2(half) bits of the
    // mix that the slot index does not hold.
    int64_t cap = 131072;
    while (2 * cap < 5 * n_merges) cap <<= 1;
    return cap;
}

extern "C" int bpe_table_image_build(const int32_t *merges, const int32_t *ranks,
                                     const int32_t *merged_ids, int64_t n, uint64_t *slots,
                                     int64_t capacity_slots, bpe_table_info_t *info) {
    if (!slots) { set_error("null pointer"); return BPE_ERR_NULL; }
    const int64_t cap = bpe_table_capacity(n);
    if (cap < 0) { set_error("n_merges %lld out of range", (long long)n); return BPE_ERR_SIZE; }
    if (capacity_slots != cap) { set_error("capacity_slots must be %lld", (long long)cap); return BPE_ERR_SIZE; }
    HostImage img;
    int rc = build_image(merges, ranks, merged_ids, n, img);
    if (rc != BPE_OK) return rc;
    memcpy(slots, img.slots.data(), (size_t)cap * 16);
    if (info) *info = img.info;
    return BPE_OK;
}

extern "C" int bpe_table_build(const int32_t *merges, const int32_t *ranks, const int32_t *merged_ids,
                               int64_t n, bpe_table **out_table) {
    if (!out_table) { set_error("out_table is NULL"); return BPE_ERR_NULL; }
    *out_table = nullptr;
    HostImage img;
    int rc = build_image(merges, ranks, merged_ids, n, img);
    if (rc != BPE_OK) return rc;
    // device slots: 8 bytes each, from the image's {key, value} pairs
    const int64_t half = img.info.capacity / 2;
    const int index_bits = log2_exact(half), low_bits = 24 - index_bits;
    const HashSeed seed = hash_seed(img.info.hash_attempt);
    std::vector<uint32_t> dev_slots((size_t)img.info.capacity * 2);
    for (int64_t i = 0; i < img.info.capacity; ++i) {
        const uint64_t key = img.slots[2 * (size_t)i], val = img.slots[2 * (size_t)i + 1];
        uint32_t rest = 0, word = kNoRank;
        if (key != kEmptyKey) {
            const uint32_t a = (uint32_t)(key >> 32), b = (uint32_t)key;
            rest = key_rest(i < half ? mix1(seed, a, b) : mix2(seed, a, b), low_bits, b);
            word = device_rank_word((uint32_t)val);
        }
        dev_slots[2 * (size_t)i] = rest;
        dev_slots[2 * (size_t)i + 1] = word;
    }
    const size_t slot_bytes = dev_slots.size() * 4, bp_bytes = img.byte_pairs.size() * 4;
    const size_t arr_bytes = ((img.merged_of.size() * 4 + 255) / 256) * 256;
    const size_t lr_bytes = img.sym_lr.size() * 4;
    std::vector<char> blob(slot_bytes + bp_bytes + 2 * arr_bytes + lr_bytes, 0);
    memcpy(blob.data(), dev_slots.data(), slot_bytes);
    memcpy(blob.data() + slot_bytes, img.byte_pairs.data(), bp_bytes);
    memcpy(blob.data() + slot_bytes + bp_bytes, img.merged_of.data(), img.merged_of.size() * 4);
    memcpy(blob.data() + slot_bytes + bp_bytes + arr_bytes, img.rank_of.data(), img.rank_of.size() * 4);
    memcpy(blob.data() + slot_bytes + bp_bytes + 2 * arr_bytes, img.sym_lr.data(), lr_bytes);

    bpe_table *t = new (std::nothrow) bpe_table();
    if (!t) { set_error("out of host memory"); return BPE_ERR_SIZE; }
    hipError_t e = hipGetDevice(&t->device);
    if (e != hipSuccess) { delete t; return hip_fail(e, "hipGetDevice"); }
    e = hipMalloc(&t->device_mem, blob.size());
    if (e != hipSuccess) { delete t; return hip_fail(e, "hipMalloc(table)"); }
    e = hipMemcpy(t->device_mem, blob.data(), blob.size(), hipMemcpyHostToDevice);
    if (e != hipSuccess) { (void)hipFree(t->device_mem); delete t; return hip_fail(e, "hipMemcpy(table)"); }
    t->info = img.info;
    t->info.device_bytes = (int64_t)blob.size();
    char *d = (char *)t->device_mem;
    t->view.slots = (const uint2 *)d;
    t->view.byte_pairs = (const uint32_t *)(d + slot_bytes);
    t->view.merged_of = (const int32_t *)(d + slot_bytes + bp_bytes);
    t->view.rank_of = (const int32_t *)(d + slot_bytes + bp_bytes + arr_bytes);
    t->view.sym_lr = (const uint2 *)(d + slot_bytes + bp_bytes + 2 * arr_bytes);
    t->view.half = (uint32_t)half;
    t->view.low_bits = low_bits;
    t->view.index_bits = index_bits;
    t->view.merged_delta = img.merged_delta;
    t->view.seed = seed;
    *out_table = t;
    return BPE_OK;
}

extern "C" int bpe_table_free(bpe_table *t) {
    if (!t) return BPE_OK;
    hipError_t e = hipFree(t->device_mem);
    delete t;
    return e == hipSuccess ? BPE_OK : hip_fail(e, "hipFree(table)");
}

extern "C" int bpe_table_info(const bpe_table *t, bpe_table_info_t *info) {
    if (!t || !info) { set_error("null pointer"); return BPE_ERR_NULL; }
    *info = t->info;
    return BPE_OK;
}

extern "C" int bpe_table_lookup(const bpe_table *t, const int32_t *pairs, int64_t n,
                                int32_t *out_rank, int32_t *out_merged, void *stream) {
    if (!t || (n > 0 && (!pairs || !out_rank || !out_merged))) { set_error("null pointer"); return BPE_ERR_NULL; }
    if (n < 0 || n > 0x7FFFFFFFll * 128) { set_error("n out of range"); return BPE_ERR_SIZE; }
    if (n == 0) return BPE_OK;
    const int dev_rc = check_device(t->device, "the table");
    if (dev_rc != BPE_OK) return dev_rc;
    const unsigned grid = (unsigned)((n + 255) / 256);
    hipLaunchKernelGGL(lookup_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, t->view, t->info.max_id,
                       pairs, n, out_rank, out_merged);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? BPE_OK : hip_fail(e, "lookup_kernel launch");
}

// Merge-table validation, host slot image, device upload and the stand-alone
// pair-lookup kernel.  Table format: paper section 3.3 (64-bit packed key and
// value, linear probing, about 50 % load).
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "bpe_common.h"

namespace bpe {

static thread_local char g_error[512] = "";

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

__global__ void __launch_bounds__(256) lookup_kernel(TableView t, const int32_t *pairs, int64_t n,
                                                    int32_t *out_rank, int32_t *out_merged) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int32_t a = pairs[2 * i], b = pairs[2 * i + 1];
    uint32_t merged = 0xFFFFFFFFu, rank = kNoRank;
    if (a >= 0 && b >= 0) rank = table_find(t, (uint32_t)a, (uint32_t)b, merged);
    out_rank[i] = (int32_t)rank;      // kNoRank -> -1
    out_merged[i] = (int32_t)merged;
}

static int log2_exact(int64_t v) {
    int l = 0;
    while ((1ll << l) < v) ++l;
    return l;
}

}  // namespace bpe

using namespace bpe;

extern "C" const char *bpe_last_error(void) { return g_error; }

extern "C" int64_t bpe_table_capacity(int64_t n_merges) {
    if (n_merges < 0 || n_merges >= (1ll << kRankBits)) return BPE_ERR_SIZE;
    int64_t cap = 16;
    while (cap < 2 * n_merges) cap <<= 1;
    return cap;
}

extern "C" int bpe_table_image_build(const int32_t *merges, const int32_t *ranks,
                                     const int32_t *merged_ids, int64_t n, uint64_t *slots,
                                     int64_t capacity_slots, bpe_table_info_t *info) {
    if (n < 0 || n >= (1ll << kRankBits)) { set_error("n_merges %lld out of range", (long long)n); return BPE_ERR_SIZE; }
    if ((n > 0 && !merges) || !slots) { set_error("null pointer"); return BPE_ERR_NULL; }
    const int64_t cap = bpe_table_capacity(n);
    if (capacity_slots != cap) { set_error("capacity_slots must be %lld", (long long)cap); return BPE_ERR_SIZE; }

    // rows in rank order; ranks unique and below 2^26
    std::vector<std::pair<int64_t, int64_t>> by_rank((size_t)n);
    for (int64_t i = 0; i < n; ++i) {
        const int64_t r = ranks ? ranks[i] : i;
        if (r < 0 || r >= (1ll << kRankBits)) { set_error("rank %lld of rule %lld is outside [0, 2^26)", (long long)r, (long long)i); return BPE_ERR_DUP_RANK; }
        by_rank[i] = {r, i};
    }
    std::sort(by_rank.begin(), by_rank.end());
    for (int64_t i = 1; i < n; ++i)
        if (by_rank[i].first == by_rank[i - 1].first) { set_error("rank %lld appears twice", (long long)by_rank[i].first); return BPE_ERR_DUP_RANK; }
    // merged ids: >= 256, unique; remember the rank that makes each id
    int64_t max_id = 255;
    for (int64_t i = 0; i < n; ++i) {
        const int64_t m = merged_ids ? merged_ids[i] : 256 + (ranks ? ranks[i] : i);
        if (m < 256 || m > 0x7FFFFFFE) { set_error("merged id %lld of rule %lld out of range", (long long)m, (long long)i); return BPE_ERR_ID_RANGE; }
        if (m > max_id) max_id = m;
    }
    if (max_id - 255 > 64 * (n + 1) + (1 << 20)) { set_error("merged ids are too sparse"); return BPE_ERR_ID_RANGE; }
    std::vector<int32_t> made_at((size_t)(max_id + 1), -2);   // -2 unknown id, -1 byte, else rank
    for (int b = 0; b < 256; ++b) made_at[b] = -1;
    for (int64_t i = 0; i < n; ++i) {
        const int64_t r = ranks ? ranks[i] : i;
        const int64_t m = merged_ids ? merged_ids[i] : 256 + r;
        if (made_at[m] != -2) { set_error("merged id %lld is produced twice", (long long)m); return BPE_ERR_DUP_MERGED; }
        made_at[m] = (int32_t)r;
    }
    // parts must exist and be made by strictly earlier ranks
    for (int64_t i = 0; i < n; ++i) {
        const int64_t r = ranks ? ranks[i] : i;
        for (int s = 0; s < 2; ++s) {
            const int64_t part = merges[2 * i + s];
            if (part < 0 || part > max_id || made_at[part] == -2) { set_error("rule %lld uses unknown id %lld", (long long)i, (long long)part); return BPE_ERR_ID_RANGE; }
            if (made_at[part] >= r) { set_error("rule %lld (rank %lld) uses id %lld made at rank %d", (long long)i, (long long)r, (long long)part, made_at[part]); return BPE_ERR_ORDER; }
        }
    }
    // place keys in rank order (deterministic image), linear probing
    for (int64_t s = 0; s < cap; ++s) { slots[2 * s] = kEmptyKey; slots[2 * s + 1] = ~0ull; }
    const int shift = 32 - log2_exact(cap);
    int max_probe = 0;
    for (int64_t k = 0; k < n; ++k) {
        const int64_t r = by_rank[k].first, i = by_rank[k].second;
        const uint32_t a = (uint32_t)merges[2 * i], b = (uint32_t)merges[2 * i + 1];
        const uint64_t key = ((uint64_t)a << 32) | b;
        const uint64_t m = (uint64_t)(merged_ids ? merged_ids[i] : 256 + r);
        uint32_t idx = pair_hash(a, b) >> shift;
        int probe = 1;
        while (slots[2 * (uint64_t)idx] != kEmptyKey) {
            if (slots[2 * (uint64_t)idx] == key) { set_error("pair (%u, %u) appears twice", a, b); return BPE_ERR_DUP_PAIR; }
            idx = (idx + 1) & (uint32_t)(cap - 1);
            ++probe;
        }
        slots[2 * (uint64_t)idx] = key;
        slots[2 * (uint64_t)idx + 1] = (m << 32) | (uint64_t)r;
        if (probe > max_probe) max_probe = probe;
    }
    if (info) {
        info->n_merges = n;
        info->capacity = cap;
        info->device_bytes = cap * 16;
        info->max_probe = max_probe;
        info->max_id = (int32_t)max_id;
    }
    return BPE_OK;
}

extern "C" int bpe_table_build(const int32_t *merges, const int32_t *ranks, const int32_t *merged_ids,
                               int64_t n, bpe_table **out_table) {
    if (!out_table) { set_error("out_table is NULL"); return BPE_ERR_NULL; }
    *out_table = nullptr;
    const int64_t cap = bpe_table_capacity(n);
    if (cap < 0) { set_error("n_merges %lld out of range", (long long)n); return BPE_ERR_SIZE; }
    std::vector<uint64_t> image((size_t)cap * 2);
    bpe_table_info_t info;
    int rc = bpe_table_image_build(merges, ranks, merged_ids, n, image.data(), cap, &info);
    if (rc != BPE_OK) return rc;
    bpe_table *t = new (std::nothrow) bpe_table();
    if (!t) { set_error("out of host memory"); return BPE_ERR_SIZE; }
    hipError_t e = hipGetDevice(&t->device);
    if (e != hipSuccess) { delete t; return hip_fail(e, "hipGetDevice"); }
    e = hipMalloc(&t->device_slots, (size_t)cap * 16);
    if (e != hipSuccess) { delete t; return hip_fail(e, "hipMalloc(table)"); }
    e = hipMemcpy(t->device_slots, image.data(), (size_t)cap * 16, hipMemcpyHostToDevice);
    if (e != hipSuccess) { (void)hipFree(t->device_slots); delete t; return hip_fail(e, "hipMemcpy(table)"); }
    t->info = info;
    t->view.slots = (const uint4 *)t->device_slots;
    t->view.mask = (uint32_t)(cap - 1);
    t->view.shift = 32 - log2_exact(cap);
    t->view.max_probe = info.max_probe > 0 ? info.max_probe : 1;
    *out_table = t;
    return BPE_OK;
}

extern "C" int bpe_table_free(bpe_table *t) {
    if (!t) return BPE_OK;
    hipError_t e = hipFree(t->device_slots);
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
    const unsigned grid = (unsigned)((n + 255) / 256);
    hipLaunchKernelGGL(lookup_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, t->view, pairs, n,
                       out_rank, out_merged);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? BPE_OK : hip_fail(e, "lookup_kernel launch");
}

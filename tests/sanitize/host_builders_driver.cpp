// Calls the host-only parts of the library (rule validation, two-choice placement of the slot image, token
// expansions of the vocabulary) on valid and invalid tables; built by tests/test_sanitizers.py with the host
// sanitizers (address, undefined), so a stray access or an undefined integer operation in them ends the run.
// Needs no GPU: bpe_vocab_build does all of its host work before its first HIP call, which may then fail.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "bpe_mi355x.h"

#define CHECK(cond) do { if (!(cond)) { std::fprintf(stderr, "check failed, line %d: %s (%s)\n", __LINE__, #cond, bpe_last_error()); return 1; } } while (0)

static uint64_t state = 0x1234567887654321ull;
static uint32_t draw(uint32_t n) {
    state ^= state >> 12; state ^= state << 25; state ^= state >> 27;
    return (uint32_t)((state * 0x2545F4914F6CDD1Dull) >> 33) % n;
}

// n rules that satisfy the order property: rule k joins two ids that exist before it, each pair once
static std::vector<int32_t> random_rules(int64_t n) {
    std::vector<int32_t> m;
    std::vector<uint64_t> seen;
    for (int64_t k = 0; k < n; ++k) {
        for (;;) {
            const int32_t a = (int32_t)draw((uint32_t)(256 + k)), b = (int32_t)draw((uint32_t)(256 + k));
            const uint64_t key = ((uint64_t)a << 32) | (uint32_t)b;
            bool dup = false;
            for (uint64_t s : seen) if (s == key) { dup = true; break; }
            if (dup) continue;
            seen.push_back(key); m.push_back(a); m.push_back(b);
            break;
        }
    }
    return m;
}

static int image(const std::vector<int32_t> &m, const int32_t *ranks, const int32_t *ids, bpe_table_info_t *info) {
    const int64_t n = (int64_t)m.size() / 2, cap = bpe_table_capacity(n);
    std::vector<uint64_t> slots((size_t)(2 * cap));
    const int rc = bpe_table_image_build(m.data(), ranks, ids, n, slots.data(), cap, info);
    if (rc == BPE_OK) {                      // every rule is in one of its two slots, and nothing else is stored
        int64_t used = 0;
        for (int64_t i = 0; i < cap; ++i) used += slots[2 * i] != ~0ull;
        if (used != n) { std::fprintf(stderr, "%lld slots used for %lld rules\n", (long long)used, (long long)n); return 1000; }
    }
    return rc;
}

int main() {
    CHECK(bpe_table_capacity(-1) == BPE_ERR_SIZE && bpe_table_capacity(0) == 131072 && bpe_table_capacity(100000) == 262144);
    bpe_table_info_t info;
    for (int64_t n : {0ll, 1ll, 700ll, 3000ll}) {
        const std::vector<int32_t> m = random_rules(n);
        CHECK(image(m, nullptr, nullptr, &info) == BPE_OK && info.n_merges == n && info.max_id == 255 + n);
    }
    std::vector<int32_t> m = random_rules(500);
    {   // ranks and merged ids of the caller's own: a permutation of the rows keeps the table valid
        std::vector<int32_t> ranks(500), ids(500), rows;
        for (int i = 0; i < 500; ++i) { ranks[i] = 3 * i + 7; ids[i] = 256 + i; }
        CHECK(image(m, ranks.data(), ids.data(), &info) == BPE_OK);
        ids[499] = 5000000;                                   // sparse ids up to 2^24
        CHECK(image(m, ranks.data(), ids.data(), &info) == BPE_OK && info.max_id == 5000000);
        ids[499] = 1 << 24;
        CHECK(image(m, ranks.data(), ids.data(), nullptr) == BPE_ERR_ID_RANGE);
        ids[499] = ids[3];
        CHECK(image(m, ranks.data(), ids.data(), nullptr) == BPE_ERR_DUP_MERGED);
        ids[499] = 256 + 499; ranks[10] = ranks[11];
        CHECK(image(m, ranks.data(), ids.data(), nullptr) == BPE_ERR_DUP_RANK);
        ranks[10] = -1;
        CHECK(image(m, ranks.data(), ids.data(), nullptr) == BPE_ERR_DUP_RANK);
    }
    {   std::vector<int32_t> bad = m; bad[2 * 400] = bad[0]; bad[2 * 400 + 1] = bad[1];
        CHECK(image(bad, nullptr, nullptr, nullptr) == BPE_ERR_DUP_PAIR); }
    {   std::vector<int32_t> bad = m; bad[2 * 20] = 256 + 20;                 // uses its own result
        CHECK(image(bad, nullptr, nullptr, nullptr) == BPE_ERR_ORDER); }
    {   std::vector<int32_t> bad = m; bad[2 * 20 + 1] = 256 + 300;            // made by a later rule
        CHECK(image(bad, nullptr, nullptr, nullptr) == BPE_ERR_ORDER); }
    {   std::vector<int32_t> bad = m; bad[7] = -3;
        CHECK(image(bad, nullptr, nullptr, nullptr) == BPE_ERR_ID_RANGE); }
    {   std::vector<int32_t> bad = m; bad[7] = 0x7fffffff;
        CHECK(image(bad, nullptr, nullptr, nullptr) == BPE_ERR_ID_RANGE); }
    CHECK(bpe_table_image_build(m.data(), nullptr, nullptr, 500, nullptr, 131072, nullptr) == BPE_ERR_NULL);
    {   std::vector<uint64_t> slots(2 * 1024);
        CHECK(bpe_table_image_build(m.data(), nullptr, nullptr, 500, slots.data(), 1024, nullptr) == BPE_ERR_SIZE); }

    // vocabulary: the expansions are built on the host, then uploaded (BPE_ERR_HIP where there is no device)
    bpe_vocab *v = nullptr;
    int rc = bpe_vocab_build(m.data(), nullptr, nullptr, 500, nullptr, 0, &v);
    CHECK(rc == BPE_OK || rc == BPE_ERR_HIP);
    if (rc == BPE_OK) CHECK(bpe_vocab_free(v) == BPE_OK);
    std::vector<int32_t> out_ids(256 + 500);
    for (int i = 0; i < 756; ++i) out_ids[i] = 755 - i;
    rc = bpe_vocab_build(m.data(), nullptr, nullptr, 500, out_ids.data(), 756, &v);
    CHECK(rc == BPE_OK || rc == BPE_ERR_HIP);
    if (rc == BPE_OK) CHECK(bpe_vocab_free(v) == BPE_OK);
    CHECK(bpe_vocab_build(m.data(), nullptr, nullptr, 500, out_ids.data(), 700, &v) == BPE_ERR_SIZE);
    out_ids[5] = out_ids[6];
    CHECK(bpe_vocab_build(m.data(), nullptr, nullptr, 500, out_ids.data(), 756, &v) == BPE_ERR_DUP_MERGED);
    out_ids[5] = -2;
    CHECK(bpe_vocab_build(m.data(), nullptr, nullptr, 500, out_ids.data(), 756, &v) == BPE_ERR_ID_RANGE);
    {   // a chain of doublings: the expansion of rule k has 2^(k+1) bytes, refused once it is too long to keep
        std::vector<int32_t> chain;
        for (int k = 0; k < 30; ++k) { const int32_t id = k ? 255 + k : 'a'; chain.push_back(id); chain.push_back(id); }
        CHECK(bpe_vocab_build(chain.data(), nullptr, nullptr, 30, nullptr, 0, &v) == BPE_ERR_SIZE);
    }
    std::puts("host builders under the sanitizers: ok");
    return 0;
}

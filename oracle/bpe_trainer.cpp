/*
 * Seeded-corpus BPE trainer that produces the merge tables of the benchmark
 * workloads.  TEST INFRASTRUCTURE ONLY (part of the CPU oracle): the HIP library
 * never calls it and shares no code with it.
 *
 * The paper takes GPT-2's ~50k-rule merge list as given (section 3.3) and only
 * cites classical BPE learning (section 2, "Algorithmic Variants of BPE"), so
 * the procedure is the textbook one:
 *   symbols start as bytes; for k = 0, 1, ...: count every adjacent pair
 *   occurrence (overlapping positions included) over all pieces, take the most
 *   frequent pair (ties: smallest left id, then smallest right id), give it id
 *   256 + k and rank k, and replace its non-overlapping occurrences left to
 *   right in every piece.  Stop after the requested number of merges or when no
 *   pair is left.
 * Identical pieces are folded into one word with a frequency.  Pair counts are
 * kept incrementally: a word that contains the chosen pair has all its pairs
 * un-counted, is rewritten, and has all its pairs counted again.  The maximum
 * is taken from a heap with stale entries skipped.  A naive Python trainer
 * that recounts everything per merge pins this one on small corpora
 * (tests/test_oracle_trainer.py).
 */
#include <algorithm>
#include <cstdint>
#include <queue>
#include <string>
#include <unordered_map>
#include <vector>

namespace {

struct HeapItem {
    int64_t count;
    uint64_t key;
    bool operator<(const HeapItem &o) const {   // max-heap: larger count first, then smaller key
        if (count != o.count) return count < o.count;
        return key > o.key;
    }
};

inline uint64_t pair_key(int32_t a, int32_t b) { return ((uint64_t)(uint32_t)a << 32) | (uint32_t)b; }

}  // namespace

extern "C" int64_t oracle_train(const uint8_t *bytes, const int32_t *off, int64_t n_pieces,
                                int64_t max_merges, int32_t *out_merges /* [max_merges][2] */) {
    // distinct pieces with frequencies
    std::unordered_map<std::string, int64_t> freq_of;
    for (int64_t p = 0; p < n_pieces; ++p)
        ++freq_of[std::string((const char *)bytes + off[p], (size_t)(off[p + 1] - off[p]))];
    std::vector<std::vector<int32_t>> words;
    std::vector<int64_t> freq;
    words.reserve(freq_of.size());
    for (auto &kv : freq_of) {
        std::vector<int32_t> w(kv.first.size());
        for (size_t i = 0; i < w.size(); ++i) w[i] = (uint8_t)kv.first[i];
        words.push_back(std::move(w));
        freq.push_back(kv.second);
    }

    std::unordered_map<uint64_t, int64_t> count;               // pair -> weighted occurrences
    std::unordered_map<uint64_t, std::vector<int32_t>> where;  // pair -> words that may hold it
    for (size_t w = 0; w < words.size(); ++w) {
        const auto &s = words[w];
        for (size_t i = 0; i + 1 < s.size(); ++i) {
            uint64_t k = pair_key(s[i], s[i + 1]);
            count[k] += freq[w];
            auto &v = where[k];
            if (v.empty() || v.back() != (int32_t)w) v.push_back((int32_t)w);
        }
    }
    std::priority_queue<HeapItem> heap;
    for (auto &kv : count) heap.push({kv.second, kv.first});

    int64_t n_done = 0;
    std::vector<uint64_t> touched;
    while (n_done < max_merges && !heap.empty()) {
        HeapItem top = heap.top();
        heap.pop();
        auto it = count.find(top.key);
        if (it == count.end() || it->second != top.count || top.count < 1) continue;  // stale
        const int32_t a = (int32_t)(top.key >> 32), b = (int32_t)(top.key & 0xFFFFFFFFu);
        const int32_t id = 256 + (int32_t)n_done;
        out_merges[2 * n_done] = a;
        out_merges[2 * n_done + 1] = b;
        ++n_done;

        std::vector<int32_t> holders;
        holders.swap(where[top.key]);
        std::sort(holders.begin(), holders.end());
        holders.erase(std::unique(holders.begin(), holders.end()), holders.end());
        touched.clear();
        for (int32_t w : holders) {
            auto &s = words[w];
            bool has = false;
            for (size_t i = 0; i + 1 < s.size(); ++i)
                if (s[i] == a && s[i + 1] == b) { has = true; break; }
            if (!has) continue;
            for (size_t i = 0; i + 1 < s.size(); ++i) {
                uint64_t k = pair_key(s[i], s[i + 1]);
                count[k] -= freq[w];
                touched.push_back(k);
            }
            size_t o = 0;
            for (size_t i = 0; i < s.size();) {
                if (i + 1 < s.size() && s[i] == a && s[i + 1] == b) { s[o++] = id; i += 2; }
                else { s[o++] = s[i++]; }
            }
            s.resize(o);
            for (size_t i = 0; i + 1 < s.size(); ++i) {
                uint64_t k = pair_key(s[i], s[i + 1]);
                count[k] += freq[w];
                touched.push_back(k);
                if (s[i] == id || s[i + 1] == id) {
                    auto &v = where[k];
                    if (v.empty() || v.back() != w) v.push_back(w);
                }
            }
        }
        std::sort(touched.begin(), touched.end());
        touched.erase(std::unique(touched.begin(), touched.end()), touched.end());
        for (uint64_t k : touched) {
            int64_t c = count[k];
            if (c > 0) heap.push({c, k});
            else count.erase(k);
        }
    }
    return n_done;
}

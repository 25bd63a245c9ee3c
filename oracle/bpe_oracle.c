/*
 * CPU oracle for greedy byte-level BPE encoding.  TEST INFRASTRUCTURE ONLY:
 * the tests, the smoke check and the benchmark's cpu_baseline leg call it; the
 * HIP library never does, and the two share no code.
 *
 * What it computes is the definition the paper gives in its introduction
 * (section 1): per piece, repeatedly find the adjacent pair with the best
 * (lowest) merge-table rank and merge its left-most occurrence, until no pair
 * of the sequence is in the table.  Ties go to the left-most position
 * (section 3.4, "block-wide argmin"); the loop ends when fewer than two symbols
 * remain or no pair is in the table (section 3.4, last paragraph).  A pair is
 * keyed by (a << 32) | b and maps to (merged id, rank) (section 3.3).
 *
 * Deliberately plain: the table is a key-sorted array searched with bsearch();
 * every pass rescans every pair of the piece; a merge shifts the tail left by
 * one.  Nothing is blocked, fused or cached.
 *
 * Pins (tests/test_oracle_*.py): hand-worked examples, an independent
 * "merge the lowest rank everywhere" brute force, closed forms on runs,
 * decode(encode(x)) == x and the no-mergeable-pair-left invariant.
 */
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    uint64_t key;    /* (left id << 32) | right id */
    int32_t rank;    /* lower merges first */
    int32_t merged;  /* id that replaces the pair */
} pair_entry;

typedef struct {
    pair_entry *e;   /* sorted by key */
    int64_t n;
    /* for decode: entries sorted by merged id */
    pair_entry *by_id;
} oracle_table;

static int cmp_key(const void *a, const void *b) {
    uint64_t x = ((const pair_entry *)a)->key, y = ((const pair_entry *)b)->key;
    return (x > y) - (x < y);
}
static int cmp_id(const void *a, const void *b) {
    int32_t x = ((const pair_entry *)a)->merged, y = ((const pair_entry *)b)->merged;
    return (x > y) - (x < y);
}

/* merges: [n][2] (left, right); ranks: [n]; merged_ids: [n] or NULL (then 256 + rank). */
oracle_table *oracle_table_create(const int32_t *merges, const int32_t *ranks,
                                  const int32_t *merged_ids, int64_t n) {
    oracle_table *t = (oracle_table *)calloc(1, sizeof(*t));
    t->n = n;
    t->e = (pair_entry *)malloc(sizeof(pair_entry) * (size_t)(n ? n : 1));
    t->by_id = (pair_entry *)malloc(sizeof(pair_entry) * (size_t)(n ? n : 1));
    for (int64_t i = 0; i < n; ++i) {
        t->e[i].key = ((uint64_t)(uint32_t)merges[2 * i] << 32) | (uint32_t)merges[2 * i + 1];
        t->e[i].rank = ranks[i];
        t->e[i].merged = merged_ids ? merged_ids[i] : 256 + ranks[i];
    }
    memcpy(t->by_id, t->e, sizeof(pair_entry) * (size_t)n);
    qsort(t->e, (size_t)n, sizeof(pair_entry), cmp_key);
    qsort(t->by_id, (size_t)n, sizeof(pair_entry), cmp_id);
    return t;
}

void oracle_table_free(oracle_table *t) {
    if (!t) return;
    free(t->e);
    free(t->by_id);
    free(t);
}

/* rank and merged id of pair (a, b); returns 0 if the pair is not in the table. */
int oracle_lookup(const oracle_table *t, int32_t a, int32_t b, int32_t *rank, int32_t *merged) {
    pair_entry probe;
    probe.key = ((uint64_t)(uint32_t)a << 32) | (uint32_t)b;
    const pair_entry *hit =
        (const pair_entry *)bsearch(&probe, t->e, (size_t)t->n, sizeof(pair_entry), cmp_key);
    if (!hit) return 0;
    *rank = hit->rank;
    *merged = hit->merged;
    return 1;
}

/* Encode one piece in place in s[0..len); returns the new length. */
static int64_t encode_piece(const oracle_table *t, int32_t *s, int64_t len) {
    while (len >= 2) {
        int64_t best_pos = -1;
        int32_t best_rank = 0, best_merged = 0;
        for (int64_t i = 0; i + 1 < len; ++i) {
            int32_t r, m;
            if (oracle_lookup(t, s[i], s[i + 1], &r, &m) && (best_pos < 0 || r < best_rank)) {
                best_pos = i;     /* strict '<' keeps the left-most among equal ranks */
                best_rank = r;
                best_merged = m;
            }
        }
        if (best_pos < 0) break;
        s[best_pos] = best_merged;
        memmove(s + best_pos + 1, s + best_pos + 2, sizeof(int32_t) * (size_t)(len - best_pos - 2));
        --len;
    }
    return len;
}

typedef struct {
    const oracle_table *t;
    const uint8_t *bytes;
    const int32_t *off;
    int64_t p0, p1;
    int32_t *tmp;     /* [n_bytes]: tokens of piece p at tmp[off[p] ...] */
    int32_t *count;   /* [n_pieces] */
} job;

static void *run_job(void *arg) {
    job *j = (job *)arg;
    for (int64_t p = j->p0; p < j->p1; ++p) {
        int64_t b = j->off[p], len = j->off[p + 1] - b;
        for (int64_t i = 0; i < len; ++i) j->tmp[b + i] = j->bytes[b + i];
        j->count[p] = (int32_t)encode_piece(j->t, j->tmp + b, len);
    }
    return NULL;
}

/*
 * Encode every piece bytes[off[p] : off[p+1]) independently; write all tokens
 * densely, in piece order, to out_ids (capacity off[n_pieces]) and the running
 * token counts to out_offsets[n_pieces + 1].  Pieces are split over n_threads
 * threads in contiguous ranges of equal piece count.  Returns the token total.
 */
int64_t oracle_encode(const oracle_table *t, const uint8_t *bytes, const int32_t *off,
                      int64_t n_pieces, int32_t *out_ids, int32_t *out_offsets, int n_threads) {
    int64_t n_bytes = n_pieces > 0 ? off[n_pieces] : 0;
    int32_t *tmp = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_bytes ? n_bytes : 1));
    int32_t *count = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_pieces ? n_pieces : 1));
    if (n_threads < 1) n_threads = 1;
    if (n_threads > 256) n_threads = 256;
    job jobs[256];
    pthread_t th[256];
    for (int k = 0; k < n_threads; ++k) {
        jobs[k].t = t; jobs[k].bytes = bytes; jobs[k].off = off;
        jobs[k].p0 = n_pieces * k / n_threads;
        jobs[k].p1 = n_pieces * (k + 1) / n_threads;
        jobs[k].tmp = tmp; jobs[k].count = count;
    }
    if (n_threads == 1) {
        run_job(&jobs[0]);
    } else {
        for (int k = 0; k < n_threads; ++k) pthread_create(&th[k], NULL, run_job, &jobs[k]);
        for (int k = 0; k < n_threads; ++k) pthread_join(th[k], NULL);
    }
    int64_t total = 0;
    for (int64_t p = 0; p < n_pieces; ++p) {
        out_offsets[p] = (int32_t)total;
        memcpy(out_ids + total, tmp + off[p], sizeof(int32_t) * (size_t)count[p]);
        total += count[p];
    }
    out_offsets[n_pieces] = (int32_t)total;
    free(tmp);
    free(count);
    return total;
}

/* Byte length of token id (ids below 256 are single bytes); -1 if id is unknown. */
static int64_t expand(const oracle_table *t, int32_t id, uint8_t *out, int64_t cap, int depth) {
    if (id >= 0 && id < 256) {
        if (out && cap >= 1) out[0] = (uint8_t)id;
        return 1;
    }
    if (depth > 100000) return -1;
    pair_entry probe;
    probe.merged = id;
    const pair_entry *hit =
        (const pair_entry *)bsearch(&probe, t->by_id, (size_t)t->n, sizeof(pair_entry), cmp_id);
    if (!hit) return -1;
    int32_t a = (int32_t)(hit->key >> 32), b = (int32_t)(hit->key & 0xFFFFFFFFu);
    int64_t la = expand(t, a, out, cap, depth + 1);
    if (la < 0) return -1;
    int64_t lb = expand(t, b, out ? out + (la < cap ? la : cap) : NULL, cap > la ? cap - la : 0, depth + 1);
    if (lb < 0) return -1;
    return la + lb;
}

/*
 * Inverse of encoding: replace every merged id by the two ids it was made from,
 * recursively, down to bytes.  Returns the number of bytes the ids expand to
 * (writes at most cap of them), or -1 on an unknown id.
 */
int64_t oracle_decode(const oracle_table *t, const int32_t *ids, int64_t n, uint8_t *out, int64_t cap) {
    int64_t total = 0;
    for (int64_t i = 0; i < n; ++i) {
        int64_t room = cap > total ? cap - total : 0;
        int64_t l = expand(t, ids[i], out ? out + (total < cap ? total : cap) : NULL, room, 0);
        if (l < 0) return -1;
        total += l;
    }
    return total;
}

/*
 * Pre-tokenization: where pieces start.  The paper's pipeline has no such step
 * (section 3.1 cuts fixed-size chunks); the piece rule of the synthetic
 * workloads is used instead: a piece starts at byte 0, at the first byte of
 * every sequence, and at every byte 0x20; nothing else splits, and no piece is
 * empty.  seq_offsets[0 .. n_seqs] are the sequence boundaries (first 0, last
 * n, non-decreasing; NULL with n_seqs == 0 means one sequence).
 * Writes piece_offsets[0 .. n_pieces] (last = n) and, if seq_first_piece is not
 * NULL, seq_first_piece[k] = number of piece starts before byte seq_offsets[k]
 * for k = 0 .. n_seqs (so sequence k owns pieces seq_first_piece[k] ..
 * seq_first_piece[k+1], none if the sequence is empty).  Returns n_pieces.
 */
int64_t oracle_pretokenize(const uint8_t *bytes, int64_t n, const int32_t *seq_offsets,
                           int64_t n_seqs, int32_t *piece_offsets, int32_t *seq_first_piece) {
    int64_t n_pieces = 0;
    for (int64_t i = 0; i < n; ++i) {
        int start = (i == 0) || bytes[i] == 0x20;
        for (int64_t k = 0; !start && seq_offsets && k <= n_seqs; ++k)
            if (seq_offsets[k] == i) start = 1;
        if (start) piece_offsets[n_pieces++] = (int32_t)i;
    }
    piece_offsets[n_pieces] = (int32_t)n;
    if (seq_first_piece && seq_offsets) {
        for (int64_t k = 0; k <= n_seqs; ++k) {
            int64_t before = 0;
            for (int64_t q = 0; q < n_pieces; ++q)
                if (piece_offsets[q] < seq_offsets[k]) ++before;
            seq_first_piece[k] = (int32_t)before;
        }
    }
    return n_pieces;
}

/*
 * Where the bytes of every token start in the decoded text: out_offsets[i] = sum
 * of the byte lengths of ids[0 .. i), out_offsets[n] = the total.  Returns the
 * total, or -1 on an unknown id.
 */
int64_t oracle_token_byte_offsets(const oracle_table *t, const int32_t *ids, int64_t n, int64_t *out_offsets) {
    int64_t total = 0;
    for (int64_t i = 0; i < n; ++i) {
        out_offsets[i] = total;
        int64_t l = expand(t, ids[i], NULL, 0, 0);
        if (l < 0) return -1;
        total += l;
    }
    out_offsets[n] = total;
    return total;
}

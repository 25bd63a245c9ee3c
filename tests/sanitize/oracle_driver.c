/* Runs the CPU oracle (trainer, encoder, decoder, pre-tokenizer) on seeded input; built by
 * tests/test_sanitizers.py with -fsanitize=address,undefined, so any out-of-bounds access, use after free,
 * leak or undefined integer operation on these inputs ends the run with a report and a non-zero status.
 * Test infrastructure: links the oracle only. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct oracle_table oracle_table;
oracle_table *oracle_table_create(const int32_t *merges, const int32_t *ranks, const int32_t *merged_ids, int64_t n);
void oracle_table_free(oracle_table *t);
int oracle_lookup(const oracle_table *t, int32_t a, int32_t b, int32_t *rank, int32_t *merged);
int64_t oracle_encode(const oracle_table *t, const uint8_t *bytes, const int32_t *off, int64_t n_pieces,
                      int32_t *out_ids, int32_t *out_offsets, int n_threads);
int64_t oracle_decode(const oracle_table *t, const int32_t *ids, int64_t n, uint8_t *out, int64_t cap);
int64_t oracle_pretokenize(const uint8_t *bytes, int64_t n, const int32_t *seq_offsets, int64_t n_seqs,
                           int32_t *piece_offsets, int32_t *seq_first_piece);
int64_t oracle_token_byte_offsets(const oracle_table *t, const int32_t *ids, int64_t n, int64_t *out_offsets);
int64_t oracle_train(const uint8_t *bytes, const int32_t *off, int64_t n_pieces, int64_t max_merges, int32_t *out_merges);

static uint64_t state = 0x9E3779B97F4A7C15ull;
static uint32_t draw(uint32_t n) {            /* xorshift64*, good enough to vary the input */
    state ^= state >> 12; state ^= state << 25; state ^= state >> 27;
    return (uint32_t)((state * 0x2545F4914F6CDD1Dull) >> 33) % n;
}

#define CHECK(cond) do { if (!(cond)) { fprintf(stderr, "check failed, line %d: %s\n", __LINE__, #cond); return 1; } } while (0)

int main(void) {
    enum { N = 60000, MERGES = 400 };
    uint8_t *text = (uint8_t *)malloc(N);
    int64_t n = 0;
    while (n < N - 80) {                      /* words, runs of one byte, arbitrary bytes, doubled spaces */
        const uint32_t kind = draw(20);
        text[n++] = ' ';
        if (kind == 0) { const int len = 1 + (int)draw(64); const uint8_t c = (uint8_t)(1 + draw(255)); for (int i = 0; i < len; ++i) text[n++] = c == ' ' ? 'x' : c; }
        else if (kind == 1) { const int len = 1 + (int)draw(40); for (int i = 0; i < len; ++i) { uint8_t c = (uint8_t)draw(256); text[n++] = c == ' ' ? 0 : c; } }
        else if (kind == 2) { /* a space of its own */ }
        else { const int len = 1 + (int)draw(9); for (int i = 0; i < len; ++i) text[n++] = (uint8_t)('a' + draw(6)); }
    }
    const int32_t seq_off[4] = {0, (int32_t)(n / 3), (int32_t)(n / 3), (int32_t)n};   /* with an empty sequence */
    int32_t *piece_off = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n + 2));
    int32_t first[4];
    const int64_t n_pieces = oracle_pretokenize(text, n, seq_off, 3, piece_off, first);
    CHECK(n_pieces > 0 && piece_off[0] == 0 && piece_off[n_pieces] == n && first[3] == n_pieces);

    int32_t *merges = (int32_t *)malloc(sizeof(int32_t) * 2 * MERGES);
    const int64_t n_merges = oracle_train(text, piece_off, n_pieces, MERGES, merges);
    CHECK(n_merges > 100 && n_merges <= MERGES);
    int32_t *ranks = (int32_t *)malloc(sizeof(int32_t) * MERGES);
    for (int i = 0; i < MERGES; ++i) ranks[i] = i;
    oracle_table *t = oracle_table_create(merges, ranks, NULL, n_merges);
    CHECK(t != NULL);
    int32_t rank = -1, merged = -1;
    CHECK(oracle_lookup(t, merges[0], merges[1], &rank, &merged) && rank == 0 && merged == 256);
    CHECK(!oracle_lookup(t, 0x7fffffff, -1, &rank, &merged));

    int32_t *ids = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n + 1));
    int32_t *out_off = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_pieces + 1));
    int32_t *ids4 = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n + 1));
    int32_t *out_off4 = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_pieces + 1));
    const int64_t n_tok = oracle_encode(t, text, piece_off, n_pieces, ids, out_off, 1);
    const int64_t n_tok4 = oracle_encode(t, text, piece_off, n_pieces, ids4, out_off4, 4);
    CHECK(n_tok > 0 && n_tok <= n && n_tok4 == n_tok && out_off[n_pieces] == n_tok);
    CHECK(!memcmp(ids, ids4, sizeof(int32_t) * (size_t)n_tok));
    CHECK(!memcmp(out_off, out_off4, sizeof(int32_t) * (size_t)(n_pieces + 1)));
    CHECK(oracle_encode(t, text, piece_off, 0, ids4, out_off4, 2) == 0);          /* no pieces */

    uint8_t *back = (uint8_t *)malloc((size_t)n + 1);
    CHECK(oracle_decode(t, ids, n_tok, back, n) == n && !memcmp(back, text, (size_t)n));
    CHECK(oracle_decode(t, ids, n_tok, back, 10) == n);                           /* short buffer: size only */
    int64_t *byte_off = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n_tok + 1));
    CHECK(oracle_token_byte_offsets(t, ids, n_tok, byte_off) == n && byte_off[0] == 0);

    free(byte_off); free(back); free(out_off4); free(ids4); free(out_off); free(ids);
    oracle_table_free(t);
    free(ranks); free(merges); free(piece_off); free(text);
    puts("oracle under the sanitizers: ok");
    return 0;
}

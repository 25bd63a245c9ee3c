/*
 * bpe_mi355x — byte-level BPE merge loop on one AMD MI355X (gfx950).
 *
 * C ABI.  Every function returns 0 (BPE_OK) or a negative bpe_status_t unless
 * stated otherwise; bpe_last_error() gives a thread-local message for the last
 * failure on the calling thread.  No function throws.  "host" / "device" says
 * where a pointer must live; device pointers are ordinary HIP allocations (for
 * example the data_ptr() of a torch tensor on the GPU) on the current device,
 * which must be the device a table or vocabulary handle was built on
 * (BPE_ERR_HIP otherwise).
 *
 * What is computed (paper, section 1): for every piece
 * bytes[piece_offsets[p] .. piece_offsets[p+1]) independently, start from one
 * symbol per byte (id = byte value) and repeatedly replace the adjacent pair
 * with the lowest merge-table rank, left-most occurrence first, by its merged
 * id, until no pair of the piece is in the table (tie-break and termination:
 * section 3.4).  The result is identical to that sequential definition; the
 * kernels only reach it in fewer passes.
 */
#ifndef BPE_MI355X_H
#define BPE_MI355X_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    BPE_OK = 0,
    BPE_ERR_NULL = -1,          /* a required pointer is NULL                               */
    BPE_ERR_SIZE = -2,          /* negative size, n_bytes >= 2^31, too many merges ...      */
    BPE_ERR_ID_RANGE = -3,      /* a token id is negative or too large, or a merged id < 256 */
    BPE_ERR_DUP_PAIR = -4,      /* the same (left, right) pair appears twice                */
    BPE_ERR_DUP_RANK = -5,      /* the same rank appears twice, or a rank is out of range   */
    BPE_ERR_DUP_MERGED = -6,    /* two merges produce the same merged id                    */
    BPE_ERR_ORDER = -7,         /* a merge uses an id that is only made by a later-or-equal rank */
    BPE_ERR_WORKSPACE = -8,     /* workspace missing, misaligned or too small               */
    BPE_ERR_HIP = -9,           /* a HIP runtime call failed (no device, out of memory ...) */
    BPE_ERR_OPTION = -10,       /* an option value is out of range                          */
    BPE_ERR_INPUT = -11         /* device-side check: piece_offsets invalid (see bpe_encode_status) */
} bpe_status_t;

const char *bpe_last_error(void);

/* ------------------------------------------------------------------------- */
/* Merge table (paper, section 3.3).                                          */
/*
 * A pair is keyed by the 64-bit word (left << 32) | right and maps to the
 * 64-bit word (merged_id << 32) | rank_word.  The low 26 bits of rank_word are
 * the rank order: the position of the rule when all rules are sorted by rank (0
 * merges first; equal to the rank itself when the ranks are 0 .. n_merges-1);
 * bit 30 / bit 31 say whether merged_id occurs as the left / right part of any
 * rule (a pair that cannot exist needs no lookup).  The table is an
 * open-addressing array of slots, capacity = the power of two >= 2.5 * n_merges
 * (load factor <= 40 %) and never below 131072 slots.  Placement is two-choice:
 * a key is stored at slot h1(key) of the lower half or at slot half + h2(key) of
 * the upper half, so a lookup reads exactly two slots and never loops.  With the
 * 24-bit multipliers K of build attempt t (see hash_attempt; every Ka is odd),
 *   m(a, b) = (((a + b * Kb) mod 2^24) * Ka) mod 2^24,
 *   h(a, b) = m(a, b) >> (24 - log2(capacity / 2)).
 * For a fixed right id b, m is a bijection of the left id a, so a slot's index, the
 * low 24 - log2(capacity / 2) bits of m and b name the key: the image that
 * bpe_table_image_build returns holds 16-byte slots {key, value} (empty key = all
 * ones), the device copy 8-byte slots {low bits of m | b << 8, rank_word}.
 * The table is built once and reused by every encode call.
 */
typedef struct bpe_table bpe_table;

typedef struct {
    int64_t n_merges;
    int64_t capacity;       /* slots */
    int64_t device_bytes;   /* 8-byte slots, the 65536-entry direct table for byte pairs (4 bytes each), two
                             * rank-order arrays, 8 bytes per token id up to max_id */
    int32_t hash_attempt;   /* which multiplier set placed all keys (0 = first) */
    int32_t max_id;         /* largest token id the table can produce or consume */
} bpe_table_info_t;

/* Slots bpe_table_build / bpe_table_image_build use for n_merges rules (pure function). */
int64_t bpe_table_capacity(int64_t n_merges);

/*
 * Validate the rules and build the slot image in caller memory (host only, no
 * GPU needed).  merges: host int32 [n_merges][2] = (left id, right id);
 * ranks: host int32 [n_merges], unique, >= 0, lower merges first, or NULL for
 * rank = row index; merged_ids: host int32 [n_merges], unique, in [256, 2^24),
 * or NULL for merged id = 256 + rank.  Ids 0..255 are the byte symbols;
 * n_merges < 2^22.
 * Required property: both parts of a rule are bytes or merged ids of rules with
 * a strictly lower rank (true of any table learned by BPE training); it is what
 * makes merging several pairs per pass exact.  slots: host uint64
 * [2 * capacity_slots], capacity_slots == bpe_table_capacity(n_merges); slot i
 * is {slots[2i] = key, slots[2i+1] = value}.  info may be NULL.
 */
int bpe_table_image_build(const int32_t *merges, const int32_t *ranks, const int32_t *merged_ids,
                          int64_t n_merges, uint64_t *slots, int64_t capacity_slots,
                          bpe_table_info_t *info);

/* Same validation, then one device allocation and one host-to-device copy.
 * The handle owns its device memory; free it with bpe_table_free. */
int bpe_table_build(const int32_t *merges, const int32_t *ranks, const int32_t *merged_ids,
                    int64_t n_merges, bpe_table **out_table);
int bpe_table_free(bpe_table *table);
int bpe_table_info(const bpe_table *table, bpe_table_info_t *info);

/*
 * Pair-rank lookup on the device (the first step of every merge pass, section
 * 3.4 "pair evaluation").  pairs: device int32 [n][2]; out_rank / out_merged:
 * device int32 [n]; a pair that is not in the table gets rank -1, merged -1.
 * Enqueues on `stream` (a hipStream_t, NULL = default stream); does not sync.
 */
int bpe_table_lookup(const bpe_table *table, const int32_t *pairs, int64_t n,
                     int32_t *out_rank, int32_t *out_merged, void *stream);

/* ------------------------------------------------------------------------- */
/* Encoding (paper, sections 3.4-3.5: pair evaluation, argmin, compaction;    */
/* section 3.1 step 4 "assembly", done on the device here).                   */

typedef struct {
    /* What a pass merges in a piece of more than 16 bytes (wavefront and workgroup
     * paths): 1 = the single best pair (sections 3.4/3.5); 2 = every occurrence of the
     * best-ranked pair, left to right without overlap; 3 = that, and every other pair
     * that the greedy order is bound to merge anyway (pieces of more than 64 bytes;
     * the exact form of the "local minima" of the paper's introduction: a pair none
     * of whose two symbols can be taken by a lower-ranked rule before the pair's own
     * turn); 0 (default) = 3, except that a piece that is mostly runs of one byte
     * takes the passes of level 2, which hold twice as many symbols in LDS.  All give
     * the sequential result exactly.  Pieces of at most 16 bytes always take one
     * merge at a time. */
    int32_t selection_level;
    /* Pieces per wavefront, 1..64 (a workgroup of four wavefronts takes four times as
     * many); -1 = one piece per workgroup; 0 = choose from n_bytes / n_pieces
     * (bpe_encode_raw: the kernels choose, once the pre-tokenizer has counted the pieces). */
    int32_t pieces_per_wave;
    /* Pieces of at most this many bytes take the lane-per-piece path; 0 = 16,
     * -1 = none.  At most 16. */
    int32_t tiny_max_len;
    /* Longer pieces of at most this many bytes take the lane-per-symbol
     * wavefront path (one piece per wavefront round); 0 = 64, -1 = none.  At most 64.
     * With the default column_max_len no piece is left for this path. */
    int32_t wave_max_len;
    /* Longer pieces of at most this many bytes are merged by one wavefront that
     * double-buffers the piece in its own LDS region; 0 = 1024, -1 = none.  At
     * most 1024. */
    int32_t wave_lds_max_len;
    /* The workgroup path (all longer pieces) keeps a piece in LDS when it is at
     * most this long, else it ping-pongs in the workspace; 0 = the LDS budget
     * (4104).  1..4104.  The passes of level 3 keep four words per symbol instead of
     * two: half this many symbols (at least 320, at most 2052; 512 for a wavefront)
     * stay in LDS, a longer piece passes through LDS in windows of that size until
     * it has shrunk to it. */
    int32_t lds_max_len;
    /* 1: one kernel does the merges and the ordered assembly of the output;
     * -1: merge kernel, emit kernel and, on deep grids, a scan kernel between them;
     * 0 (default): one kernel for grids of up to 256 workgroups whose pieces average
     * at most 64 bytes, several otherwise.  In the single kernel a workgroup waits for
     * the ones before it, for at most about two seconds; a wait that runs out is
     * reported by bpe_encode_status as BPE_ERR_HIP, and the output of such a call is
     * undefined.  While every workgroup of the grid is resident at once (up to 1024)
     * no wait can last; beyond that, and with long pieces, the waits only end because
     * the hardware dispatches workgroups in index order, which HIP does not promise:
     * 1 is therefore refused (BPE_ERR_OPTION) for grids of more than 1024 workgroups
     * or pieces that average more than 64 bytes; 2 forces the single kernel anyway
     * (for tests and measurements). */
    int32_t fused;
    /* Input bytes per workgroup of the pre-tokenizer (bpe_pretokenize,
     * bpe_encode_raw), in KiB: 4, 16, 64 or 128; -64 or -128 for tiles of that
     * size whose stores are made contiguous in LDS first (pays on inputs of tens
     * of MiB and more); 0 = choose from n_bytes. */
    int32_t pretokenize_tile_kib;
    /* Comparison only: run the paper's own kernel on every piece instead, one
     * workgroup per piece (the paper's "chunk"), exactly one merge per pass:
     * 1 = its baseline kernel (section 3.4: pieces of up to 256 symbols compact by a
     * prefix sum over "removed" flags, longer ones by the shift), 2 = its optimized
     * kernel (section 3.5: always the shift).  Same tokens as the default (0).
     * Not available in bpe_encode_raw; fused is ignored. */
    int32_t paper_kernel;
    /* Longer pieces than tiny_max_len of at most this many bytes take the lane-per-piece
     * path as well, with columns of 64 symbols (16 pieces per wavefront and round);
     * 0 = 64, -1 = none (the lane-per-symbol path then takes them).  At most 64. */
    int32_t column_max_len;
    /* 1: piece de-duplication (the paper's section 6 names it as future work): every
     * distinct piece of at most 16 bytes is merged once and its tokens are handed to all
     * its occurrences (kernels: every piece writes its index into a hash table slot, then
     * compares bytes with the piece it finds there; the distinct pieces are compacted and
     * merged, their records handed out; emit).  Same tokens as without.
     * bpe_encode only, pieces_per_wave 64 (the default for word-sized pieces), not with
     * fused > 0 or paper_kernel; the workspace must hold bpe_dedup_workspace_bytes.
     * 0 (default): off. */
    int32_t dedup;
    /* bpe_encode on word-sized pieces (pieces_per_wave 64; bpe_encode_raw: only if the caller
     * gives that value, it is not the kernels' to choose then), several kernels: the pieces of more
     * than tiny_max_len bytes are not merged by the workgroup of their tile but by workgroups
     * of their own at the head of the merge kernel's grid, each for this many consecutive
     * tiles (1..256); 0 (default) = 4, from grids of 1025 tiles on; -1 = never (every workgroup
     * merges all pieces of its tile). */
    int32_t long_groups;
} bpe_encode_options;

/* Device bytes bpe_encode needs for inputs of up to n_bytes bytes and n_pieces
 * pieces (pure function; negative bpe_status_t on bad sizes). */
int64_t bpe_workspace_bytes(int64_t n_bytes, int64_t n_pieces);

/* Device bytes bpe_encode needs with the option dedup = 1 (pure function). */
int64_t bpe_dedup_workspace_bytes(int64_t n_bytes, int64_t n_pieces);

/*
 * Encode all pieces.  Only enqueues kernels on `stream`: no allocation, no
 * synchronisation, no host-device copy.  Results are valid once the stream has
 * been synchronised.
 *   bytes          device uint8 [n_bytes], all sequences concatenated
 *   piece_offsets  device int32 [n_pieces + 1], non-decreasing, first 0, last n_bytes;
 *                  a sequence boundary must be a piece boundary
 *   out_ids        device int32, capacity >= n_bytes (tokens never outnumber bytes);
 *                  all tokens densely, in piece order
 *   out_offsets    device int32 [n_pieces + 1]; tokens of piece p are
 *                  out_ids[out_offsets[p] .. out_offsets[p+1]); [n_pieces] = total
 *   workspace      device, 256-byte aligned, >= bpe_workspace_bytes(n_bytes, n_pieces);
 *                  contents need not be initialised; calls that share a workspace
 *                  must be ordered on one stream
 *   opts           NULL for defaults
 * n_bytes < 2^31.  An empty piece yields no token; n_pieces == 0 writes only
 * out_offsets[0] = 0.  Offsets that are out of range or decreasing are detected
 * on the device: the affected pieces yield no tokens, nothing is read or written
 * out of bounds, and bpe_encode_status reports BPE_ERR_INPUT.
 */
int bpe_encode(const bpe_table *table, const uint8_t *bytes, const int32_t *piece_offsets,
               int64_t n_bytes, int64_t n_pieces, int32_t *out_ids, int32_t *out_offsets,
               void *workspace, int64_t workspace_bytes, const bpe_encode_options *opts,
               void *stream);

/*
 * bpe_encode without the workspace arguments, for callers that cannot allocate
 * device memory and have no workspace to bring: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  The kernels use a
 * built-in device array of 16 MiB instead (each GPU the library runs on holds its
 * own copy until the process ends); its address is looked up on the first call on
 * a device (no allocation; make that first call outside a capture).  Inputs whose
 * bpe_workspace_bytes(n_bytes, n_pieces) exceeds 16 MiB (16,777,216 bytes: about
 * 1.4 MB of word-like text) are refused with BPE_ERR_SIZE.  The call allocates
 * nothing, frees nothing, does not synchronise and only enqueues kernels.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one
 * GPU (two streams, two threads) race and give undefined results; order them on
 * one stream.  The array keeps the last call's contents and needs no clearing.
 * The device-side verdict of the last such call on the current device:
 * bpe_encode_status(NULL, stream).  Other arguments and results as in bpe_encode.
 */
int bpe_encode_static(const bpe_table *table, const uint8_t *bytes, const int32_t *piece_offsets,
                      int64_t n_bytes, int64_t n_pieces, int32_t *out_ids, int32_t *out_offsets,
                      const bpe_encode_options *opts, void *stream);

/*
 * Measurement aid with the arguments of bpe_encode: records a HIP event on
 * `stream` before the first kernel and after each kernel, waits for the last
 * one and writes the three intervals in milliseconds to host float kernel_ms[3]
 * = {merge (the whole path when fused), tile scan, emit}.  It creates and
 * destroys events and synchronises, so it is not for the serving path; the
 * paper's binding likewise returns an event-timed kernel time (section 3.7).
 */
int bpe_encode_timed(const bpe_table *table, const uint8_t *bytes, const int32_t *piece_offsets,
                     int64_t n_bytes, int64_t n_pieces, int32_t *out_ids, int32_t *out_offsets,
                     void *workspace, int64_t workspace_bytes, const bpe_encode_options *opts,
                     void *stream, float *kernel_ms);

/*
 * What bpe_encode / bpe_encode_raw launch for inputs of these sizes and these
 * options, without launching anything (pure functions of their arguments; no GPU
 * needed): the kernels in launch order with their grids, so that a measurement can
 * name the kernels it timed without re-deriving the library's choices.  `interval`
 * is the index of the kernel_ms[] entry of bpe_encode_timed / bpe_encode_raw_timed
 * (called with the same sizes and options) that the launch falls into.
 * bpe_encode_raw_plan: has_seq_offsets != 0 means the call passes seq_offsets,
 * wants_piece_arrays != 0 that it passes any of piece_offsets, out_offsets, n_pieces.
 * Errors as in the calls themselves (BPE_ERR_SIZE, BPE_ERR_OPTION).
 */
#define BPE_PLAN_MAX_LAUNCHES 8
typedef struct {
    int32_t n_launches;
    int32_t single_kernel;      /* 1: merges and assembly of the output in one launch */
    int32_t selection_level;    /* 1, 2 or 3 (the default 0 resolved) */
    int32_t pieces_per_wave;    /* resolved; bpe_encode_raw may still change it on the device */
    int32_t waves_per_tile;     /* 4, or 1 with one piece per workgroup */
    int32_t reserved;
    int64_t n_tiles;            /* bpe_encode_raw: the bound that max_pieces allows for */
    struct {
        char kernel[32];
        int64_t grid;           /* workgroups */
        int32_t block;          /* threads per workgroup */
        int32_t interval;
    } launch[BPE_PLAN_MAX_LAUNCHES];
} bpe_encode_plan_t;

int bpe_encode_plan(int64_t n_bytes, int64_t n_pieces, const bpe_encode_options *opts,
                    bpe_encode_plan_t *plan);
int bpe_encode_raw_plan(int64_t n_bytes, int64_t max_pieces, int64_t n_seqs, int has_seq_offsets,
                        int wants_piece_arrays, const bpe_encode_options *opts, bpe_encode_plan_t *plan);

/* Synchronise `stream` and return the device-side verdict of the last
 * bpe_encode, bpe_pretokenize, bpe_encode_raw or bpe_decode that used
 * `workspace` (NULL: of the last bpe_encode_static on the current device): BPE_OK, BPE_ERR_INPUT (invalid piece_offsets, seq_offsets or token
 * ids), BPE_ERR_SIZE (more pieces than max_pieces, more bytes than out_capacity)
 * or BPE_ERR_HIP.  A condition is reported once: the call clears it, so that
 * replays of a graph that recorded the call are judged afresh (the verdict then
 * covers all replays since the last bpe_encode_status).  A workspace in which no
 * call has finished yet (fresh or zero-filled memory) gives BPE_OK and is not
 * written to.  The outputs of a call are defined only if its verdict is BPE_OK. */
int bpe_encode_status(void *workspace, void *stream);

/* The same verdict from a host copy of the first 8 int32 words of a workspace, for a
 * caller that brings them back with its own asynchronous copy, behind the call's
 * kernels on their stream, and so needs one synchronisation for results and verdict
 * (host only: no GPU call, nothing is cleared; a verdict refers to the last call that
 * finished in that workspace before the copy). */
int bpe_status_from_words(const int32_t *status_words);

/* ------------------------------------------------------------------------- */
/* Pre-tokenization on the device: where pieces start.  The paper's pipeline  */
/* (section 3.1) has no such step: it cuts the input into fixed-size chunks,  */
/* which forbids merges across a cut.  Here the merge loop runs per piece,    */
/* and a piece starts at byte 0, at the first byte of every sequence and at   */
/* every space byte (0x20); nothing else splits, no piece is empty.           */

/* Device bytes bpe_pretokenize needs (pure function). */
int64_t bpe_pretokenize_workspace_bytes(int64_t n_bytes);

/*
 * One pass over the bytes, one kernel; only enqueues on `stream`.
 *   bytes            device uint8 [n_bytes], any alignment
 *   seq_offsets      device int32 [n_seqs + 1], non-decreasing, first 0, last n_bytes;
 *                    NULL = one sequence (n_seqs is then ignored)
 *   piece_offsets    device int32 [max_pieces + 1], out: start of every piece, then n_bytes
 *   max_pieces       capacity; n_bytes is always enough
 *   n_pieces         device int32 [1], out
 *   seq_first_piece  device int32 [n_seqs + 1] ([2] without seq_offsets) or NULL, out:
 *                    number of pieces that start before byte seq_offsets[k]; sequence
 *                    k owns pieces seq_first_piece[k] .. seq_first_piece[k+1]
 *   workspace        device, 256-byte aligned, >= bpe_pretokenize_workspace_bytes(n_bytes)
 *   opts             NULL for defaults; only pretokenize_tile_kib is read
 * If the input has more than max_pieces pieces, the first max_pieces are written,
 * *n_pieces = max_pieces and bpe_encode_status reports BPE_ERR_SIZE.  Invalid
 * seq_offsets are detected on the device (BPE_ERR_INPUT); nothing is read or
 * written out of bounds.
 */
int bpe_pretokenize(const uint8_t *bytes, int64_t n_bytes, const int32_t *seq_offsets, int64_t n_seqs,
                    int32_t *piece_offsets, int64_t max_pieces, int32_t *n_pieces,
                    int32_t *seq_first_piece, void *workspace, int64_t workspace_bytes,
                    const bpe_encode_options *opts, void *stream);

/* Device bytes bpe_encode_raw needs; max_pieces == 0 means n_bytes. */
int64_t bpe_encode_raw_workspace_bytes(int64_t n_bytes, int64_t max_pieces, int64_t n_seqs);

/*
 * bpe_pretokenize followed by bpe_encode without a host pass in between: the
 * piece count stays on the device and the encode kernels are launched for
 * max_pieces pieces (workgroups past the last piece return at once), so a tight
 * max_pieces saves launch work.  Only enqueues on `stream`.
 *   seq_token_offsets  device int32 [n_seqs + 1] ([2] without seq_offsets), out:
 *                      sequence k owns out_ids[seq_token_offsets[k] .. seq_token_offsets[k+1])
 *   piece_offsets, out_offsets   device int32 [max_pieces + 1] as in bpe_encode, or
 *                      NULL to keep them in the workspace
 *   n_pieces           device int32 [1] or NULL
 * Other arguments as in bpe_encode and bpe_pretokenize; max_pieces == 0 means
 * n_bytes.  The single-kernel path (fused > 0) is not used here.
 * A call that asks for tokens only (piece_offsets, out_offsets and n_pieces all NULL),
 * with the default capacity (max_pieces 0 or >= n_bytes) and pieces_per_wave left 0, on
 * at most 1,310,720 bytes (1024 workgroups) launches no pre-tokenizer: the workgroups
 * of the merge kernel find the pieces in their own 1280 bytes (kernels
 * merge_bytes_kernel, emit_bytes_kernel); the option fused = -1 takes the
 * pre-tokenizer path all the same.  Same tokens either way.
 */
int bpe_encode_raw(const bpe_table *table, const uint8_t *bytes, int64_t n_bytes,
                   const int32_t *seq_offsets, int64_t n_seqs, int64_t max_pieces, int32_t *out_ids,
                   int32_t *seq_token_offsets, int32_t *piece_offsets, int32_t *out_offsets,
                   int32_t *n_pieces, void *workspace, int64_t workspace_bytes,
                   const bpe_encode_options *opts, void *stream);

/* Measurement aid like bpe_encode_timed: host float kernel_ms[5] = {pre-tokenizer,
 * merge, tile scan, emit, sequence offsets}.  The tile scan is only launched when
 * max_pieces allows for more than 8192 tiles, and the sequence offsets
 * have a kernel of their own only with more than 1023 sequences or when max_pieces
 * allows for 4096 tiles or more (else the emit kernel writes them); an interval
 * without a launch holds the time between two event records. */
int bpe_encode_raw_timed(const bpe_table *table, const uint8_t *bytes, int64_t n_bytes,
                         const int32_t *seq_offsets, int64_t n_seqs, int64_t max_pieces, int32_t *out_ids,
                         int32_t *seq_token_offsets, int32_t *piece_offsets, int32_t *out_offsets,
                         int32_t *n_pieces, void *workspace, int64_t workspace_bytes,
                         const bpe_encode_options *opts, void *stream, float *kernel_ms);

/* ------------------------------------------------------------------------- */
/* Vocabulary: what every token id stands for.  The paper takes GPT-2's       */
/* vocabulary files as given (section 3.2) and turns ids back into text on    */
/* the host; here the byte expansion of every id follows from the rules (a    */
/* merged id expands to the expansions of its two parts, section 3.3) and     */
/* lives on the device.                                                       */
typedef struct bpe_vocab bpe_vocab;

typedef struct {
    int64_t n_ids;            /* largest id of the rules + 1 (ids 0..255 are the bytes) */
    int64_t n_output_ids;     /* largest output id + 1, 0 without a renumbering */
    int64_t pool_bytes;       /* all expansions, each padded to 4 bytes */
    int64_t device_bytes;
    int32_t max_token_bytes;  /* longest expansion */
    int32_t has_output_ids;
} bpe_vocab_info_t;

/*
 * merges, ranks, merged_ids, n_merges: as in bpe_table_build (same checks).
 * output_ids: host int32 [n_output_ids] or NULL.  With it, n_output_ids must be
 * the largest id + 1, and output_ids[id] is the id under which the caller's
 * vocabulary file lists token `id` (for every byte and every merged id; entries
 * of unused ids are ignored): unique, in [0, 2^24).  GPT-2's files, for example,
 * number the 256 byte symbols differently from their byte values.
 * Expansions longer than 2^20 bytes, or 2^30 bytes in total, are refused
 * (BPE_ERR_SIZE).  One device allocation, owned by the handle.
 */
int bpe_vocab_build(const int32_t *merges, const int32_t *ranks, const int32_t *merged_ids,
                    int64_t n_merges, const int32_t *output_ids, int64_t n_output_ids,
                    bpe_vocab **out_vocab);
int bpe_vocab_free(bpe_vocab *vocab);
int bpe_vocab_info(const bpe_vocab *vocab, bpe_vocab_info_t *info);

/*
 * Renumber ids on the device: ids_out[i] = output id of ids_in[i] (to_output_ids
 * != 0) or the id whose output id is ids_in[i] (to_output_ids == 0); -1 for a
 * value that is not in the vocabulary.  ids_in, ids_out: device int32 [n], may be
 * the same buffer.  n_device: device int32 [1] or NULL; with it only the first
 * min(n, *n_device) entries are touched, so that a count that is still on the
 * device (out_offsets[n_pieces] of bpe_encode) needs no host round trip.
 * Only enqueues on `stream`.  BPE_ERR_OPTION if the vocabulary has no output ids.
 */
int bpe_map_ids(const bpe_vocab *vocab, const int32_t *ids_in, int32_t *ids_out, int64_t n,
                const int32_t *n_device, int to_output_ids, void *stream);

/* Device bytes bpe_decode needs for up to n_tokens tokens (pure function). */
int64_t bpe_decode_workspace_bytes(int64_t n_tokens);

/*
 * Token ids back to bytes: out_bytes = the expansions of ids[0 .. n) one after
 * the other.  One kernel; only enqueues on `stream`.
 *   ids                 device int32 [n_tokens]
 *   n_tokens_device     device int32 [1] or NULL: decode min(n_tokens, *n_tokens_device) tokens
 *   ids_are_output_ids  != 0: ids are the vocabulary's output ids
 *   out_bytes           device uint8 [out_capacity], any alignment
 *   token_byte_offsets  device int32 [n_tokens + 1] or NULL, out: where every token's
 *                       bytes start; [n] = their total
 *   n_bytes             device int32 [1] or NULL, out: bytes written
 *   workspace           device, 256-byte aligned, >= bpe_decode_workspace_bytes(n_tokens)
 * An id that is not in the vocabulary contributes no byte and makes
 * bpe_encode_status report BPE_ERR_INPUT; bytes beyond out_capacity are not
 * written and reported as BPE_ERR_SIZE.  out_capacity < 2^31.
 */
int bpe_decode(const bpe_vocab *vocab, const int32_t *ids, int64_t n_tokens,
               const int32_t *n_tokens_device, int ids_are_output_ids, uint8_t *out_bytes,
               int64_t out_capacity, int32_t *token_byte_offsets, int32_t *n_bytes, void *workspace,
               int64_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------------- */
/* Preallocated workspace pool (the paper's profiling, section 5.3, finds     */
/* allocation to be 70-80 % of its API time and names pooling as the next     */
/* step).  One allocation at creation, none afterwards.  The buffer is large   */
/* enough for every entry point that takes a workspace: bpe_encode and        */
/* bpe_encode_raw on up to max_bytes bytes, max_pieces pieces and max_pieces  */
/* sequences, bpe_pretokenize on max_bytes bytes, bpe_decode of max_bytes     */
/* tokens.  Calls that share it must be ordered on one stream.                */
typedef struct bpe_pool bpe_pool;

int bpe_pool_create(int64_t max_bytes, int64_t max_pieces, bpe_pool **out_pool);
int bpe_pool_destroy(bpe_pool *pool);
/* The pool's buffer, to pass to bpe_encode as workspace / workspace_bytes. */
int bpe_pool_workspace(const bpe_pool *pool, void **workspace, int64_t *workspace_bytes);

#ifdef __cplusplus
}
#endif
#endif /* BPE_MI355X_H */

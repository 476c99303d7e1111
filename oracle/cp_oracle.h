/*
 * CPU oracle for the token-granular KV sharing path of CachePrune.
 *
 * TEST INFRASTRUCTURE ONLY.  This is a plain, sequential, deliberately slow
 * reference that the tests, the smoke check and the benchmark's CPU-baseline
 * leg call to decide whether the GPU library is right.  It shares no source,
 * header, table or helper with the GPU library and must never be used as a
 * product code path or as a fallback.
 *
 * All pointers are HOST pointers.  Nothing here is thread-safe.
 *
 * What each function follows (paper = CachePrune):
 *   - Sensitive tokens (mask = 1) are separators that cut a prompt into
 *     segments; only tokens with mask = 0 may be shared (Sec. 3.3 definition
 *     of selective sharing, Sec. 4.2.1 first paragraph).
 *   - Segments are identified by a polynomial rolling hash (Sec. 4.2.2,
 *     "Choice of rolling hash algorithm").  This build takes the hash modulo
 *     2^64 with a fixed base and hashes every run from its first token
 *     (a "chain" hash), one key per token.
 *   - The pool keeps one copy of a duplicated segment (Sec. 4.3.5 "Lifecycle
 *     management"): insertion is insert-if-absent, first occurrence wins.
 *   - Matched segments are linked into the request, unmatched positions are
 *     left for the engine (Sec. 4.1 "KV Retriever", Sec. 4.3.1 "Operational
 *     details").  Here "linking" is a copy of the token's K and V rows of
 *     every layer into the request's buffers.
 *   - Key re-rotation by a position delta (RoPE) is not in the paper; it is
 *     the textbook rotary embedding, evaluated in double precision.
 */
#ifndef CP_ORACLE_H
#define CP_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CPO_HASH_NONE 0xFFFFFFFFFFFFFFFFull /* hash of a sensitive token      */
#define CPO_SLOT_NONE 0xFFFFFFFFu           /* "no pool slot"                 */

#define CPO_FLAG_SPANS_OVERFLOW 1u /* more spans than max_spans; extra dropped */
#define CPO_FLAG_POOL_FULL 2u      /* free list exhausted; later tokens dropped */
#define CPO_FLAG_TABLE_FULL 4u     /* a bounded table cannot take the batch's new keys: none stored */

/* Byte address of the row of (token or slot t, layer l, kv in {0 = K, 1 = V}):
 *   base + t * tok_stride + l * layer_stride + kv * kv_stride
 * A row is n_kv_heads * head_dim bf16 values, contiguous. */
typedef struct {
  uint32_t n_layers, n_kv_heads, head_dim;
  uint64_t tok_stride, layer_stride, kv_stride; /* bytes */
} cpo_layout;

/* Rotary embedding parameters.  style 0: element j pairs with j + head_dim/2;
 * style 1: element 2j pairs with 2j + 1. */
typedef struct {
  double theta;
  uint32_t style;
} cpo_rope;

/* The pool index: an associative container key -> slot.  Opaque. */
typedef struct cpo_index cpo_index;
cpo_index *cpo_index_new(void);
void cpo_index_free(cpo_index *);
uint64_t cpo_index_size(const cpo_index *);
/* The index as a table of `capacity` entries (0 = unbounded, the default): start a fresh table that
 * holds the keys with a slot.  A key takes an entry when an insert first sees it and keeps it also
 * while it has no slot (dropped for lack of pool slots, evicted) until the next rebuild.  An insert
 * whose new keys do not all fit sets CPO_FLAG_TABLE_FULL and stores nothing. */
void cpo_index_rebuild(cpo_index *, uint64_t capacity);
uint64_t cpo_index_entries(const cpo_index *);

/* Chain hash of every token.  R requests are packed back to back, request r
 * holds tokens off[r] .. off[r+1]-1.  For a sensitive token hash_out = NONE
 * and the chain restarts; the chain also restarts at every request start.
 * For the k-th token (k = 0, 1, ..) of a run t_0 .. t_k:
 *   hash = sum_{m=0..k} (t_m + 1) * base^(k-m)   (mod 2^64),
 * and a result equal to NONE is replaced by NONE - 1. */
void cpo_hash_segments(const uint32_t *tok, const uint8_t *mask, const uint32_t *off, uint32_t R,
                       uint64_t base, uint64_t *hash_out);

/* slot_out[i] = slot stored under hash[i], or SLOT_NONE (also for hash NONE). */
void cpo_probe(const cpo_index *, const uint64_t *hash, uint32_t N, uint32_t *slot_out);

/* Run-length pass.  A span is a maximal run of consecutive positions of one
 * request whose slots are valid and consecutive and (if slot_pos is given)
 * share one position delta = (position inside the request) - slot_pos[slot].
 * Spans come out in (request, position) order; dst is the packed token index.
 * Returns the number of spans found; only the first max_spans are stored and
 * SPANS_OVERFLOW is or-ed into *flags if there were more.  slot_pos and
 * span_delta may be NULL (delta = 0). */
uint32_t cpo_build_spans(const uint32_t *slot, const uint32_t *off, uint32_t R,
                         const int32_t *slot_pos, uint32_t max_spans, uint32_t *span_src,
                         uint32_t *span_dst, uint32_t *span_len, int32_t *span_delta,
                         uint32_t *flags);

/* For every span, k < len, layer, K and V: copy the row of pool slot src+k to
 * the row of request token dst+k.  If span_delta and rope are non-NULL, K rows
 * of spans with delta != 0 are rotated by delta positions (double precision,
 * one rounding to bf16, round-to-nearest-even); V rows and delta = 0 are byte
 * copies.  Rows not covered by a span are not touched. */
void cpo_gather_kv(const void *pool, cpo_layout pool_l, void *dst, cpo_layout dst_l,
                   const uint32_t *span_src, const uint32_t *span_dst, const uint32_t *span_len,
                   const int32_t *span_delta, uint32_t n_spans, const cpo_rope *rope);

/* Insert-if-absent, in packed order.  A token with a valid hash whose key is
 * absent takes the next slot of free_slots, records slot_pos[slot] = position
 * inside its request, and has all its rows copied from src to the pool.  When
 * the free list is used up POOL_FULL is flagged and the token is dropped
 * (slot_out = NONE).  slot_out[i] = slot now holding the key, NONE for
 * sensitive tokens.  tok / slot_tok (both nullable) record which token id was
 * stored in each slot, for audits.  Returns the number of newly stored tokens. */
uint32_t cpo_insert_kv(cpo_index *, const uint64_t *hash, const uint32_t *off, uint32_t R,
                       const uint32_t *free_slots, uint32_t n_free, const void *src,
                       cpo_layout src_l, void *pool, cpo_layout pool_l, int32_t *slot_pos,
                       uint32_t *slot_out, uint32_t *flags, const uint32_t *tok,
                       uint32_t *slot_tok);

/* ---- One copy of a text that is stored already (Sec. 4.3.5 "Lifecycle management": a segment that another
 * stored segment contains is kept once) ----
 * Before a batch is stored, a lookup says which of its tokens the pool already has: slot[k][i] is what key
 * stream k (run-start keys, then the candidate streams) found for token i and seg_off[k][i] the token's offset
 * in that stream's segment.  A token that some stream finds is not stored again.  Every other token is stored
 * as the continuation of the text that the latest found token before it (in its run) belongs to: behind a
 * token found at offset o of a stored text, the next tokens extend that stored text; a run in which nothing was
 * found yet starts a text of its own, as in cpo_insert_kv.
 *   ins_off_out[i]  = offset of token i in the text it belongs to (0xFFFFFFFF for sensitive tokens),
 *   ins_hash_out[i] = chain hash of that text from its first token through token i (the table key),
 *   found_out[i]    = slot of the first stream that found token i, else CPO_SLOT_NONE.
 * cpo_insert_kv_dedup is cpo_insert_kv with these keys, skipping the found tokens (slot_out = found).
 * Texts stored within one batch do not see each other: only what earlier batches stored is found. */
void cpo_insert_keys(const uint64_t *hash, const uint32_t *run_off, const uint32_t *const *seg_off,
                     const uint32_t *const *slot, uint32_t n_streams, uint32_t N, uint64_t base,
                     uint64_t *ins_hash_out, uint32_t *ins_off_out, uint32_t *found_out);
uint32_t cpo_insert_kv_dedup(cpo_index *, const uint64_t *ins_hash, const uint32_t *found, const uint32_t *off,
                             uint32_t R, const uint32_t *free_slots, uint32_t n_free, const void *src,
                             cpo_layout src_l, void *pool, cpo_layout pool_l, int32_t *slot_pos,
                             uint32_t *slot_out, uint32_t *flags, const uint32_t *tok, uint32_t *slot_tok);

/* ---- Floating anchors (Sec. 4.2.2, Step 1 "prefix filtering" and Step 2's O(1) substring hash) ----
 * The pool also keeps, for every stored run of at least W tokens, the rolling hash of its first W
 * tokens.  A lookup slides a W-token window over each run of the request; where the window's hash is
 * one of the stored prefix hashes, a stored run may start there ("anchor"), and the tokens from
 * there on get a second key: the hash of the request's tokens from the anchor through the token,
 * computed in O(1) from the run's chain hashes and a power of the base.  Step 1 yields a set of
 * candidates and Step 2 checks each of them over the text stored behind it; a request token can lie in
 * the text of several candidates.  Every token that some candidate's text covers is served: the
 * candidates that serve are chosen like the intervals of a greedy cover and handed alternately to two
 * key streams, so that the texts inside one stream do not overlap.  A token is served under its
 * run-start key if that hits, else under the first stream's key, else under the second's. */
typedef struct cpo_anchor_set cpo_anchor_set; /* prefix hash -> slot of the run's W-th token. Opaque. */
cpo_anchor_set *cpo_anchor_set_new(void);
void cpo_anchor_set_free(cpo_anchor_set *);
uint64_t cpo_anchor_set_size(const cpo_anchor_set *);

/* run_off_out[i] = number of non-sensitive tokens between the start of token i's run and i
 * (0 for the first token of a run), 0xFFFFFFFF for sensitive tokens. */
void cpo_run_offsets(const uint8_t *mask, const uint32_t *off, uint32_t R, uint32_t *run_off_out);

/* Store the prefix hash of every run whose first W tokens are in the pool: the chain hash of its W-th
 * token, for every such token that has a slot (slot[i], as an insert reported it, is not NONE).  The
 * prefix hash lives as long as that slot does: cpo_evict drops it with the slot. */
void cpo_insert_anchors(cpo_anchor_set *, const uint64_t *hash, const uint32_t *run_off,
                        const uint32_t *slot, uint32_t N, uint32_t W);

/* A candidate is a position a after its run's first token such that the W tokens from a lie inside the
 * run and their hash is in the set.  Its stored text covers the tokens a .. e: e the last token of the
 * run such that every key (tokens a..j), a+W-1 <= j <= e, is in the index (the pre-check by substring
 * hashes of Step 2).
 * Choice of the candidates that serve, per run: a piece of covered text begins at the first candidate
 * that no chosen text reaches; as long as a candidate that starts inside the text covered so far
 * reaches beyond it, the one that reaches furthest (the earliest such) is chosen next.  The chosen
 * candidates of a piece go alternately to stream a and stream b, the first to a.
 *   hash_a_out[i] / hash_b_out[i] = key of tokens c..i if i lies in the text of a chosen candidate c
 *     of that stream, else CPO_HASH_NONE (also for sensitive tokens);
 *   off_*_out (nullable): i - c, or 0xFFFFFFFF.  hash_b_out may be NULL. */
void cpo_hash_floating(const cpo_anchor_set *, const cpo_index *, const uint64_t *hash,
                       const uint32_t *run_off, uint32_t N, uint64_t base, uint32_t W,
                       uint64_t *hash_a_out, uint32_t *off_a_out, uint64_t *hash_b_out, uint32_t *off_b_out);

/* Lookup with two keys per token: slot under hash_a if present, else under hash_b, else NONE. */
void cpo_probe2(const cpo_index *, const uint64_t *hash_a, const uint64_t *hash_b, uint32_t N,
                uint32_t *slot_out);
/* ... with three keys (hash_b, hash_c may be NULL). */
void cpo_probe3(const cpo_index *, const uint64_t *hash_a, const uint64_t *hash_b, const uint64_t *hash_c,
                uint32_t N, uint32_t *slot_out);

/* ---- Exact verification (Sec. 4.2.2, Step 2 "full verification") ----
 * A hash match is only a candidate.  The paper confirms it with a cryptographic hash of the
 * substring so that no collision of the rolling hash can produce a false match; what that reaches
 * is "the stored text equals the request's text", and this oracle writes that definition out: it
 * keeps the text every slot was stored for and compares token by token.
 * A match is extended from the start of its segment (run start, or floating anchor) one token at a
 * time and ends at the first token that fails: token i is accepted iff token i-1 of the segment was
 * (or i starts it) and its candidate slot holds exactly the segment's tokens up to i. */
typedef struct cpo_text cpo_text; /* per slot: the token string it was stored for. Opaque. */
cpo_text *cpo_text_new(uint32_t n_slots);
void cpo_text_free(cpo_text *);
/* Call after cpo_insert_kv with the batch's tokens, run offsets and slot_out.  Slots seen for the
 * first time get their text (the run from its start through the token); a token whose slot holds
 * a different text, or that follows such a token in its run, gets slot_out = NONE, and a slot
 * first filled by such a token never matches anything. */
void cpo_text_record(cpo_text *, const uint32_t *tok, const uint32_t *run_off, uint32_t N,
                     uint32_t *slot_out);
/* The same after cpo_insert_kv_dedup, with ins_off in place of run_off; a token that the lookup found
 * is checked against its slot's whole text, whatever came before it. */
void cpo_text_record_dedup(cpo_text *, const uint32_t *tok, const uint32_t *ins_off, const uint32_t *found,
                           uint32_t N, uint32_t *slot_out);
/* seg_off[i] = offset of token i in its segment (0 = first, 0xFFFFFFFF = in none); cand[i] = the
 * slot found under the segment's key for i.  slot_out[i] = cand[i] if accepted, else NONE; with
 * merge != 0 only entries of slot_out that are NONE are written. */
void cpo_verify(const cpo_text *, const uint32_t *tok, const uint32_t *seg_off, const uint32_t *cand,
                uint32_t N, int merge, uint32_t *slot_out);
/* ---- Pool policies ----
 * Minimum segment length (Sec. 4.2.1 "Optimization"): a stretch = a maximal run of consecutive
 * positions of one request with slot_in != NONE; a stretch shorter than min_len is dropped whole.
 * Recompute marks (Sec. 4.2.1 Step 3): in a kept stretch, a token whose slot is marked in
 * slot_recompute (nullable) is dropped.  Dropped = slot_out NONE. */
void cpo_filter_matches(const uint32_t *slot_in, const uint32_t *off, uint32_t R, uint32_t min_len,
                        const uint8_t *slot_recompute, uint32_t n_pool_slots, uint32_t *slot_out);
/* slot_recompute[slot[i]] = 1 for every token with a slot and recompute[i] != 0 (marks accumulate). */
void cpo_mark_recompute(const uint32_t *slot, const uint8_t *recompute, uint32_t N,
                        uint32_t n_pool_slots, uint8_t *slot_recompute);
/* Zero placeholders (Sec. 4.3.1 "Operational details"): all rows of every token with slot NONE
 * are set to zero; other rows are not touched. */
void cpo_fill_unmatched(const uint32_t *slot, uint32_t N, void *dst, cpo_layout dst_l);
/* Least-recently-used eviction (Sec. 4.3.5 "Lifecycle management").  slot_stamp[s] = epoch of the
 * last batch that used slot s, 0 = free.  cpo_touch raises the stamp of every named slot to epoch.
 * cpo_lru_threshold returns the smallest T of the form epoch_now - a + 1, a < max_age, such that at
 * least n_needed slots were last used before T (all slots of age max_age - 1 or more count as one
 * class); epoch_now + 1 if even that is not enough, 0 if n_needed = 0.  cpo_evict frees every slot
 * in use with stamp < threshold: its key leaves the index, its stamp, mark and text are cleared, a
 * prefix hash recorded for it leaves the anchor set; the freed slots are listed in ascending order;
 * returns their number. */
void cpo_touch(const uint32_t *slot, uint32_t N, uint32_t epoch, uint32_t n_pool_slots,
               uint32_t *slot_stamp);
uint32_t cpo_lru_threshold(const uint32_t *slot_stamp, uint32_t n_pool_slots, uint32_t epoch_now,
                           uint32_t n_needed, uint32_t max_age);
uint32_t cpo_evict(cpo_index *, uint32_t *slot_stamp, uint32_t n_pool_slots, uint32_t threshold,
                   uint32_t *freed_slots, cpo_text *text /* nullable */,
                   uint8_t *slot_recompute /* nullable */, cpo_anchor_set *anchors /* nullable */);
/* ---- KV annotator (Sec. 4.2.1 "C1", Steps 1-3) ----
 * attn: n x n attention weights of one request, row i = what token i attends to, row stride ld
 * (elements).  Arithmetic is exact: every weight is first turned into the integer
 * round(x * 2^32) (entries above the diagonal and non-finite values and |x| > 2^18 count as 0), and all
 * sums are 64-bit integers, so no result depends on the order of the additions.
 * Step 1, cpo_sat_build: the summed-area table by the recurrence
 *     T[i,j] = A[i,j] + T[i-1,j] + T[i,j-1] - T[i-1,j-1]        (T dense, n x n).
 * cpo_sat_rect: sum of A over rows x1..x2, columns y1..y2 from four table entries.
 * Steps 2-3, cpo_annotate, for every coarse segment (maximal run of mask = 0 tokens):
 *   Step 2: among its substrings [l, r] of at least min_len tokens, the one that maximises
 *     IntraAttn - InterAttn = sum(rows l..r, cols l..r) - sum(rows l..r, cols < l);
 *     ties: smallest l, then smallest r.  best_l / best_r / best_score are written for every token
 *     of the segment (0xFFFFFFFF, 0 if the segment is shorter than min_len or the token sensitive);
 *     reusable[i] = 1 inside the chosen substring if it meets the reuse criterion
 *     IntraAttn > InterAttn (best_score > 0); otherwise the segment yields nothing to store.
 *   Step 3: tokens of a chosen substring that is reusable are ranked by (their row's attention to columns < l)
 *     - (their row's attention to columns l..i), largest first, earlier token first on ties;
 *     the first floor(len * rho_percent / 100) get recompute[i] = 1. */
void cpo_sat_build(const float *attn, uint32_t n, uint64_t ld, int64_t *T);
int64_t cpo_sat_rect(const int64_t *T, uint32_t n, int64_t x1, int64_t x2, int64_t y1, int64_t y2);
void cpo_annotate(const int64_t *T, uint32_t n, const uint8_t *mask, uint32_t min_len,
                  uint32_t rho_percent, uint32_t *best_l, uint32_t *best_r, int64_t *best_score,
                  uint8_t *reusable, uint8_t *recompute);
/* Building blocks exposed so that tests can pin them one by one. */
double cpo_bf16_to_double(uint16_t bits);
uint16_t cpo_double_to_bf16(double x); /* round-to-nearest-even, one rounding */
/* Rotate one head (head_dim bf16 values) by delta positions. */
void cpo_rope_head(const uint16_t *in, uint16_t *out, uint32_t head_dim, int32_t delta,
                   double theta, uint32_t style);
/* Same rotation without any rounding: double in, double out. */
void cpo_rope_head_f64(const double *in, double *out, uint32_t head_dim, double delta,
                       double theta, uint32_t style);

#ifdef __cplusplus
}
#endif
#endif

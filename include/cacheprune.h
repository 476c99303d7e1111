/*
 * libcacheprune — token-granular, privacy-aware KV-cache sharing on AMD MI355X
 * (gfx950).  C ABI of the data-parallel hot path of CachePrune:
 *
 *   lookup :  cp_hash_segments -> cp_probe -> cp_build_spans -> cp_gather_kv
 *             (cp_hash_probe does the first two in one pass)
 *   insert :  cp_hash_segments -> cp_insert_kv
 *
 * and, further down, the calls that widen it to the paper's retrieval and pool
 * life cycle: floating anchors (cp_hash_runs, cp_insert_anchors, cp_hash_floating,
 * cp_probe2, cp_probe3), exact confirmation of matches (cp_insert_kv_chain, cp_verify_chain,
 * cp_verify_streams),
 * one copy of stored text (cp_insert_keys, cp_insert_kv_dedup), pool policies
 * (cp_filter_matches, cp_mark_recompute, cp_fill_unmatched, cp_touch, cp_lru_threshold, cp_evict,
 * cp_table_compact, cp_table_count) and the KV annotator (cp_sat_build, cp_annotate).
 *
 * Conventions for every call
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls enqueue work and return; none synchronises.  Work of successive
 *     calls on one stream runs in order.
 *   - Unless a parameter says "host", every pointer is a DEVICE pointer owned
 *     by the caller.  The library allocates and frees nothing and keeps no state
 *     between calls besides each host thread's last HIP error code: every option
 *     of a call is an argument of that call.
 *   - `scratch` is caller-provided device memory of at least
 *     cp_scratch_bytes(N, max_spans, n_pool_slots) bytes, 256-byte aligned, whose contents are
 *     meaningless between calls; calls that share a scratch buffer must be on
 *     one stream.
 *   - R requests are packed back to back: request r holds the tokens
 *     off[r] .. off[r+1]-1, off[0] = 0, off[R] = N, off non-decreasing.
 *   - Return value: CP_OK or a negative CP_ERR_* code.  Argument errors are
 *     detected on the host before anything is enqueued.  Capacity conditions
 *     found on the device do not fail the call; they set bits in the caller's
 *     device word `status_flags` (or-ed in, never cleared by the library).
 *   - Limits: N < 2^31 tokens per call, pool slots < 2^31, table capacity
 *     < 2^32 entries, bf16 KV only.
 */
#ifndef CACHEPRUNE_H
#define CACHEPRUNE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CP_HASH_NONE 0xFFFFFFFFFFFFFFFFull /* hash of a sensitive token; also "empty" table key */
#define CP_SLOT_NONE 0xFFFFFFFFu           /* "no pool slot" */

#define CP_OK 0
#define CP_ERR_INVALID_ARG (-1) /* null / misaligned pointer, inconsistent sizes          */
#define CP_ERR_UNSUPPORTED (-2) /* shape or size outside the limits above                  */
#define CP_ERR_HIP (-3)         /* a launch failed; see cp_last_hip_error()                */
#define CP_ERR_SCRATCH (-4)     /* scratch_bytes smaller than cp_scratch_bytes() demands   */
#define CP_ERR_STATIC_LIMIT (-5) /* cp_gather_kv_static: a size above CP_STATIC_MAX_*      */

#define CP_FLAG_SPANS_OVERFLOW 1u /* more than max_spans spans: only the first max_spans kept  */
#define CP_FLAG_POOL_FULL 2u      /* free list used up: later new tokens were not stored       */
#define CP_FLAG_TABLE_FULL 4u     /* the table cannot take the batch's new keys: none was stored */
#define CP_FLAG_BAD_INDEX 8u      /* a span / free-list entry points outside pool or buffer: skipped */

#define CP_TABLE_BUCKET 16u /* table entries per bucket; capacity is a multiple of it */

/* Open-addressing hash table  chain hash -> pool slot  (the pool index of
 * Sec. 4.3.5 "Storage format and indexing", one key per pooled token).
 * `capacity` entries, a multiple of CP_TABLE_BUCKET, any such value (not only
 * powers of two).  cp_table_init makes it empty.  Only the mapping is part of
 * the contract; the arrangement of entries is not. */
typedef struct {
  uint64_t *keys;    /* [capacity], 128-byte aligned */
  uint32_t *vals;    /* [capacity], 64-byte aligned  */
  uint64_t capacity; /* entries */
} cp_table;

/* Where the KV rows of a token (or pool slot) live.  Row (t, layer, kv) with
 * kv = 0 for K and 1 for V starts at byte
 *     base + t * tok_stride + layer * layer_stride + kv * kv_stride
 * and holds n_kv_heads * head_dim bf16 values contiguously.  Base and strides
 * are multiples of 16 bytes and so is the row size. */
typedef struct {
  uint32_t n_layers, n_kv_heads, head_dim;
  uint64_t tok_stride, layer_stride, kv_stride; /* bytes */
} cp_kv_layout;

/* Rotary position embedding used when a cached key is reused at another
 * position (not part of the paper; the textbook rotation).  style 0 pairs
 * element j with j + head_dim/2, style 1 pairs 2j with 2j + 1. */
typedef struct {
  double theta;
  uint32_t style;
} cp_rope;

/* Smallest valid table capacity that keeps n_keys keys at or below load_factor. */
uint64_t cp_table_capacity_for(uint64_t n_keys, double load_factor);

/* Device bytes of scratch that any call below needs for N tokens (the larger of
 * the batch size and the number of destination tokens), max_spans spans and a
 * pool of n_pool_slots slots. */
size_t cp_scratch_bytes(uint32_t N, uint32_t max_spans, uint32_t n_pool_slots);

/* hipError_t of the last failed launch of this thread's calls (0 = none). */
int32_t cp_last_hip_error(void);

/* Launch options of the row mover behind cp_gather_kv / cp_insert_kv* (the one kernel of a call
 * that is bound by HBM).  Passed per call as a HOST pointer that is read before the call returns;
 * NULL, or a zeroed struct, means the defaults.  Results never depend on these options.
 *   read_sharing     1 = tokens of one gather that read the same pool slot share one read of it
 *                    ("read once, write many"), 2 = every token reads for itself, 0 = default: shared
 *                    from 4096 destination tokens on (below that the two extra launches cost more)
 *   blocks_per_cu    resident workgroups per compute unit (0 = default: one workgroup on seven of
 *                    every eight units where a token's rows allow 16 loads in flight, else 2; 2 for a
 *                    gather that re-rotates keys)
 *   nontemporal      0 = default (stores only), else 1 + (bit 0: non-temporal loads, bit 1: non-temporal stores)
 *   loads_in_flight  16-byte loads a lane issues before its first store (0 = default: 16 for the
 *                    Llama row shapes, fewer for small tokens, 8 for a gather that re-rotates keys;
 *                    4, 8 or 16, a rotating gather at most 8)
 *   workgroups       grid size of the kernel; overrides blocks_per_cu (0 = not given)
 *   fanout           destinations written per pass over the rows of a shared slot (0 = default 16,
 *                    1..16; fewer means the rows are fetched again, normally from cache)
 *   start_event, stop_event   two hipEvent_t (host handles as void*, created and destroyed by the
 *                    caller; NULL = none) recorded on the call's stream right before and right
 *                    after the row-mover kernel, so that a benchmark can time it apart from the
 *                    small set-up kernels of the call. */
typedef struct {
  uint32_t read_sharing, blocks_per_cu, nontemporal, loads_in_flight, fanout, workgroups;
  uint32_t reserved[2]; /* must be 0 */
  void *start_event, *stop_event;
} cp_launch_opts;

/* hipEvent helpers for callers without their own HIP binding: create a timing
 * event (NULL on failure), milliseconds between two recorded events (negative
 * on failure, e.g. not yet complete), destroy. */
void *cp_event_create(void);
float cp_event_elapsed_ms(void *start_event, void *stop_event);
void cp_event_destroy(void *event);

/* Empty the table: every key CP_HASH_NONE, every value CP_SLOT_NONE. */
int32_t cp_table_init(void *stream, cp_table table);

/* Segmented chain hash (Sec. 4.2.1: sensitive tokens are separators that cut a
 * prompt into segments; Sec. 4.2.2: polynomial rolling hash, here modulo 2^64).
 * For the k-th token of a run of non-sensitive tokens t_0 .. t_k inside one
 * request:  hash = sum_{m<=k} (t_m + 1) * base^(k-m)  mod 2^64, with the value
 * CP_HASH_NONE replaced by CP_HASH_NONE - 1.  Sensitive tokens (mask != 0) get
 * CP_HASH_NONE; runs restart after them and at every request start.
 *   tok [N] uint32, mask [N] uint8, off [R+1] uint32  ->  hash_out [N] uint64. */
int32_t cp_hash_segments(void *stream, const uint32_t *tok, const uint8_t *mask, const uint32_t *off,
                         uint32_t N, uint32_t R, uint64_t base, uint64_t *hash_out, void *scratch,
                         size_t scratch_bytes);

/* Table lookup (the hash lookup the retriever performs, Sec. 4.2.2 / 4.3.1):
 * slot_out[i] = slot stored under hash[i], or CP_SLOT_NONE if the key is absent
 * or hash[i] is CP_HASH_NONE.  A sensitive token is therefore never served. */
int32_t cp_probe(void *stream, cp_table table, const uint64_t *hash, uint32_t N, uint32_t *slot_out);

/* cp_hash_segments (or cp_hash_runs, if run_off_out is not NULL) and cp_probe in one pass: every
 * token's hash is looked up where it is computed, which saves a launch on the way to the slots
 * (a single request is bound by its launches, Sec. 5.4.2 measures the retriever per request).
 * Same results as the two calls. */
int32_t cp_hash_probe(void *stream, const uint32_t *tok, const uint8_t *mask, const uint32_t *off, uint32_t N,
                      uint32_t R, uint64_t base, cp_table table, uint64_t *hash_out, uint32_t *run_off_out,
                      uint32_t *slot_out, void *scratch, size_t scratch_bytes);

/* ---- Floating anchors: matches that do not start at the start of a run --------------------------
 * Sec. 4.2.2 Step 1 ("prefix filtering"): every stored segment keeps the hash of its first W tokens;
 * a W-token window slides over the request and is compared with those prefix hashes, which yields a
 * set of candidates.  Step 2: each candidate is checked over the text stored behind it; the hash of
 * any substring follows in O(1) from prefix hashes and a power of the base.  Here:
 *   - cp_hash_runs is cp_hash_segments that also returns run_off[i], the number of tokens between
 *     the start of token i's run and i (0xFFFFFFFF for sensitive tokens);
 *   - the hash of a stored run's first W tokens is the table key of the run's W-th token, so the
 *     set of stored prefix hashes is kept as one mark byte per pool slot, slot_anchor
 *     (u8[n_pool_slots], caller-owned, initialised to 0): the keys whose slot is marked are the
 *     prefix hashes.  cp_insert_anchors, called after an insert with the slot_out it reported, sets
 *     slot_anchor[slot[i]] = 1 for every token with run_off[i] == W - 1 and a slot.  A prefix hash
 *     thus lives exactly as long as the run's W-th token is stored (cp_evict clears the mark);
 *   - a candidate is a position a after its run's first token whose W-token window lies inside the
 *     run and hashes to a key of `table` whose slot is marked.  Its stored text reaches ext(a), the
 *     last token e of the run such that the key of the request's tokens a..j,
 *         hash[j] - hash[a-1] * base^(j-a+1)   (mod 2^64; CP_HASH_NONE -> NONE-1),
 *     is in `table` for every j from the window's end through e.  That key equals the chain hash the
 *     same tokens get as the beginning of a stored run, so it is looked up in the ordinary table.
 *     (Stored runs are closed under taking prefixes - every insert, truncation and eviction of this
 *     library keeps them so - and ext(a) is found by bisection.)
 *   - a token can lie in the text of several candidates, and every token that some candidate covers
 *     is to be served.  The candidates that serve are chosen like the intervals of a greedy cover: a
 *     piece of covered text begins at the first candidate that no earlier candidate's text reaches;
 *     as long as a candidate that starts inside the text covered so far reaches beyond it, the one
 *     that reaches furthest (the earliest such) is chosen next.  A chosen candidate then overlaps
 *     only with the one chosen before it and the one chosen after it, and the chosen candidates of a
 *     piece are handed alternately to two key streams, a and b (the first to a): inside a stream the
 *     texts are whole and never overlap, which is what cp_verify_chain and cp_build_spans need.
 *     cp_hash_floating gives every token its key in either stream: hash_a_out[i] / hash_b_out[i] =
 *     key of c..i if i lies in the text of a chosen candidate c of that stream, else CP_HASH_NONE.
 *     off_a_out / off_b_out (device u32[N], may be NULL): i - c, or 0xFFFFFFFF.  hash_b_out may be
 *     NULL.
 *   - cp_probe2 / cp_probe3 look every token up under the first key and, while that misses, under
 *     the next.
 * A token is thus served under its run-start key if possible, else from the candidate chosen for it
 * in stream a, else in stream b: every token that any candidate's stored text covers is served,
 * however many candidates overlap there.
 * `base` must be odd.  W >= 1. */
int32_t cp_hash_runs(void *stream, const uint32_t *tok, const uint8_t *mask, const uint32_t *off, uint32_t N,
                     uint32_t R, uint64_t base, uint64_t *hash_out, uint32_t *run_off_out, void *scratch,
                     size_t scratch_bytes);
int32_t cp_insert_anchors(void *stream, const uint32_t *run_off, const uint32_t *slot, uint32_t N, uint32_t W,
                          uint32_t n_pool_slots, uint8_t *slot_anchor);
int32_t cp_hash_floating(void *stream, cp_table table, const uint8_t *slot_anchor, uint32_t n_pool_slots,
                         const uint64_t *hash, const uint32_t *run_off, uint32_t N, uint64_t base, uint32_t W,
                         uint64_t *hash_a_out, uint32_t *off_a_out, uint64_t *hash_b_out, uint32_t *off_b_out,
                         void *scratch, size_t scratch_bytes);
int32_t cp_probe2(void *stream, cp_table table, const uint64_t *hash_a, const uint64_t *hash_b, uint32_t N,
                  uint32_t *slot_out);
int32_t cp_probe3(void *stream, cp_table table, const uint64_t *hash_a, const uint64_t *hash_b, const uint64_t *hash_c,
                  uint32_t N, uint32_t *slot_out);

/* ---- Exact matches: no false match from a collision of the rolling hash -------------------------
 * Sec. 4.2.2 Step 2 ("full verification"): a candidate found through the rolling hash is confirmed
 * before it is used, so that a collision cannot link another text's KV.  The paper confirms with a
 * cryptographic hash of the substring; this library confirms by comparison with what the pool
 * recorded when it stored the tokens, which is exact.  Two caller-owned device arrays of
 * n_pool_slots words describe the stored runs as a trie whose nodes are slots:
 *     slot_tok[s]    = token id slot s was stored for,
 *     slot_parent[s] = slot of the token before it in its run, CP_SLOT_NONE for a run's first token.
 * Initialise slot_parent to CP_PARENT_POISON (a value no lookup ever equals); slot_tok needs none.
 *
 * cp_insert_kv_chain is cp_insert_kv that also maintains the two arrays.  tok / run_off: the batch's
 * tokens and run offsets (cp_hash_runs).  Every token's slot is confirmed against the recorded
 * chains before it is reported: slot_out[i] = the slot that holds exactly the tokens of i's run up to
 * i, CP_SLOT_NONE for a sensitive token, a token that could not be stored, and a token whose key
 * belongs to another text (or that follows such a token in its run).  A slot taken by a token of the
 * last kind is consumed but can never match (its parent is set to CP_PARENT_POISON).
 *
 * cp_verify_chain confirms the candidates of one key stream of a lookup.  seg_off[i] = offset of
 * token i in its segment: run_off for run-start keys, off_a / off_b for the two floating
 * streams; 0xFFFFFFFF = in no segment.  cand[i] = slot found under that stream's key (cp_probe).  Token i is accepted iff
 * every token from its segment's start through i is consistent: cand < n_pool_slots,
 * slot_tok[cand[i]] == tok[i], and slot_parent[cand[i]] == cand[i-1] (CP_SLOT_NONE at offset 0); by
 * induction cand[i] then holds exactly the segment's tokens up to i.  slot_out[i] = cand[i] if
 * accepted, else CP_SLOT_NONE; with merge != 0 only entries of slot_out that are CP_SLOT_NONE are
 * written (second key stream).  stream_out (may be NULL) receives this stream's own result for
 * every token whatever slot_out held: a token that both streams accept is served from the first,
 * but the second stream's slots were used to get there and count as used for eviction (cp_touch).
 * cand must not be the same array as slot_out or stream_out. */
#define CP_PARENT_POISON 0xFFFFFFFEu
int32_t cp_insert_kv_chain(void *stream, cp_table table, const uint64_t *hash, const uint32_t *tok,
                           const uint32_t *run_off, const uint32_t *off, uint32_t N, uint32_t R,
                           const uint32_t *free_slots, uint32_t n_free, const void *src, cp_kv_layout src_l,
                           void *pool, cp_kv_layout pool_l, uint32_t n_pool_slots, int32_t *slot_pos,
                           uint32_t *slot_tok, uint32_t *slot_parent, uint32_t *slot_out, uint32_t *n_inserted,
                           uint32_t *status_flags, void *scratch, size_t scratch_bytes, const cp_launch_opts *opts);
int32_t cp_verify_chain(void *stream, const uint32_t *tok, const uint32_t *seg_off, const uint32_t *cand, uint32_t N,
                        const uint32_t *slot_tok, const uint32_t *slot_parent, uint32_t n_pool_slots, int32_t merge,
                        uint32_t *slot_out, uint32_t *stream_out, void *scratch, size_t scratch_bytes);

/* cp_verify_streams: the three key streams of a lookup with floating anchors confirmed in one call -
 * what cp_probe + cp_verify_chain per stream and the merge in serving order give, in three launches
 * instead of eight.  Stream 0: run-start keys, candidates cand_0 already looked up (cp_hash_probe),
 * offsets seg_off_0 = run_off.  Streams a and b: keys and offsets of cp_hash_floating, looked up here.
 * slot_out[i] = the slot of the first stream (0, a, b) that accepts token i, else CP_SLOT_NONE;
 * stream_out_0 / _a / _b (each may be NULL): every stream's own result (for cp_touch and
 * cp_insert_keys).  cand_0 must not alias an output. */
int32_t cp_verify_streams(void *stream, cp_table table, const uint32_t *tok, uint32_t N, const uint32_t *seg_off_0,
                          const uint32_t *cand_0, const uint64_t *key_a, const uint32_t *seg_off_a,
                          const uint64_t *key_b, const uint32_t *seg_off_b, const uint32_t *slot_tok,
                          const uint32_t *slot_parent, uint32_t n_pool_slots, uint32_t *slot_out,
                          uint32_t *stream_out_0, uint32_t *stream_out_a, uint32_t *stream_out_b, void *scratch,
                          size_t scratch_bytes);

/* Run-length pass: turn per-token slots into copy descriptors (the "token
 * spans" of the retriever's metadata, Sec. 4.3.1).  A span is a maximal run of
 * consecutive positions of one request whose slots are valid and consecutive
 * and, if slot_pos is given, share one position delta
 *     delta = (position inside the request) - slot_pos[slot].
 * Spans are written in (request, position) order: span_src = first pool slot,
 * span_dst = packed index of the first token, span_len, span_delta.
 * *n_spans (device) = min(number of spans, max_spans); if there were more,
 * CP_FLAG_SPANS_OVERFLOW is set and the first max_spans are kept.
 * slot_pos and span_delta may be NULL (then delta is 0 / not written).
 * span_off, if not NULL, receives [max_spans + 1] exclusive prefix sums of
 * span_len (span_off[k] = tokens covered by spans 0..k-1, entries up to
 * *n_spans are valid); passing it on to cp_gather_kv saves that call a pass. */
int32_t cp_build_spans(void *stream, const uint32_t *slot, const uint32_t *off, uint32_t N, uint32_t R,
                       const int32_t *slot_pos, uint32_t max_spans, uint32_t *span_src,
                       uint32_t *span_dst, uint32_t *span_len, int32_t *span_delta,
                       uint32_t *span_off, uint32_t *n_spans, uint32_t *status_flags, void *scratch,
                       size_t scratch_bytes);

/* Token-granular gather ("links them to the sequence", Sec. 4.1 KV Retriever;
 * here a copy out of the pool into the request's per-layer K/V buffers).
 * For every span s < *n_spans, k < span_len[s], every layer, K and V:
 *     row(dst, span_dst[s] + k)  <-  row(pool, span_src[s] + k).
 * Rows of tokens not covered by a span are not written (Sec. 4.3.1: unmatched
 * positions are left for the engine).  If rope and span_delta are both
 * non-NULL, K rows of spans with delta != 0 are rotated by delta positions
 * (evaluated in double precision, rounded once to bf16); V rows and spans with
 * delta == 0 are copied bit for bit.  `rope` is a HOST pointer, read before
 * the call returns.  span_off may be NULL (computed internally) or the array
 * cp_build_spans produced.  Spans must not overlap in dst.  pool_l and dst_l must agree on n_layers, n_kv_heads and head_dim;
 * rotation needs head_dim a power of two in [16, 512].  The pool holds
 * n_pool_slots slots and dst n_dst_tokens tokens: a token of a span that falls
 * outside either is skipped and CP_FLAG_BAD_INDEX is set.  opts: see cp_launch_opts (may be NULL). */
int32_t cp_gather_kv(void *stream, const void *pool, cp_kv_layout pool_l, uint32_t n_pool_slots, void *dst,
                     cp_kv_layout dst_l, uint32_t n_dst_tokens, const uint32_t *span_src,
                     const uint32_t *span_dst, const uint32_t *span_len, const int32_t *span_delta,
                     const uint32_t *span_off, const uint32_t *n_spans, uint32_t max_spans,
                     const cp_rope *rope, uint32_t *status_flags, void *scratch, size_t scratch_bytes,
                     const cp_launch_opts *opts);

/* cp_gather_kv for callers that cannot allocate device memory or have nowhere to keep a scratch
 * buffer: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments and results as cp_gather_kv without `scratch`: the working memory (span offsets,
 * per-token descriptors, chain heads, rotation tables) is an array inside the library's device code,
 * about 10 MiB, which every GPU the library runs on holds from the library's first use there until the
 * process ends.  Sizes are limited to n_dst_tokens <= CP_STATIC_MAX_TOKENS, max_spans <=
 * CP_STATIC_MAX_SPANS and n_pool_slots <= CP_STATIC_MAX_SLOTS; anything larger returns
 * CP_ERR_STATIC_LIMIT and enqueues nothing.  The call allocates and frees nothing.  The stream must
 * belong to the calling thread's current device.  All calls on one GPU share the one array: calls
 * that may overlap on a GPU (different streams, different threads) race and must be ordered by the
 * caller; calls on one stream are ordered already. */
#define CP_STATIC_MAX_TOKENS 131072u
#define CP_STATIC_MAX_SPANS 131072u
#define CP_STATIC_MAX_SLOTS 524288u
int32_t cp_gather_kv_static(void *stream, const void *pool, cp_kv_layout pool_l, uint32_t n_pool_slots, void *dst,
                            cp_kv_layout dst_l, uint32_t n_dst_tokens, const uint32_t *span_src,
                            const uint32_t *span_dst, const uint32_t *span_len, const int32_t *span_delta,
                            const uint32_t *span_off, const uint32_t *n_spans, uint32_t max_spans,
                            const cp_rope *rope, uint32_t *status_flags, const cp_launch_opts *opts);

/* Insert-if-absent with the matching scatter (post-inference storing, Sec. 4.1
 * "Workflow"; one copy of a duplicate, Sec. 4.3.5 "Lifecycle management").
 * Every token with hash != CP_HASH_NONE whose key is not in the table gets a
 * table entry and a pool slot; its rows are copied  row(src, i) -> row(pool,
 * slot)  and slot_pos[slot] = position inside its request.  Determinism: if a
 * key occurs several times in one call the occurrence with the lowest packed
 * index stores it, keys already present are left alone, and new slots are
 * free_slots[0], free_slots[1], .. in packed order of the storing tokens — the
 * result does not depend on scheduling.  When the n_free slots are used up the
 * remaining new tokens are dropped and CP_FLAG_POOL_FULL is set.  Free-list
 * entries >= n_pool_slots are never used (CP_FLAG_BAD_INDEX).  A key takes a
 * table entry when an insert first sees it and keeps it, also without a slot
 * (pool full, evicted), until the table is rebuilt (cp_table_compact).  If the
 * table cannot take every new key of the call, CP_FLAG_TABLE_FULL is set and the
 * call stores nothing (slot_out still reports the keys that were stored before;
 * *n_inserted = 0); which of the new keys took the last entries is unspecified,
 * so rebuild the table into a larger one before storing again.
 *   slot_out [N]: slot holding each token's key after the call, CP_SLOT_NONE
 *                 for sensitive or dropped tokens.
 *   *n_inserted (device): number of tokens stored by this call.
 *   opts: launch options of the scatter (may be NULL); read_sharing and fanout do not apply. */
int32_t cp_insert_kv(void *stream, cp_table table, const uint64_t *hash, const uint32_t *off, uint32_t N,
                     uint32_t R, const uint32_t *free_slots, uint32_t n_free, const void *src,
                     cp_kv_layout src_l, void *pool, cp_kv_layout pool_l, uint32_t n_pool_slots,
                     int32_t *slot_pos, uint32_t *slot_out, uint32_t *n_inserted, uint32_t *status_flags,
                     void *scratch, size_t scratch_bytes, const cp_launch_opts *opts);

/* ---- One copy of a text that the pool already holds -------------------------------------------
 * Sec. 4.3.5 "Lifecycle management": the pool keeps one copy of duplicated segments, and of a
 * segment that another stored segment contains.  cp_insert_kv alone keeps one copy of equal run
 * beginnings; with floating anchors a batch can also be checked for text that is stored behind other
 * text or as a run of its own.  Before storing, look the batch up: per key stream k (run-start keys,
 * then the candidate streams) slot_k[i] = what the stream found for token i (confirmed, if the pool
 * confirms matches) and seg_off_k[i] = the token's offset in the stream's segment.
 *   cp_insert_keys: for every non-sensitive token, the stored text it belongs to starts at
 *     c = i - seg_off_k[i] for the first stream k that found it; else at the c of its left neighbour
 *     in its run; else (first token of a run) at i.  ins_off_out[i] = i - c, ins_hash_out[i] = chain
 *     hash of the request's tokens c..i (the table key), found_out[i] = slot_k[i] or CP_SLOT_NONE.
 *     A token that was not found thus continues the stored text before it, so stored texts stay closed
 *     under taking prefixes.  Unused streams: both pointers NULL.  Sensitive tokens: CP_HASH_NONE,
 *     0xFFFFFFFF, CP_SLOT_NONE.
 *   cp_insert_kv_dedup: cp_insert_kv (slot_tok == slot_parent == NULL) or cp_insert_kv_chain under
 *     the keys ins_hash, with ins_off in the place of run_off, that leaves out every token with
 *     found[i] != CP_SLOT_NONE: it gets no table entry and no slot, slot_out[i] = found[i], and for
 *     the chain records it counts as confirmed.  Pass ins_off and slot_out on to cp_insert_anchors.
 * Texts stored by one call do not see each other (the lookup ran before): two requests of a batch
 * that bring the same new text behind different leads each store it. */
int32_t cp_insert_keys(void *stream, const uint64_t *hash, const uint32_t *run_off, uint32_t N, uint64_t base,
                       const uint32_t *seg_off_a, const uint32_t *slot_a, const uint32_t *seg_off_b,
                       const uint32_t *slot_b, const uint32_t *seg_off_c, const uint32_t *slot_c,
                       uint64_t *ins_hash_out, uint32_t *ins_off_out, uint32_t *found_out, void *scratch,
                       size_t scratch_bytes);
int32_t cp_insert_kv_dedup(void *stream, cp_table table, const uint64_t *ins_hash, const uint32_t *found,
                           const uint32_t *tok, const uint32_t *ins_off, const uint32_t *off, uint32_t N, uint32_t R,
                           const uint32_t *free_slots, uint32_t n_free, const void *src, cp_kv_layout src_l,
                           void *pool, cp_kv_layout pool_l, uint32_t n_pool_slots, int32_t *slot_pos,
                           uint32_t *slot_tok, uint32_t *slot_parent, uint32_t *slot_out, uint32_t *n_inserted,
                           uint32_t *status_flags, void *scratch, size_t scratch_bytes, const cp_launch_opts *opts);

/* ---- Pool policies -----------------------------------------------------------------------------
 * All arrays are device memory owned by the caller; scratch as for the other calls
 * (cp_scratch_bytes(N, 0, n_pool_slots)).
 *
 * cp_filter_matches - minimum segment length (Sec. 4.2.1 "Optimization": a segment qualifies as
 * reusable only from a minimum length) and recompute marks (Sec. 4.2.1 Step 3: marked tokens of a
 * reused segment are recomputed, not reused).  A stretch is a maximal run of consecutive positions
 * of one request with slot_in != CP_SLOT_NONE.  slot_out[i] = CP_SLOT_NONE for every token of a
 * stretch shorter than min_len and, in the other stretches, for tokens whose slot is marked in
 * slot_recompute (u8[n_pool_slots], may be NULL); slot_in[i] otherwise.  A marked token counts
 * towards the length of its stretch.  slot_out may be slot_in.
 *
 * cp_mark_recompute - slot_recompute[slot[i]] = 1 for every token with a slot and
 * recompute[i] != 0.  Called with the slot_out of an insert; marks accumulate over batches.
 *
 * cp_fill_unmatched - zero placeholders (Sec. 4.3.1 "Operational details": tokens that are not
 * linked are represented as zeros for the engine to fill): all rows of every token i < N of dst
 * with slot[i] == CP_SLOT_NONE are set to zero; no other row is written.
 *
 * Least-recently-used eviction (Sec. 4.3.5 "Lifecycle management"), at the granularity of batches:
 * slot_stamp[s] (u32[n_pool_slots]) = number (epoch >= 1) of the last batch that used slot s, 0 =
 * the slot is free.
 *   cp_touch: slot_stamp[slot[i]] = max(itself, epoch) for every token with a slot.  Call it with
 *     the unfiltered slots of a lookup - with two key streams, with what EACH stream accepted
 *     (cp_verify_chain's stream_out), not only with the merged result - and with the slot_out of an
 *     insert; since a match at a token implies matches of the same stream at the tokens before it
 *     in its segment, a token is then never older than the tokens stored behind it, and eviction by
 *     age never takes the head of a stored run whose tail stays.
 *   cp_lru_threshold: *threshold_out (device) = the smallest T = epoch_now - a + 1, 0 <= a <
 *     CP_LRU_MAX_AGE, such that at least n_needed slots in use have stamp < T (slots of age
 *     CP_LRU_MAX_AGE - 1 or more count as one class; stamps above epoch_now are never chosen);
 *     epoch_now + 1 if all slots in use together are fewer; 0 if n_needed == 0.
 *   cp_evict: every slot in use with stamp < *threshold (device) is freed: the value of its key's
 *     table entry becomes CP_SLOT_NONE (the key stays and is reused if the text is stored again),
 *     its stamp becomes 0, its slot_parent CP_PARENT_POISON, its slot_recompute and slot_anchor 0
 *     (each of the three arrays may be NULL).  freed_slots (u32[n_pool_slots]) receives the freed slots in ascending order,
 *     *n_freed (device) their number: append them to the free list.
 *   cp_table_compact: copy the live entries (value != CP_SLOT_NONE) of src into dst, which must be
 *     initialised and must not share memory with src; drops the keys eviction left behind.
 *     CP_FLAG_TABLE_FULL if dst is too small. */
#define CP_LRU_MAX_AGE 4096u
int32_t cp_filter_matches(void *stream, const uint32_t *slot_in, const uint32_t *off, uint32_t N, uint32_t R,
                          uint32_t min_len, const uint8_t *slot_recompute, uint32_t n_pool_slots, uint32_t *slot_out,
                          void *scratch, size_t scratch_bytes);
int32_t cp_mark_recompute(void *stream, const uint32_t *slot, const uint8_t *recompute, uint32_t N,
                          uint32_t n_pool_slots, uint8_t *slot_recompute);
int32_t cp_fill_unmatched(void *stream, const uint32_t *slot, uint32_t N, void *dst, cp_kv_layout dst_l);
int32_t cp_touch(void *stream, const uint32_t *slot, uint32_t N, uint32_t epoch, uint32_t n_pool_slots,
                 uint32_t *slot_stamp);
int32_t cp_lru_threshold(void *stream, const uint32_t *slot_stamp, uint32_t n_pool_slots, uint32_t epoch_now,
                         uint32_t n_needed, uint32_t *threshold_out, void *scratch, size_t scratch_bytes);
int32_t cp_evict(void *stream, cp_table table, uint32_t *slot_stamp, uint32_t n_pool_slots, const uint32_t *threshold,
                 uint32_t *freed_slots, uint32_t *n_freed, uint32_t *slot_parent, uint8_t *slot_recompute,
                 uint8_t *slot_anchor, void *scratch, size_t scratch_bytes);
int32_t cp_table_compact(void *stream, cp_table src, cp_table dst, uint32_t *status_flags);
/* How full the index is (Sec. 4.3.5 "Lifecycle management": the pool's bookkeeping between evictions):
 * counts_out (device, u32[2]) receives [0] the number of table entries that hold a key and [1] the number of
 * those whose key has a slot.  [0] - [1] entries are held by keys without a slot (dropped when the pool was
 * full, evicted, or claimed by a call that ended with CP_FLAG_TABLE_FULL): cp_table_compact gives them back.  Fails like cp_table_init on a malformed table. */
int32_t cp_table_count(void *stream, cp_table table, uint32_t *counts_out);

/* ---- KV annotator: which tokens of a finished request are worth storing ------------------------
 * Sec. 4.2.1 ("C1"), Steps 1-3.  attn (device, float[n][ld], ld >= n): attention weight from token
 * i (row) to token j (column) of one request.  mask (device, u8[n]): 1 = sensitive; sensitive
 * tokens cut the request into coarse segments.
 *
 * Exact arithmetic: a weight x counts as the integer round(x * 2^32), ties to even; entries above
 * the diagonal, non-finite values and |x| > 2^18 count as 0; all sums are 64-bit integers.
 *
 * cp_sat_build (Step 1): T (device, int64[n][n], dense) = summed-area table,
 *     T[i][j] = sum of the weights of rows <= i and columns <= j,
 *   valid for every j <= i.  No token attends to a later one, so T[i][j] = T[i][i] for j > i;
 *   those entries are not needed, cp_annotate never reads them, and most of them are not written.
 *   mask (device, u8[n], may be NULL): if given, only the part of the table that cp_annotate can
 *   read for this mask is written - the diagonal entries and, for the rows of a coarse segment
 *   [a, b], the columns from a - 64 on (in whole tiles) - and nothing else of T is defined.  A
 *   search only looks inside segments, so with sensitive tokens every few hundred positions most of
 *   the table is never asked for.  The weights are still all read (every sum needs them).
 *   cp_annotate must then be given the same mask (with another one it would read undefined
 *   entries: wrong decisions, though never memory outside T).
 * cp_annotate (Steps 2, 3), for every coarse segment [a, b]:
 *   - among its substrings [l, r] with at least min_len tokens (0 counts as 1) the one with the
 *     largest  IntraAttn - InterAttn = sum(rows l..r, columns l..r) - sum(rows l..r, columns < l);
 *     ties: smallest l, then smallest r.  For every token i of the segment best_l[i], best_r[i],
 *     best_score[i] describe that substring (0xFFFFFFFF, 0xFFFFFFFF, 0 for sensitive tokens and for
 *     segments shorter than min_len); the substring is reusable if it meets the reuse criterion of
 *     Sec. 4.2.1, IntraAttn > InterAttn, i.e. best_score > 0: reusable[i] = 1 iff that holds and
 *     best_l <= i <= best_r; store_mask (may be NULL) = 1 - reusable: the mask to hash and insert
 *     the request with, so that only the chosen substrings are stored;
 *   - the tokens of a reusable chosen substring are ranked by (their row's weight on columns < l) - (their
 *     row's weight on columns l..i), largest first, earlier token first on ties, and the first
 *     floor(len * rho_percent / 100) get recompute[i] = 1 (input of cp_mark_recompute).
 * n <= 2^20.  Scratch: cp_sat_scratch_bytes(n), 256-byte aligned, for either call. */
size_t cp_sat_scratch_bytes(uint32_t n);
int32_t cp_sat_build(void *stream, const float *attn, uint32_t n, uint64_t ld, const uint8_t *mask, int64_t *T,
                     void *scratch, size_t scratch_bytes);
int32_t cp_annotate(void *stream, const int64_t *T, uint32_t n, const uint8_t *mask, uint32_t min_len,
                    uint32_t rho_percent, uint32_t *best_l, uint32_t *best_r, int64_t *best_score, uint8_t *reusable,
                    uint8_t *recompute, uint8_t *store_mask, void *scratch, size_t scratch_bytes);

#ifdef __cplusplus
}
#endif
#endif

// Host-side declarations shared by the translation units of libcacheprune.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/cacheprune.h"

namespace cp {

// Launch options of the row mover, resolved from a call's cp_launch_opts (defaults chosen from
// measurements on MI355X).  Held by value for the duration of one call; nothing is process wide.
struct MoveOpts {
  bool share_reads;         // tokens that read the same pool slot are served by one read
  uint32_t blocks_per_cu;   // resident workgroups per compute unit (0 = chosen at launch)
  uint32_t workgroups;      // grid size, overrides blocks_per_cu (0 = not given)
  uint32_t nontemporal;     // bit 0: non-temporal loads, bit 1: non-temporal stores
  uint32_t loads_in_flight; // 16-byte loads a lane issues before its first store (4, 8, 16; 0 = chosen at launch)
  uint32_t fanout;          // destinations written per pass over a shared slot's rows (1..16)
  hipEvent_t start, stop;   // recorded right before / after the row-mover launch, if not null
};
// opts may be null (defaults); false if a field holds a value outside its documented range.
bool resolve_opts(const cp_launch_opts *opts, bool rotating, MoveOpts *out);

// Bump allocator over the caller's scratch buffer (256-byte aligned pieces).
struct Scratch {
  uint8_t *p;
  size_t left;
  Scratch(void *base, size_t bytes) : p((uint8_t *)base), left(bytes) {}
  template <class T>
  T *take(size_t n) {
    size_t bytes = (n * sizeof(T) + 255) & ~(size_t)255;
    if (bytes > left) return nullptr;
    T *r = (T *)p;
    p += bytes;
    left -= bytes;
    return r;
  }
};

bool layout_ok(const cp_kv_layout &l);
bool layouts_match(const cp_kv_layout &a, const cp_kv_layout &b);

// One token's worth of work for the row mover: copy all rows of `from` (a pool
// slot when gathering, a request token when scattering) to `to`.  `next` links
// the items that share a source into a chain (0xFFFFFFFF ends it); an item
// whose `from` is 0xFFFFFFFF is skipped.
struct alignas(16) MoveItem {
  uint32_t from, to;
  int32_t delta;
  uint32_t next;
};

// Row mover used by the insert path: for w < *n_items (device count, at most
// max_items) copy all rows of token items[w].from of `src` to slot items[w].to
// of `pool`.  `counter` is a device word that is 0 when the kernel starts.
// Items naming a token >= n_src_tokens or a slot >= n_pool_slots are skipped
// and flagged.
int32_t launch_scatter(hipStream_t stream, const void *src, const cp_kv_layout &src_l, uint32_t n_src_tokens,
                       void *pool, const cp_kv_layout &pool_l, uint32_t n_pool_slots, const MoveItem *items,
                       const uint32_t *n_items, uint32_t max_items, uint32_t *counter, uint32_t *status_flags,
                       const MoveOpts &mo);

// Exclusive prefix sums of span_len[0 .. *n_spans) into span_off[0 .. *n_spans],
// agg = div_up(max_spans, 1024) + 1 words of scratch.
int32_t launch_span_offsets(hipStream_t stream, const uint32_t *span_len, const uint32_t *n_spans, uint32_t max_spans,
                            uint32_t *span_off, uint32_t *agg);

// out_a[i], out_b[i] = slot stored under hash_a[i], hash_b[i] (CP_SLOT_NONE if absent): two lookups per token, one launch.
int32_t launch_probe_each(hipStream_t stream, cp_table table, const uint64_t *hash_a, const uint64_t *hash_b,
                          uint32_t N, uint32_t *out_a, uint32_t *out_b);

// ext1[a] = 1 + the last token t such that the key of tokens a..t is stored, for every position a that is a
// candidate (a W-token window starting at a, inside one run and after the run's first token, hashes to a
// key of `table` whose slot carries an anchor mark); 0 for every other position.
int32_t launch_anchor_extents(hipStream_t stream, const cp_table &table, const uint8_t *slot_anchor,
                              uint32_t n_pool_slots, const uint64_t *hash, const uint32_t *run_off, uint32_t N,
                              uint32_t W, uint64_t base, uint32_t *ext1);

// Segmented prefix AND of the per-token chain checks (see verify.hip): slot_out[i] = cand[i] if every
// token from the start of i's segment through i is consistent with slot_tok / slot_parent, else
// CP_SLOT_NONE; with merge only entries that are CP_SLOT_NONE are written; stream_out (nullable) gets
// the same values without regard to merge.  agg: one word per scan tile of N elements, + 1.
int32_t launch_chain_verify(hipStream_t stream, const uint32_t *tok, const uint32_t *seg_off, const uint32_t *cand,
                            uint32_t N, const uint32_t *slot_tok, const uint32_t *slot_parent, uint32_t n_pool_slots,
                            uint32_t merge, uint32_t *slot_out, uint32_t *stream_out, uint32_t *agg,
                            const uint32_t *trusted /* nullable: tokens with trusted[i] != NONE pass and start anew */);

}  // namespace cp

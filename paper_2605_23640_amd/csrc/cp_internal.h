// Host-side declarations shared by the translation units of libcacheprune.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/cacheprune.h"

namespace cp {

// Tunables (set through cp_tune; defaults chosen from measurements on MI355X).
struct Tuning {
  uint32_t move_rows_per_item = 0;   // rows of one token a workgroup moves per work item; 0 = all rows
  uint32_t move_blocks_per_cu = 8;   // resident workgroups per compute unit for the row mover
  uint32_t move_nontemporal = 3;     // bit 0: non-temporal loads, bit 1: non-temporal stores
};
Tuning &tuning();

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

// Row mover used by the insert path: for w < *n_items (device count, at most
// max_items) copy all rows of token item_tok[w] of `src` to slot item_slot[w] of
// `pool`.  Items naming a token >= n_src_tokens or a slot >= n_pool_slots are
// skipped and flagged.
int32_t launch_scatter(hipStream_t stream, const void *src, const cp_kv_layout &src_l, uint32_t n_src_tokens,
                       void *pool, const cp_kv_layout &pool_l, uint32_t n_pool_slots, const uint32_t *item_tok,
                       const uint32_t *item_slot, const uint32_t *n_items, uint32_t max_items,
                       uint32_t *status_flags);

// Exclusive prefix sums of span_len[0 .. *n_spans) into span_off[0 .. *n_spans],
// agg = div_up(max_spans, 1024) + 1 words of scratch.
int32_t launch_span_offsets(hipStream_t stream, const uint32_t *span_len, const uint32_t *n_spans, uint32_t max_spans,
                            uint32_t *span_off, uint32_t *agg);

}  // namespace cp

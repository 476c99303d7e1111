/* The boundary from plain C: the header compiles as C99, structs pass by value, and the host-side
 * checks of a few entry points answer as documented.  No GPU is needed: every call here returns
 * before anything is enqueued.  Built and run by tests/test_abi.py. */
#include <stdio.h>

#include "cacheprune.h"

int main(void) {
  static uint64_t keys[32];
  static uint32_t vals[32], out[4];
  cp_table table;
  cp_kv_layout lay;
  table.keys = keys;
  table.vals = vals;
  table.capacity = 32;
  lay.n_layers = 2;
  lay.n_kv_heads = 2;
  lay.head_dim = 64;
  lay.tok_stride = 1024;
  lay.layer_stride = 512;
  lay.kv_stride = 256;
  if (cp_table_capacity_for(131072, 0.85) != 154208) return 1;
  if (cp_scratch_bytes(1000, 1000, 0) == 0 || cp_sat_scratch_bytes(100) == 0) return 2;
  if (cp_probe(NULL, table, NULL, 4, out) != CP_ERR_INVALID_ARG) return 3;   /* no hashes */
  table.capacity = 33;
  if (cp_probe(NULL, table, keys, 4, out) != CP_ERR_INVALID_ARG) return 4;   /* not a multiple of the bucket size */
  if (cp_fill_unmatched(NULL, out, 4, NULL, lay) != CP_ERR_INVALID_ARG) return 5;
  if (cp_probe(NULL, table, keys, 0, out) != CP_OK) return 6;                /* an empty batch is not an error */
  puts("abi ok");
  return 0;
}

/* The hot path from plain C, with device memory from the HIP runtime and nothing else (no Python,
 * no torch): a batch is inserted and then looked up, and what comes back must be what went in.
 *   insert :  cp_hash_segments -> cp_insert_kv
 *   lookup :  cp_hash_segments -> cp_probe -> cp_build_spans -> cp_gather_kv
 * Every non-sensitive token must be served from a slot of its own or of its duplicate, its rows must
 * equal the rows it was stored with, and the rows of sensitive tokens must stay untouched.
 * Built by __graft_entry__.build(), run by tests/test_gpu_c_abi.py.  Exit code 0 = all checks passed. */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "cacheprune.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %d at line %d\n", (int)e_, __LINE__); return 10; } } while (0)
#define CHECK_CP(x) do { int32_t r_ = (x); if (r_ != CP_OK) { printf("cacheprune error %d at line %d\n", (int)r_, __LINE__); return 11; } } while (0)

enum { L = 3, H = 2, D = 64, ROW = H * D * 2, TOKB = L * 2 * ROW, R = 3, N = 3000, S = 4096, CAP = 8192 };

static uint32_t rnd(uint64_t *s) {
  *s = *s * 6364136223846793005ull + 1442695040888963407ull;
  return (uint32_t)(*s >> 33);
}

int main(void) {
  static uint32_t tok[N], off[R + 1] = {0, 1000, 1000, N}, free_slots[S], slot[N], slot_out[N];
  static uint8_t mask[N];
  uint64_t seed = 0xC0FFEE0Cull;
  uint8_t *src = (uint8_t *)malloc((size_t)N * TOKB), *back = (uint8_t *)malloc((size_t)N * TOKB);
  uint32_t i, n_inserted = 0, n_spans = 0, flags = 0, served = 0, sensitive = 0;
  size_t b;
  if (!src || !back) return 12;
  for (i = 0; i < N; ++i) {
    tok[i] = i >= 2000 && i < 2500 ? tok[i - 2000] : rnd(&seed) % 32000;  /* 500 tokens repeat request 0's start */
    mask[i] = rnd(&seed) % 16 == 0;
  }
  for (i = 2000; i < 2500; ++i) mask[i] = mask[i - 2000];                 /* the same text carries the same mask */
  for (i = 0; i < S; ++i) free_slots[i] = S - 1 - i;
  for (b = 0; b < (size_t)N * TOKB; ++b) src[b] = (uint8_t)rnd(&seed);

  uint32_t *d_tok, *d_off, *d_free, *d_slot, *d_slot_out, *d_counts, *d_spans;
  uint8_t *d_mask, *d_src, *d_dst, *d_pool;
  uint64_t *d_hash, *d_keys;
  uint32_t *d_vals;
  int32_t *d_slot_pos;
  void *d_scratch;
  const size_t scratch_bytes = cp_scratch_bytes(N, N, S);
  CHECK_HIP(hipMalloc((void **)&d_tok, sizeof tok));
  CHECK_HIP(hipMalloc((void **)&d_off, sizeof off));
  CHECK_HIP(hipMalloc((void **)&d_free, sizeof free_slots));
  CHECK_HIP(hipMalloc((void **)&d_mask, sizeof mask));
  CHECK_HIP(hipMalloc((void **)&d_slot, sizeof slot));
  CHECK_HIP(hipMalloc((void **)&d_slot_out, sizeof slot_out));
  CHECK_HIP(hipMalloc((void **)&d_counts, 3 * sizeof(uint32_t)));  /* n_inserted, n_spans, status flags */
  CHECK_HIP(hipMalloc((void **)&d_spans, (5 * (size_t)N + 1) * sizeof(uint32_t)));
  CHECK_HIP(hipMalloc((void **)&d_hash, N * sizeof(uint64_t)));
  CHECK_HIP(hipMalloc((void **)&d_keys, CAP * sizeof(uint64_t)));
  CHECK_HIP(hipMalloc((void **)&d_vals, CAP * sizeof(uint32_t)));
  CHECK_HIP(hipMalloc((void **)&d_slot_pos, S * sizeof(int32_t)));
  CHECK_HIP(hipMalloc((void **)&d_src, (size_t)N * TOKB));
  CHECK_HIP(hipMalloc((void **)&d_dst, (size_t)N * TOKB));
  CHECK_HIP(hipMalloc((void **)&d_pool, (size_t)S * TOKB));
  CHECK_HIP(hipMalloc(&d_scratch, scratch_bytes));
  CHECK_HIP(hipMemcpy(d_tok, tok, sizeof tok, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(d_off, off, sizeof off, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(d_free, free_slots, sizeof free_slots, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(d_mask, mask, sizeof mask, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(d_src, src, (size_t)N * TOKB, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemset(d_dst, 0xEE, (size_t)N * TOKB));
  CHECK_HIP(hipMemset(d_counts, 0, 3 * sizeof(uint32_t)));
  CHECK_HIP(hipMemset(d_slot_pos, 0, S * sizeof(int32_t)));

  cp_table table;
  cp_kv_layout pool_l, buf_l;
  table.keys = d_keys, table.vals = d_vals, table.capacity = CAP;
  pool_l.n_layers = buf_l.n_layers = L, pool_l.n_kv_heads = buf_l.n_kv_heads = H, pool_l.head_dim = buf_l.head_dim = D;
  pool_l.tok_stride = TOKB, pool_l.layer_stride = 2 * ROW, pool_l.kv_stride = ROW;                  /* token-major pool */
  buf_l.tok_stride = ROW, buf_l.layer_stride = 2ull * N * ROW, buf_l.kv_stride = (uint64_t)N * ROW; /* layer-major buffers */
  uint32_t *sp_src = d_spans, *sp_dst = d_spans + N, *sp_len = d_spans + 2 * N, *sp_off = d_spans + 4 * N;
  int32_t *sp_delta = (int32_t *)(d_spans + 3 * N);

  CHECK_CP(cp_table_init(NULL, table));
  CHECK_CP(cp_hash_segments(NULL, d_tok, d_mask, d_off, N, R, 0x100000001B3ull, d_hash, d_scratch, scratch_bytes));
  CHECK_CP(cp_insert_kv(NULL, table, d_hash, d_off, N, R, d_free, S, d_src, buf_l, d_pool, pool_l, S, d_slot_pos,
                        d_slot_out, d_counts + 0, d_counts + 2, d_scratch, scratch_bytes, NULL));
  CHECK_CP(cp_probe(NULL, table, d_hash, N, d_slot));
  CHECK_CP(cp_build_spans(NULL, d_slot, d_off, N, R, NULL, N, sp_src, sp_dst, sp_len, sp_delta, sp_off, d_counts + 1,
                          d_counts + 2, d_scratch, scratch_bytes));
  cp_launch_opts opts;  /* explicit options: no sharing of reads, 4 workgroups per unit */
  memset(&opts, 0, sizeof opts);
  opts.read_sharing = 2;
  opts.blocks_per_cu = 4;
  CHECK_CP(cp_gather_kv(NULL, d_pool, pool_l, S, d_dst, buf_l, N, sp_src, sp_dst, sp_len, NULL, sp_off, d_counts + 1, N,
                        NULL, d_counts + 2, d_scratch, scratch_bytes, &opts));
  CHECK_HIP(hipDeviceSynchronize());
  uint32_t counts[3];
  CHECK_HIP(hipMemcpy(counts, d_counts, sizeof counts, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(slot, d_slot, sizeof slot, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(slot_out, d_slot_out, sizeof slot_out, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(back, d_dst, (size_t)N * TOKB, hipMemcpyDeviceToHost));
  n_inserted = counts[0], n_spans = counts[1], flags = counts[2];

  if (flags != 0) { printf("status flags %u\n", flags); return 1; }
  /* a slot belongs to the first token that was given it; later tokens with the same run prefix share it */
  static uint32_t owner[S];
  for (i = 0; i < S; ++i) owner[i] = N;
  for (i = N; i-- > 0;)
    if (slot_out[i] < S) owner[slot_out[i]] = i;
  for (i = 0; i < N; ++i) {
    uint32_t l, kv;
    if (slot[i] != slot_out[i]) { printf("token %u: probe says %u, insert said %u\n", i, slot[i], slot_out[i]); return 2; }
    if (mask[i]) {
      ++sensitive;
      if (slot[i] != CP_SLOT_NONE) { printf("sensitive token %u was served\n", i); return 3; }
    } else {
      ++served;
      if (slot[i] >= S) { printf("token %u not served\n", i); return 4; }
      if (tok[owner[slot[i]]] != tok[i]) { printf("token %u is served another token's slot\n", i); return 7; }
    }
    for (l = 0; l < L; ++l)
      for (kv = 0; kv < 2; ++kv) {
        const size_t plane = (size_t)l * buf_l.layer_stride + kv * buf_l.kv_stride, at = plane + (size_t)i * ROW;
        const uint8_t *want = mask[i] ? NULL : src + plane + (size_t)owner[slot[i]] * ROW;
        size_t k;
        for (k = 0; k < ROW; ++k) {
          const uint8_t w = want ? want[k] : 0xEE;  /* rows of sensitive tokens are never written */
          if (back[at + k] != w) { printf("token %u layer %u kv %u byte %zu: %u, expected %u\n", i, l, kv, k, back[at + k], w); return 5; }
        }
      }
  }
  /* request 2 repeats 500 tokens of request 0 from its start, with the same mask: those runs are stored once */
  if (!(n_inserted < served)) { printf("no duplicate was shared: %u stored, %u served\n", n_inserted, served); return 6; }
  printf("c abi ok: %u tokens, %u sensitive, %u stored, %u spans\n", (unsigned)N, sensitive, n_inserted, n_spans);
  return 0;
}

// cp_verify_chain: exact confirmation of hash matches (Sec. 4.2.2 Step 2, "full verification": a
// candidate found by the rolling hash is confirmed so that no hash collision yields a false match).
//
// The paper confirms a candidate with a cryptographic hash of the substring.  Here every pool slot
// records the token it was stored for and the slot of the token before it in its run
// (slot_tok, slot_parent; CP_SLOT_NONE for the first token of a run), i.e. the stored runs form a
// trie whose nodes are slots.  A request token i at offset k > 0 of its segment is consistent if
//     slot_tok[cand[i]] == tok[i]   and   slot_parent[cand[i]] == cand[i-1],
// at offset 0 if the parent is CP_SLOT_NONE.  If every token from the segment's start through i is
// consistent then, by induction over k, slot cand[i] was stored for exactly the segment's tokens up
// to i: an exact comparison, at O(1) per token.  "Every token so far is consistent" is a segmented
// prefix AND, computed with the ordered scan.
#include "cp_device.h"
#include "cp_internal.h"

namespace cp {
namespace {

struct ChainOp {
  using T = uint32_t;  // bit 0: a token failed since the last segment start; bit 1: the piece holds a segment start
  const uint32_t *tok;
  const uint32_t *seg_off;
  const uint32_t *cand;
  const uint32_t *slot_tok;
  const uint32_t *slot_parent;
  uint32_t *slot_out;
  uint32_t *stream_out;     // nullable: this stream's own result, whatever slot_out already held
  const uint32_t *trusted;  // nullable: trusted[i] != NONE = the caller has confirmed cand[i] already
  uint32_t N, n_pool_slots, merge;

  static __device__ __forceinline__ T identity() { return 0u; }
  static __device__ __forceinline__ T combine(T f, T g) { return (g & 2u) ? g : (f | g); }
  __device__ __forceinline__ uint32_t count() const { return N; }
  __device__ __forceinline__ T load(uint32_t i) const {
    const uint32_t k = seg_off[i];
    if (k == 0xFFFFFFFFu) return 3u;  // in no segment: fails, and nothing carries over it
    if (trusted && trusted[i] != CP_SLOT_NONE) return 2u;  // confirmed elsewhere: passes, whatever came before it
    const uint32_t s = cand[i];
    bool ok = s < n_pool_slots;
    uint32_t want_parent = CP_SLOT_NONE;
    if (k != 0) {
      ok = ok && i != 0 && seg_off[i - 1] == k - 1;  // offsets must count up along the segment
      want_parent = ok ? cand[i - 1] : CP_SLOT_NONE;
      ok = ok && want_parent < n_pool_slots;
    }
    ok = ok && slot_tok[s] == tok[i] && slot_parent[s] == want_parent;
    return (ok ? 0u : 1u) | (k == 0 ? 2u : 0u);
  }
  __device__ __forceinline__ void store(uint32_t i, T, T incl) const {
    const uint32_t r = (incl & 1u) ? CP_SLOT_NONE : cand[i];
    if (!merge || slot_out[i] == CP_SLOT_NONE) slot_out[i] = r;
    if (stream_out) stream_out[i] = r;
  }
  __device__ __forceinline__ void finish(T) const {}
};

// The three key streams of a lookup with floating anchors (run-start keys, candidate stream a, candidate stream
// b) confirmed in one scan: two bits per stream, each stream's prefix AND independent of the others.  A token
// is served from the first stream that accepts it.
struct ChainOp3 {
  using T = uint32_t;  // bits 2s, 2s+1: stream s's "failed since the segment start" and "holds a segment start"
  const uint32_t *tok;
  const uint32_t *seg_off[3];
  const uint32_t *cand[3];
  const uint32_t *slot_tok;
  const uint32_t *slot_parent;
  uint32_t *slot_out;
  uint32_t *stream_out[3];  // nullable, each
  uint32_t N, n_pool_slots;

  static __device__ __forceinline__ T identity() { return 0u; }
  static __device__ __forceinline__ T combine(T f, T g) {
    const uint32_t starts = (g >> 1) & 0x15u;           // bit 2s set where g's stream s holds a segment start
    return g | (f & ~(starts | (starts << 1)) & 0x3Fu);  // there g stands alone, elsewhere the failures add up
  }
  __device__ __forceinline__ uint32_t count() const { return N; }
  __device__ __forceinline__ T one(uint32_t s, uint32_t i) const {
    const uint32_t k = seg_off[s][i];
    if (k == 0xFFFFFFFFu) return 3u;  // in no segment: fails, and nothing carries over it
    const uint32_t c = cand[s][i];
    bool ok = c < n_pool_slots;
    uint32_t want_parent = CP_SLOT_NONE;
    if (k != 0) {
      ok = ok && i != 0 && seg_off[s][i - 1] == k - 1;  // offsets must count up along the segment
      want_parent = ok ? cand[s][i - 1] : CP_SLOT_NONE;
      ok = ok && want_parent < n_pool_slots;
    }
    ok = ok && slot_tok[c] == tok[i] && slot_parent[c] == want_parent;
    return (ok ? 0u : 1u) | (k == 0 ? 2u : 0u);
  }
  __device__ __forceinline__ T load(uint32_t i) const { return one(0, i) | (one(1, i) << 2) | (one(2, i) << 4); }
  __device__ __forceinline__ void store(uint32_t i, T, T incl) const {
    uint32_t served = CP_SLOT_NONE;
#pragma unroll
    for (int s = 2; s >= 0; --s) {
      const uint32_t r = ((incl >> (2 * s)) & 1u) ? CP_SLOT_NONE : cand[s][i];
      if (stream_out[s]) stream_out[s][i] = r;
      if (r != CP_SLOT_NONE) served = r;  // the earliest stream that accepts the token wins
    }
    slot_out[i] = served;
  }
  __device__ __forceinline__ void finish(T) const {}
};

}  // namespace

int32_t launch_chain_verify(hipStream_t stream, const uint32_t *tok, const uint32_t *seg_off, const uint32_t *cand,
                            uint32_t N, const uint32_t *slot_tok, const uint32_t *slot_parent, uint32_t n_pool_slots,
                            uint32_t merge, uint32_t *slot_out, uint32_t *stream_out, uint32_t *agg,
                            const uint32_t *trusted) {
  ChainOp op{tok, seg_off, cand, slot_tok, slot_parent, slot_out, stream_out, trusted, N, n_pool_slots, merge};
  return run_scan<ChainOp>(stream, op, N, agg);
}

}  // namespace cp

extern "C" int32_t cp_verify_chain(void *stream, const uint32_t *tok, const uint32_t *seg_off, const uint32_t *cand,
                                   uint32_t N, const uint32_t *slot_tok, const uint32_t *slot_parent,
                                   uint32_t n_pool_slots, int32_t merge, uint32_t *slot_out, uint32_t *stream_out,
                                   void *scratch, size_t scratch_bytes) {
  using namespace cp;
  if (N == 0) return CP_OK;
  if (N >= 0x80000000u || n_pool_slots >= 0x80000000u) return CP_ERR_UNSUPPORTED;
  if (!tok || !seg_off || !cand || !slot_tok || !slot_parent || !slot_out || !scratch || !aligned(scratch, 256))
    return CP_ERR_INVALID_ARG;
  if (cand == slot_out || cand == stream_out) return CP_ERR_INVALID_ARG;  // neighbours read cand while results are written
  if (scratch_bytes < cp_scratch_bytes(N, 0, 0)) return CP_ERR_SCRATCH;
  Scratch sc(scratch, scratch_bytes);
  uint32_t *agg = sc.take<uint32_t>(div_up(N, kScanTile) + 1);
  if (!agg) return CP_ERR_SCRATCH;
  return launch_chain_verify((hipStream_t)stream, tok, seg_off, cand, N, slot_tok, slot_parent, n_pool_slots,
                             merge ? 1u : 0u, slot_out, stream_out, agg, nullptr);
}

extern "C" int32_t cp_verify_streams(void *stream_, cp_table table, const uint32_t *tok, uint32_t N,
                                     const uint32_t *seg_off_0, const uint32_t *cand_0, const uint64_t *key_a,
                                     const uint32_t *seg_off_a, const uint64_t *key_b, const uint32_t *seg_off_b,
                                     const uint32_t *slot_tok, const uint32_t *slot_parent, uint32_t n_pool_slots,
                                     uint32_t *slot_out, uint32_t *stream_out_0, uint32_t *stream_out_a,
                                     uint32_t *stream_out_b, void *scratch, size_t scratch_bytes) {
  using namespace cp;
  hipStream_t stream = (hipStream_t)stream_;
  if (N == 0) return CP_OK;
  if (N >= 0x80000000u || n_pool_slots >= 0x80000000u) return CP_ERR_UNSUPPORTED;
  if (!tok || !seg_off_0 || !cand_0 || !key_a || !seg_off_a || !key_b || !seg_off_b || !slot_tok || !slot_parent ||
      !slot_out || !scratch || !aligned(scratch, 256) || !aligned(key_a, 8) || !aligned(key_b, 8))
    return CP_ERR_INVALID_ARG;
  if (cand_0 == slot_out || cand_0 == stream_out_0 || cand_0 == stream_out_a || cand_0 == stream_out_b)
    return CP_ERR_INVALID_ARG;  // neighbours read cand while results are written
  if (scratch_bytes < cp_scratch_bytes(N, 0, 0)) return CP_ERR_SCRATCH;
  Scratch sc(scratch, scratch_bytes);
  uint32_t *agg = sc.take<uint32_t>(div_up(N, kScanTile) + 1);
  uint32_t *cand_a = sc.take<uint32_t>(N);
  uint32_t *cand_b = sc.take<uint32_t>(N);
  if (!agg || !cand_a || !cand_b) return CP_ERR_SCRATCH;
  if (int32_t rc = launch_probe_each(stream, table, key_a, key_b, N, cand_a, cand_b)) return rc;
  ChainOp3 op{tok, {seg_off_0, seg_off_a, seg_off_b}, {cand_0, cand_a, cand_b}, slot_tok, slot_parent, slot_out,
              {stream_out_0, stream_out_a, stream_out_b}, N, n_pool_slots};
  return run_scan<ChainOp3>(stream, op, N, agg);
}

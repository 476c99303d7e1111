// cp_hash_segments / cp_hash_runs: segmented polynomial chain hash (Sec. 4.2.1
// segmentation by sensitive tokens, Sec. 4.2.2 polynomial rolling hash; modulus
// 2^64), and cp_hash_floating: the keys of the floating-anchor lookup (Sec. 4.2.2
// Step 1, sliding window against stored prefix hashes; Step 2, O(1) substring
// hash from prefix hashes and a power of the base).
//
// The recurrence  c <- c * base + (tok + 1)  is the affine map x -> x*m + a with
// (m, a) = (base, tok + 1).  Affine maps compose associatively,
//   (m1, a1) then (m2, a2)  =  (m1*m2, a1*m2 + a2),
// so the chain value of every token is an ordered scan over that monoid.  A
// chain restart (sensitive token, request start) is the map with m = 0, which
// forgets everything before it, so the hash needs no separate segment flags.
// The same scan counts the tokens of the run so far (restart flag + length).
#include "cp_device.h"
#include "cp_internal.h"

namespace cp {
namespace {

struct HashOp {
  struct T {
    uint64_t m, a;
    uint32_t len, reset;  // tokens of the current run in this piece; does the piece contain a restart
  };
  const uint32_t *tok;
  const uint8_t *mask;
  const uint32_t *off;
  uint64_t *out;
  uint32_t *run_off;  // nullable
  uint64_t base;
  uint32_t N, R;

  static __device__ __forceinline__ T identity() { return T{1ull, 0ull, 0u, 0u}; }
  static __device__ __forceinline__ T combine(T f, T g) {
    return T{f.m * g.m, f.a * g.m + g.a, g.reset ? g.len : f.len + g.len, f.reset | g.reset};
  }
  __device__ __forceinline__ uint32_t count() const { return N; }
  __device__ __forceinline__ T load(uint32_t i) const {
    if (mask[i]) return T{0ull, 0ull, 0u, 1u};  // value after a sensitive token is 0: the next token starts a run
    bool start = off[request_of(off, R, i)] == i;
    return T{start ? 0ull : base, (uint64_t)tok[i] + 1ull, 1u, start ? 1u : 0u};
  }
  __device__ __forceinline__ void store(uint32_t i, T, T incl) const {
    uint64_t h = incl.a;  // the composed map applied to the initial value 0
    if (h == CP_HASH_NONE) h = CP_HASH_NONE - 1;
    const bool sensitive = mask[i] != 0;
    out[i] = sensitive ? CP_HASH_NONE : h;
    if (run_off) run_off[i] = sensitive ? 0xFFFFFFFFu : incl.len - 1;
  }
  __device__ __forceinline__ void finish(T) const {}
};

__device__ __forceinline__ uint64_t pow_u64(uint64_t b, uint32_t k) {  // b^k mod 2^64
  uint64_t r = 1;
  while (k) {
    if (k & 1) r *= b;
    b *= b;
    k >>= 1;
  }
  return r;
}

// Latest floating anchor at or before every token: a plain running maximum of (position + 1) over
// the anchor flags; whether that anchor lies in the token's own run is checked when storing.
struct FloatKeyOp {
  using T = uint32_t;
  const uint64_t *hash;
  const uint32_t *run_off;
  const uint8_t *hit;  // hit[i]: the W-token window ending at i matches a stored prefix hash
  uint64_t *out;
  uint32_t *float_off;  // nullable: i - a for tokens with an anchor, else 0xFFFFFFFF
  uint64_t base;
  uint32_t N, W;

  static __device__ __forceinline__ T identity() { return 0u; }
  static __device__ __forceinline__ T combine(T a, T b) { return a > b ? a : b; }
  __device__ __forceinline__ uint32_t count() const { return N; }
  __device__ __forceinline__ T load(uint32_t a) const {
    const uint64_t end = (uint64_t)a + W - 1;  // last token of the window that starts at a
    return (end < N && hit[end]) ? a + 1 : 0u;
  }
  __device__ __forceinline__ void store(uint32_t i, T, T incl) const {
    uint64_t key = CP_HASH_NONE;
    uint32_t fo = 0xFFFFFFFFu;
    const uint32_t ro = run_off[i];
    if (hash[i] != CP_HASH_NONE && incl != 0) {
      const uint32_t a = incl - 1;
      if (a > i - ro) {  // inside this run and after its start (a window at the run start is the plain key)
        key = hash[i] - hash[a - 1] * pow_u64(base, i - a + 1);
        if (key == CP_HASH_NONE) key = CP_HASH_NONE - 1;
        fo = i - a;
      }
    }
    out[i] = key;
    if (float_off) float_off[i] = fo;
  }
  __device__ __forceinline__ void finish(T) const {}
};

}  // namespace
}  // namespace cp

static int32_t hash_common(void *stream, const uint32_t *tok, const uint8_t *mask, const uint32_t *off, uint32_t N,
                           uint32_t R, uint64_t base, uint64_t *hash_out, uint32_t *run_off_out, void *scratch,
                           size_t scratch_bytes) {
  using namespace cp;
  if (N == 0) return CP_OK;
  if (N >= 0x80000000u) return CP_ERR_UNSUPPORTED;
  if (!tok || !mask || !off || !hash_out || !scratch || R == 0) return CP_ERR_INVALID_ARG;
  if (!aligned(tok, 4) || !aligned(off, 4) || !aligned(hash_out, 8) || !aligned(scratch, 256))
    return CP_ERR_INVALID_ARG;
  if (scratch_bytes < cp_scratch_bytes(N, 0, 0)) return CP_ERR_SCRATCH;
  Scratch sc(scratch, scratch_bytes);
  HashOp::T *agg = sc.take<HashOp::T>(div_up(N, kScanTile) + 1);
  if (!agg) return CP_ERR_SCRATCH;
  HashOp op{tok, mask, off, hash_out, run_off_out, base, N, R};
  return run_scan<HashOp>((hipStream_t)stream, op, N, agg);
}

extern "C" int32_t cp_hash_segments(void *stream, const uint32_t *tok, const uint8_t *mask, const uint32_t *off,
                                    uint32_t N, uint32_t R, uint64_t base, uint64_t *hash_out, void *scratch,
                                    size_t scratch_bytes) {
  return hash_common(stream, tok, mask, off, N, R, base, hash_out, nullptr, scratch, scratch_bytes);
}

extern "C" int32_t cp_hash_runs(void *stream, const uint32_t *tok, const uint8_t *mask, const uint32_t *off,
                                uint32_t N, uint32_t R, uint64_t base, uint64_t *hash_out, uint32_t *run_off_out,
                                void *scratch, size_t scratch_bytes) {
  if (N && !run_off_out) return CP_ERR_INVALID_ARG;
  return hash_common(stream, tok, mask, off, N, R, base, hash_out, run_off_out, scratch, scratch_bytes);
}

extern "C" int32_t cp_hash_floating(void *stream_, cp_table table, const uint8_t *slot_anchor, uint32_t n_pool_slots,
                                    const uint64_t *hash, const uint32_t *run_off, uint32_t N, uint64_t base,
                                    uint32_t W, uint64_t *hash_float_out, uint32_t *float_off_out, void *scratch,
                                    size_t scratch_bytes) {
  using namespace cp;
  hipStream_t stream = (hipStream_t)stream_;
  if (N == 0) return CP_OK;
  if (N >= 0x80000000u) return CP_ERR_UNSUPPORTED;
  if (n_pool_slots >= 0x80000000u) return CP_ERR_UNSUPPORTED;
  if (W == 0 || !slot_anchor || !hash || !run_off || !hash_float_out || !scratch || !aligned(scratch, 256) ||
      !aligned(hash, 8) || !aligned(hash_float_out, 8))
    return CP_ERR_INVALID_ARG;
  if (scratch_bytes < cp_scratch_bytes(N, 0, 0)) return CP_ERR_SCRATCH;
  Scratch sc(scratch, scratch_bytes);
  uint32_t *agg = sc.take<uint32_t>(div_up(N, kScanTile) + 1);
  uint8_t *hit = sc.take<uint8_t>(N);
  if (!agg || !hit) return CP_ERR_SCRATCH;
  uint64_t pw = 1;  // base^W mod 2^64
  for (uint64_t b = base, k = W; k; k >>= 1, b *= b)
    if (k & 1) pw *= b;
  if (int32_t rc = launch_window_hits(stream, table, slot_anchor, n_pool_slots, hash, run_off, N, W, pw, hit)) return rc;
  FloatKeyOp op{hash, run_off, hit, hash_float_out, float_off_out, base, N, W};
  return run_scan<FloatKeyOp>(stream, op, N, agg);
}

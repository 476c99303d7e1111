// cp_hash_segments: segmented polynomial chain hash (Sec. 4.2.1 segmentation by
// sensitive tokens, Sec. 4.2.2 polynomial rolling hash; modulus 2^64).
//
// The recurrence  c <- c * base + (tok + 1)  is the affine map x -> x*m + a with
// (m, a) = (base, tok + 1).  Affine maps compose associatively,
//   (m1, a1) then (m2, a2)  =  (m1*m2, a1*m2 + a2),
// so the chain value of every token is an ordered scan over that monoid.  A
// chain restart (sensitive token, request start) is the map with m = 0, which
// forgets everything before it, so no separate segment flags are needed.
#include "cp_device.h"

namespace cp {
namespace {

struct HashOp {
  struct T { uint64_t m, a; };
  const uint32_t *tok;
  const uint8_t *mask;
  const uint32_t *off;
  uint64_t *out;
  uint64_t base;
  uint32_t N, R;

  static __device__ __forceinline__ T identity() { return T{1ull, 0ull}; }
  static __device__ __forceinline__ T combine(T f, T g) { return T{f.m * g.m, f.a * g.m + g.a}; }
  __device__ __forceinline__ uint32_t count() const { return N; }
  __device__ __forceinline__ T load(uint32_t i) const {
    if (mask[i]) return T{0ull, 0ull};  // value after a sensitive token is 0: the next token starts a run
    bool start = off[request_of(off, R, i)] == i;
    return T{start ? 0ull : base, (uint64_t)tok[i] + 1ull};
  }
  __device__ __forceinline__ void store(uint32_t i, T, T incl) const {
    uint64_t h = incl.a;  // the composed map applied to the initial value 0
    if (h == CP_HASH_NONE) h = CP_HASH_NONE - 1;
    out[i] = mask[i] ? CP_HASH_NONE : h;
  }
  __device__ __forceinline__ void finish(T) const {}
};

}  // namespace
}  // namespace cp

extern "C" int32_t cp_hash_segments(void *stream, const uint32_t *tok, const uint8_t *mask,
                                    const uint32_t *off, uint32_t N, uint32_t R, uint64_t base,
                                    uint64_t *hash_out, void *scratch, size_t scratch_bytes) {
  using namespace cp;
  if (N == 0) return CP_OK;
  if (N >= 0x80000000u) return CP_ERR_UNSUPPORTED;
  if (!tok || !mask || !off || !hash_out || !scratch || R == 0) return CP_ERR_INVALID_ARG;
  if (!aligned(tok, 4) || !aligned(off, 4) || !aligned(hash_out, 8) || !aligned(scratch, 16))
    return CP_ERR_INVALID_ARG;
  if (scratch_bytes < cp_scratch_bytes(N, 0, 0)) return CP_ERR_SCRATCH;
  HashOp op{tok, mask, off, hash_out, base, N, R};
  return run_scan<HashOp>((hipStream_t)stream, op, N, (HashOp::T *)scratch);
}

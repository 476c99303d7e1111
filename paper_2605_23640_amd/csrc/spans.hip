// cp_build_spans: run-length pass from per-token pool slots to copy
// descriptors (the "token spans" the retriever keeps as metadata, Sec. 4.3.1).
//
// Token i opens a span ("head") when its slot is valid and it does not continue
// its left neighbour (same request, neighbour's slot + 1, same position delta).
// An ordered scan carries (number of heads so far, index of the latest head,
// number of tokens with a slot so far): the head count gives every span its
// output index, so spans come out in (request, position) order, the latest-head
// index lets the last token of a span write the span's length, and the token
// count before a head is the number of tokens the earlier spans cover (span_off).
#include "cp_device.h"
#include "cp_internal.h"

namespace cp {
namespace {

struct SpanOp {
  struct T { uint32_t heads, last, covered; };  // last = 1 + index of the latest head, 0 if none; covered = tokens in spans
  const uint32_t *slot;
  const uint32_t *off;
  const int32_t *slot_pos;  // nullable
  uint32_t *span_src, *span_dst, *span_len, *span_off;
  int32_t *span_delta;  // nullable
  uint32_t *n_spans, *status_flags;
  uint32_t N, R, max_spans;

  static __device__ __forceinline__ T identity() { return T{0u, 0u, 0u}; }
  static __device__ __forceinline__ T combine(T a, T b) {
    return T{a.heads + b.heads, b.last ? b.last : a.last, a.covered + b.covered};
  }
  __device__ __forceinline__ uint32_t count() const { return N; }

  // Does token i (valid slot s, i > 0) continue the span of token i - 1?
  __device__ __forceinline__ bool continues(uint32_t i, uint32_t s) const {
    uint32_t sp = slot[i - 1];
    if (sp == CP_SLOT_NONE || sp + 1 != s) return false;
    if (off[request_of(off, R, i)] == i) return false;  // i starts a request
    // same request, so the positions differ by one: equal deltas <=> cached positions differ by one
    if (slot_pos && slot_pos[s] - slot_pos[sp] != 1) return false;
    return true;
  }
  __device__ __forceinline__ bool is_head(uint32_t i) const {
    uint32_t s = slot[i];
    if (s == CP_SLOT_NONE) return false;
    return i == 0 || !continues(i, s);
  }
  __device__ __forceinline__ T load(uint32_t i) const {
    if (slot[i] == CP_SLOT_NONE) return T{0u, 0u, 0u};
    return is_head(i) ? T{1u, i + 1, 1u} : T{0u, 0u, 1u};
  }
  __device__ __forceinline__ void store(uint32_t i, T excl, T incl) const {
    uint32_t s = slot[i];
    if (s == CP_SLOT_NONE) return;
    uint32_t k = incl.heads - 1, head = incl.last - 1;  // a valid token always lies in a span
    // tokens that the spans before span k cover; for the first span that is dropped: what the kept ones cover
    if (span_off && head == i && k <= max_spans) span_off[k] = excl.covered;
    if (k >= max_spans) return;
    if (head == i) {
      span_src[k] = s;
      span_dst[k] = i;
      if (span_delta) {
        int32_t p = (int32_t)(i - off[request_of(off, R, i)]);
        span_delta[k] = slot_pos ? p - slot_pos[s] : 0;
      }
    }
    bool last = (i + 1 == N);
    if (!last) {
      uint32_t sn = slot[i + 1];
      last = sn == CP_SLOT_NONE || !continues(i + 1, sn);
    }
    if (last) span_len[k] = i - head + 1;
  }
  __device__ __forceinline__ void finish(T total) const {
    *n_spans = total.heads < max_spans ? total.heads : max_spans;
    if (total.heads > max_spans) atomicOr(status_flags, CP_FLAG_SPANS_OVERFLOW);
    else if (span_off) span_off[total.heads] = total.covered;  // (on overflow the first dropped span wrote it)
  }
};

// Exclusive prefix sums of the span lengths (the number of tokens before each span).
struct SpanOffOp {
  using T = uint32_t;
  const uint32_t *span_len;
  const uint32_t *n_spans;
  uint32_t *span_off;
  uint32_t max_spans;
  static __device__ __forceinline__ T identity() { return 0; }
  static __device__ __forceinline__ T combine(T a, T b) { return a + b; }
  __device__ __forceinline__ uint32_t count() const {
    uint32_t n = *n_spans;
    return n < max_spans ? n : max_spans;
  }
  __device__ __forceinline__ T load(uint32_t i) const { return span_len[i]; }
  __device__ __forceinline__ void store(uint32_t i, T excl, T) const { span_off[i] = excl; }
  __device__ __forceinline__ void finish(T total) const { span_off[count()] = total; }
};

}  // namespace

int32_t launch_span_offsets(hipStream_t stream, const uint32_t *span_len, const uint32_t *n_spans, uint32_t max_spans,
                            uint32_t *span_off, uint32_t *agg) {
  SpanOffOp op{span_len, n_spans, span_off, max_spans};
  return run_scan<SpanOffOp>(stream, op, max_spans, agg);
}

}  // namespace cp

extern "C" int32_t cp_build_spans(void *stream_, const uint32_t *slot, const uint32_t *off, uint32_t N, uint32_t R,
                                  const int32_t *slot_pos, uint32_t max_spans, uint32_t *span_src, uint32_t *span_dst,
                                  uint32_t *span_len, int32_t *span_delta, uint32_t *span_off, uint32_t *n_spans,
                                  uint32_t *status_flags, void *scratch, size_t scratch_bytes) {
  using namespace cp;
  hipStream_t stream = (hipStream_t)stream_;
  if (N >= 0x80000000u) return CP_ERR_UNSUPPORTED;
  if (!n_spans || !status_flags || !scratch || !aligned(scratch, 256)) return CP_ERR_INVALID_ARG;
  if (N && (!slot || !off || R == 0)) return CP_ERR_INVALID_ARG;
  if (max_spans && (!span_src || !span_dst || !span_len)) return CP_ERR_INVALID_ARG;
  if (scratch_bytes < cp_scratch_bytes(N, max_spans, 0)) return CP_ERR_SCRATCH;
  Scratch sc(scratch, scratch_bytes);
  uint32_t tiles = div_up(N > max_spans ? N : max_spans, kScanTile) + 1;
  SpanOp::T *agg = sc.take<SpanOp::T>(tiles);
  if (!agg) return CP_ERR_SCRATCH;
  SpanOp op{slot, off, slot_pos, span_src, span_dst, span_len, span_off, span_delta, n_spans, status_flags, N, R, max_spans};
  return run_scan<SpanOp>(stream, op, N, agg);
}

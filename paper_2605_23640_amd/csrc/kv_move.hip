// Token-granular KV row mover: cp_gather_kv (pool -> request buffers, with
// optional key re-rotation) and the scatter half of cp_insert_kv (request
// buffers -> pool).  "Linking" matched segments into the request (Sec. 4.1 KV
// Retriever, Sec. 4.3.1) becomes a copy of every matched token's K and V rows;
// positions that no span covers are never written.
//
// This is the HBM-bound part of the path: every matched token needs
// 2 * n_layers * row_bytes bytes written, and the same amount read unless
// several requests of the batch reuse the same pool slot (a shared system
// prompt, a retrieved passage used twice).  Design:
//   - spans are first expanded into one 16-byte descriptor per token
//     (source slot, destination token, position delta, link), so the mover
//     never searches;
//   - tokens that read the same pool slot are linked into a chain while being
//     expanded (one atomic exchange per token on a per-slot head word); the
//     token that ends up as head of a chain moves the rows for the whole chain:
//     each 16-byte piece is loaded once and stored to every destination
//     ("read once, write many").  The order inside a chain depends on timing,
//     the bytes written do not;
//   - work items (chains) are handed to workgroups through an atomic counter,
//     so long chains and single tokens balance; every workgroup leaves the loop
//     as soon as the counter passes the item count;
//   - inside an item the 256 lanes walk the (row, 16-byte column) space in
//     row-major order, so every wavefront touches whole contiguous 1 KiB pieces,
//     several loads are issued before the first store, and both directions can
//     be non-temporal (nothing is read back by this kernel).
// Key re-rotation (textbook RoPE, not in the paper) is done in double precision
// on the way through registers: cos/sin of delta * inv_freq[j] are computed once
// per destination into LDS, the partner element of a pair comes from the
// neighbouring lane (half-split style) or from the same 16 bytes (interleaved).
#include "cp_device.h"
#include "cp_internal.h"

#include <cmath>

namespace cp {

Tuning &tuning() {
  static Tuning t;
  return t;
}

int32_t &last_hip_error() {
  static thread_local int32_t e = 0;
  return e;
}

bool layout_ok(const cp_kv_layout &l) {
  uint64_t row = (uint64_t)l.n_kv_heads * l.head_dim * 2;
  if (l.n_layers == 0 || l.n_kv_heads == 0 || l.head_dim == 0) return false;
  if (row % 16 || row > (1u << 20) || l.n_layers > (1u << 15)) return false;
  if (l.tok_stride % 16 || l.layer_stride % 16 || l.kv_stride % 16) return false;
  return true;
}

bool layouts_match(const cp_kv_layout &a, const cp_kv_layout &b) {
  return a.n_layers == b.n_layers && a.n_kv_heads == b.n_kv_heads && a.head_dim == b.head_dim;
}

namespace {

constexpr int kMoveThreads = 256;
constexpr uint32_t kMaxHalfDim = 256;    // head_dim <= 512 when rotating
constexpr uint32_t kMaxFanout = 16;      // destinations served per pass over the source rows
constexpr uint32_t kTrigDoubles = 2048;  // LDS doubles for cos (and as many for sin): fan-out * head_dim/2 <= this
constexpr uint32_t kNone = 0xFFFFFFFFu;

struct RopeArg {
  uint32_t style, head_dim;
  double inv_freq[kMaxHalfDim];  // theta^(-2j/head_dim), evaluated on the host
};
struct NoRope {  // stand-in for kernels that never rotate: keeps their argument block small
  uint32_t style, head_dim;
  double inv_freq[1];
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <bool NT>
__device__ __forceinline__ u32x4 load16(const uint8_t *p) {
  if (NT) return __builtin_nontemporal_load((const u32x4 *)p);
  return *(const u32x4 *)p;
}
template <bool NT>
__device__ __forceinline__ void store16(uint8_t *p, u32x4 v) {
  if (NT) __builtin_nontemporal_store(v, (u32x4 *)p);
  else *(u32x4 *)p = v;
}

__device__ __forceinline__ double bf16_to_f64(uint32_t b) { return (double)__uint_as_float(b << 16); }

// double -> bf16 bits, one rounding to nearest, ties to even.
__device__ __forceinline__ uint32_t f64_to_bf16(double x) {
  const uint64_t u = (uint64_t)__double_as_longlong(x);
  const uint32_t hi = (uint32_t)(u >> 32), lo = (uint32_t)u;
  // keep sign(1) exponent(11) mantissa(7): round the bit pattern at bit 13 of the high word
  uint32_t t = hi + 0xFFFu + (((hi >> 13) & 1u) | (lo != 0u));
  uint32_t top = t >> 13;
  int32_t e = (int32_t)((top >> 7) & 0x7FFu) - 896;  // re-bias 1023 -> 127
  if (e >= 1 && e <= 254) return ((top >> 18) << 15) | ((uint32_t)e << 7) | (top & 0x7Fu);
  // zero, bf16-subnormal, overflow, inf, nan: go through float with a sticky bit (round to odd)
  if (x != x) return 0x7FC0u;
  float f = (float)x;
  uint32_t b = __float_as_uint(f);
  double back = (double)f;
  if (back != x) {
    if (fabs(back) > fabs(x)) b -= 1u;  // undo a rounding away from zero
    b |= 1u;
  }
  b += 0x7FFFu + ((b >> 16) & 1u);
  return b >> 16;
}

// Rotate the 8 bf16 values of one 16-byte vector.  `own` holds this lane's
// values, `par` the partner values (half-split) — unused for interleaved.
// cs points at cos[0..half), sn at sin[0..half) in LDS.
__device__ __forceinline__ u32x4 rotate_vec(u32x4 own, u32x4 par, uint32_t col_in_head, uint32_t style, uint32_t half,
                                            const double *cs, const double *sn) {
  u32x4 out;
  if (style == 0) {
    const uint32_t vec_per_half = half / 8;
    const bool second = col_in_head >= vec_per_half;
    const uint32_t j0 = (second ? col_in_head - vec_per_half : col_in_head) * 8;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      uint32_t r = 0;
#pragma unroll
      for (int hlf = 0; hlf < 2; ++hlf) {
        uint32_t j = j0 + 2 * w + hlf;
        double a = bf16_to_f64((own[w] >> (16 * hlf)) & 0xFFFFu);
        double b = bf16_to_f64((par[w] >> (16 * hlf)) & 0xFFFFu);
        double c = cs[j], s = sn[j];
        // first half:  a*c - b*s   (b is the second-half partner)
        // second half: a*c + b*s   (b is the first-half partner)
        double y = second ? fma(a, c, b * s) : fma(a, c, -(b * s));
        r |= f64_to_bf16(y) << (16 * hlf);
      }
      out[w] = r;
    }
  } else {
    const uint32_t j0 = col_in_head * 4;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      double a = bf16_to_f64(own[w] & 0xFFFFu), b = bf16_to_f64(own[w] >> 16);
      double c = cs[j0 + w], s = sn[j0 + w];
      out[w] = f64_to_bf16(fma(a, c, -(b * s))) | (f64_to_bf16(fma(b, c, a * s)) << 16);
    }
  }
  return out;
}

// ---- gather front end: clear the per-slot chain heads, expand spans, link chains -------------

__global__ __launch_bounds__(256) void gather_init_kernel(uint32_t *__restrict__ head, uint32_t n_head,
                                                          uint32_t *__restrict__ counter) {
  uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_head) head[i] = kNone;
  if (i == 0) *counter = 0;
}

// One thread per token of the concatenated spans.
__global__ __launch_bounds__(256) void gather_expand_kernel(
    const uint32_t *__restrict__ span_src, const uint32_t *__restrict__ span_dst,
    const uint32_t *__restrict__ span_off, const int32_t *__restrict__ span_delta, const uint32_t *__restrict__ n_spans,
    uint32_t max_spans, uint32_t n_pool_slots, uint32_t n_dst_tokens, MoveItem *__restrict__ items,
    uint32_t *__restrict__ head /* nullable: no grouping */, uint32_t *__restrict__ n_items,
    uint32_t *__restrict__ status_flags) {
  uint32_t n = *n_spans;
  if (n > max_spans) n = max_spans;
  uint32_t total = span_off[n];
  if (total > n_dst_tokens) total = n_dst_tokens;  // spans that do not overlap cannot cover more
  const uint32_t w = blockIdx.x * blockDim.x + threadIdx.x;
  if (w == 0) *n_items = total;
  if (w >= total) return;
  uint32_t lo = 0, hi = n;  // invariant: span_off[lo] <= w < span_off[hi]
  while (hi - lo > 1) {
    uint32_t mid = (lo + hi) >> 1;
    if (span_off[mid] <= w) lo = mid; else hi = mid;
  }
  const uint32_t k = w - span_off[lo];
  MoveItem it{span_src[lo] + k, span_dst[lo] + k, span_delta ? span_delta[lo] : 0, kNone};
  if (it.from >= n_pool_slots || it.to >= n_dst_tokens) {
    atomicOr(status_flags, CP_FLAG_BAD_INDEX);
    it.from = it.to = kNone;  // the mover skips it
  } else if (head) {
    it.next = atomicExch(&head[it.from], w);  // push onto the chain of tokens that read this slot
  }
  items[w] = it;
}

// ---- the mover ---------------------------------------------------------------------------------

template <class RA, bool ROPE, bool NTL, bool NTS, int U>
__device__ __forceinline__ void move_rows_body(
    const MoveItem *__restrict__ items, const uint32_t *__restrict__ n_items_ptr, uint32_t max_items,
    const uint32_t *__restrict__ head /* nullable: every item is its own chain */, uint32_t *counter,
    const uint8_t *__restrict__ from, const cp_kv_layout &fl, uint32_t n_from, uint8_t *__restrict__ to,
    const cp_kv_layout &tl, uint32_t n_to, uint32_t fanout, uint32_t *status_flags, const RA &rope) {
  __shared__ uint32_t s_next_w;     // next work item of this workgroup
  __shared__ uint32_t s_k, s_more;  // destinations in this pass; chain node to continue with
  __shared__ uint32_t s_to[kMaxFanout];
  __shared__ int32_t s_delta[kMaxFanout];
  __shared__ double s_cos[ROPE ? kTrigDoubles : 1], s_sin[ROPE ? kTrigDoubles : 1];

  uint32_t n_items = *n_items_ptr;
  if (n_items > max_items) n_items = max_items;
  const uint32_t n_rows = fl.n_layers * 2;
  const uint32_t vpr = fl.n_kv_heads * fl.head_dim / 8;  // 16-byte vectors per row
  // lane t starts at vector t of the token and advances by 256 vectors per step
  const uint32_t r_step = kMoveThreads / vpr, c_step = kMoveThreads % vpr;
  const uint32_t r_init = threadIdx.x / vpr, c_init = threadIdx.x % vpr;
  const uint32_t vph = fl.head_dim / 8;  // vectors per head
  const uint32_t half = fl.head_dim / 2;
  const uint32_t steps = (n_rows * vpr + kMoveThreads - 1) / kMoveThreads;  // same for every lane

  if (threadIdx.x == 0) s_next_w = atomicAdd(counter, 1u);
  __syncthreads();
  while (true) {
    const uint32_t w = s_next_w;  // same value in every lane
    if (w >= n_items) break;      // the counter only grows: every workgroup gets here
    MoveItem cur = items[w];
    const bool leader = cur.from != kNone && (head == nullptr || head[cur.from] == w);
    __syncthreads();  // everyone has read s_next_w
    if (threadIdx.x == 0) s_next_w = atomicAdd(counter, 1u);  // fetched while this item is being moved
    if (leader && cur.from < n_from) {
      const uint8_t *fbase = from + (uint64_t)cur.from * fl.tok_stride;
      uint32_t node = w;
      do {  // passes of at most `fanout` destinations over the same source rows
        if (threadIdx.x == 0) {
          uint32_t k = 0, nd = node;
          MoveItem it = nd == w ? cur : items[nd];
          while (true) {
            if (it.to < n_to) {
              s_to[k] = it.to;
              s_delta[k] = it.delta;
              ++k;
            }
            nd = it.next;
            if (nd == kNone || nd >= n_items || k == fanout) break;
            it = items[nd];
          }
          s_k = k;
          s_more = (nd != kNone && nd < n_items) ? nd : kNone;
        }
        __syncthreads();
        const uint32_t K = s_k;
        if (ROPE) {
          for (uint32_t i = threadIdx.x; i < K * half; i += kMoveThreads) {
            const uint32_t k = i / half, j = i - k * half;
            const int32_t dl = s_delta[k];
            if (dl != 0) {
              double sn, cs;
              sincos((double)dl * rope.inv_freq[j], &sn, &cs);
              s_cos[i] = cs;
              s_sin[i] = sn;
            }
          }
          __syncthreads();
        }
        uint32_t r = r_init, c = c_init;
        for (uint32_t j = 0; j < steps; j += U) {
          u32x4 v[U], par[U];
          uint64_t doff[U];
          uint32_t cc[U];
          bool ok[U], is_k[U];
#pragma unroll
          for (int u = 0; u < U; ++u) {
            ok[u] = r < n_rows;  // r only grows, so the valid steps of a lane are a prefix
            const uint64_t l = r >> 1, kv = r & 1;
            is_k[u] = kv == 0;
            cc[u] = c;
            doff[u] = l * tl.layer_stride + kv * tl.kv_stride + (uint64_t)c * 16;
            v[u] = u32x4{0, 0, 0, 0};
            if (ok[u]) v[u] = load16<NTL>(fbase + l * fl.layer_stride + kv * fl.kv_stride + (uint64_t)c * 16);
            par[u] = v[u];
            c += c_step;
            r += r_step;
            if (c >= vpr) {
              c -= vpr;
              r += 1;
            }
          }
          if (ROPE && rope.style == 0) {
            // partner vector sits half a head away: vph/2 lanes further (all lanes take part)
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
              for (int q = 0; q < 4; ++q) par[u][q] = __shfl_xor(v[u][q], (int)(vph / 2), kWave);
          }
          for (uint32_t k = 0; k < K; ++k) {
            uint8_t *tbase = to + (uint64_t)s_to[k] * tl.tok_stride;
            const bool rot = ROPE && s_delta[k] != 0;
#pragma unroll
            for (int u = 0; u < U; ++u) {
              if (!ok[u]) continue;
              u32x4 x = v[u];
              if (rot && is_k[u])
                x = rotate_vec(v[u], par[u], cc[u] % vph, rope.style, half, s_cos + k * half, s_sin + k * half);
              store16<NTS>(tbase + doff[u], x);
            }
          }
        }
        node = s_more;
        __syncthreads();  // lists and tables are free for the next pass / item
      } while (node != kNone);
    } else {
      if (cur.from != kNone && cur.from >= n_from && threadIdx.x == 0) atomicOr(status_flags, CP_FLAG_BAD_INDEX);
      __syncthreads();  // s_next_w is written
    }
  }
}

// The two users of the mover get kernels of their own name, so that profiles tell them apart.
template <class RA, bool ROPE, bool NTL, bool NTS, int U>
__global__ __launch_bounds__(kMoveThreads) void gather_rows_kernel(
    const MoveItem *__restrict__ items, const uint32_t *__restrict__ n_items_ptr, uint32_t max_items,
    const uint32_t *__restrict__ head, uint32_t *counter, const uint8_t *__restrict__ pool, cp_kv_layout pool_l,
    uint32_t n_pool_slots, uint8_t *__restrict__ dst, cp_kv_layout dst_l, uint32_t n_dst_tokens, uint32_t fanout,
    uint32_t *status_flags, RA rope) {
  move_rows_body<RA, ROPE, NTL, NTS, U>(items, n_items_ptr, max_items, head, counter, pool, pool_l, n_pool_slots, dst,
                                        dst_l, n_dst_tokens, fanout, status_flags, rope);
}

template <class RA, bool ROPE, bool NTL, bool NTS, int U>
__global__ __launch_bounds__(kMoveThreads) void scatter_rows_kernel(
    const MoveItem *__restrict__ items, const uint32_t *__restrict__ n_items_ptr, uint32_t max_items,
    const uint32_t *__restrict__ head, uint32_t *counter, const uint8_t *__restrict__ src, cp_kv_layout src_l,
    uint32_t n_src_tokens, uint8_t *__restrict__ pool, cp_kv_layout pool_l, uint32_t n_pool_slots, uint32_t fanout,
    uint32_t *status_flags, RA rope) {
  move_rows_body<RA, ROPE, NTL, NTS, U>(items, n_items_ptr, max_items, head, counter, src, src_l, n_src_tokens, pool,
                                        pool_l, n_pool_slots, fanout, status_flags, rope);
}

uint32_t cu_count() {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0)
      v = 256;
    cus = v;
  }
  return (uint32_t)cus;
}

template <class RA, bool ROPE, bool GATHER>
int32_t launch_move(hipStream_t stream, const MoveItem *items, const uint32_t *n_items, uint32_t max_items,
                    const uint32_t *head, uint32_t *counter, const void *from, const cp_kv_layout &fl, uint32_t n_from,
                    void *to, const cp_kv_layout &tl, uint32_t n_to, uint32_t *status_flags, const RA &rope) {
  if (max_items == 0) return CP_OK;
  const Tuning &tn = tuning();
  uint64_t grid = (uint64_t)cu_count() * (tn.move_blocks_per_cu ? tn.move_blocks_per_cu : 8);
  if (grid > max_items) grid = max_items;
  uint32_t fanout = kMaxFanout;
  if (ROPE) {
    uint32_t cap = kTrigDoubles / (fl.head_dim / 2);
    if (fanout > cap) fanout = cap;
  }
  const uint8_t *f = (const uint8_t *)from;
  uint8_t *t = (uint8_t *)to;
#define CP_LAUNCH(NTL, NTS, UN)                                                                             \
  if (GATHER)                                                                                               \
    gather_rows_kernel<RA, ROPE, NTL, NTS, UN><<<(uint32_t)grid, kMoveThreads, 0, stream>>>(                \
        items, n_items, max_items, head, counter, f, fl, n_from, t, tl, n_to, fanout, status_flags, rope);  \
  else                                                                                                      \
    scatter_rows_kernel<RA, ROPE, NTL, NTS, UN><<<(uint32_t)grid, kMoveThreads, 0, stream>>>(               \
        items, n_items, max_items, head, counter, f, fl, n_from, t, tl, n_to, fanout, status_flags, rope)
  const bool deep = !ROPE && tn.move_unroll >= 8;  // rotation keeps the short form: it needs the registers
  switch ((tn.move_nontemporal & 3u) | (deep ? 4u : 0u)) {
    case 0: CP_LAUNCH(false, false, 4); break;
    case 1: CP_LAUNCH(true, false, 4); break;
    case 2: CP_LAUNCH(false, true, 4); break;
    case 3: CP_LAUNCH(true, true, 4); break;
    case 4: CP_LAUNCH(false, false, 8); break;
    case 5: CP_LAUNCH(true, false, 8); break;
    case 6: CP_LAUNCH(false, true, 8); break;
    default: CP_LAUNCH(true, true, 8); break;
  }
#undef CP_LAUNCH
  return check_launch();
}

}  // namespace

int32_t launch_scatter(hipStream_t stream, const void *src, const cp_kv_layout &src_l, uint32_t n_src_tokens,
                       void *pool, const cp_kv_layout &pool_l, uint32_t n_pool_slots, const MoveItem *items,
                       const uint32_t *n_items, uint32_t max_items, uint32_t *counter, uint32_t *status_flags) {
  NoRope none{};
  return launch_move<NoRope, false, false>(stream, items, n_items, max_items, nullptr, counter, src, src_l, n_src_tokens, pool,
                                    pool_l, n_pool_slots, status_flags, none);
}

}  // namespace cp

extern "C" int32_t cp_gather_kv(void *stream_, const void *pool, cp_kv_layout pool_l, uint32_t n_pool_slots, void *dst,
                                cp_kv_layout dst_l, uint32_t n_dst_tokens, const uint32_t *span_src,
                                const uint32_t *span_dst, const uint32_t *span_len, const int32_t *span_delta,
                                const uint32_t *span_off, const uint32_t *n_spans, uint32_t max_spans,
                                const cp_rope *rope, uint32_t *status_flags, void *scratch, size_t scratch_bytes) {
  using namespace cp;
  hipStream_t stream = (hipStream_t)stream_;
  if (max_spans == 0 || n_dst_tokens == 0 || n_pool_slots == 0) return CP_OK;
  if (n_dst_tokens >= 0x80000000u || n_pool_slots >= 0x80000000u) return CP_ERR_UNSUPPORTED;
  if (!pool || !dst || !span_src || !span_dst || !span_len || !n_spans || !status_flags) return CP_ERR_INVALID_ARG;
  if (!scratch || !aligned(scratch, 256) || !aligned(pool, 16) || !aligned(dst, 16)) return CP_ERR_INVALID_ARG;
  if (!layout_ok(pool_l) || !layout_ok(dst_l) || !layouts_match(pool_l, dst_l)) return CP_ERR_UNSUPPORTED;
  const bool use_rope = rope != nullptr && span_delta != nullptr;
  RopeArg ra{};
  if (use_rope) {
    const uint32_t D = pool_l.head_dim;
    // pairs must not straddle 16-byte vectors or wavefronts: power-of-two head_dim in [16, 512]
    if (D < 16 || D > 2 * kMaxHalfDim || (D & (D - 1))) return CP_ERR_UNSUPPORTED;
    if (rope->style > 1 || !(rope->theta > 0.0)) return CP_ERR_INVALID_ARG;
    ra.style = rope->style;
    ra.head_dim = D;
    for (uint32_t j = 0; j < D / 2; ++j) ra.inv_freq[j] = std::pow(rope->theta, -2.0 * (double)j / (double)D);
  }
  if (scratch_bytes < cp_scratch_bytes(n_dst_tokens, max_spans, n_pool_slots)) return CP_ERR_SCRATCH;
  Scratch sc(scratch, scratch_bytes);
  uint32_t *agg = sc.take<uint32_t>(div_up(max_spans, kScanTile) + 1);
  uint32_t *offs = sc.take<uint32_t>((size_t)max_spans + 1);
  uint32_t *counters = sc.take<uint32_t>(2);  // [0] work counter, [1] item count
  MoveItem *items = sc.take<MoveItem>(n_dst_tokens);
  const bool group = tuning().move_multicast != 0;
  uint32_t *head = group ? sc.take<uint32_t>(n_pool_slots) : nullptr;
  if (!agg || !offs || !counters || !items || (group && !head)) return CP_ERR_SCRATCH;
  if (!span_off) {
    if (int32_t rc = launch_span_offsets(stream, span_len, n_spans, max_spans, offs, agg)) return rc;
    span_off = offs;
  }
  gather_init_kernel<<<group ? div_up(n_pool_slots, 256) : 1, 256, 0, stream>>>(head, group ? n_pool_slots : 0,
                                                                                counters);
  // spans do not overlap in dst, so they cover at most n_dst_tokens tokens
  gather_expand_kernel<<<div_up(n_dst_tokens, 256), 256, 0, stream>>>(
      span_src, span_dst, span_off, use_rope ? span_delta : nullptr, n_spans, max_spans, n_pool_slots, n_dst_tokens,
      items, head, counters + 1, status_flags);
  if (int32_t rc = check_launch()) return rc;
  const Tuning &tn = tuning();
  if (tn.gather_start && hipEventRecord(tn.gather_start, stream) != hipSuccess) return CP_ERR_HIP;
  int32_t rc;
  if (use_rope) {
    rc = launch_move<RopeArg, true, true>(stream, items, counters + 1, n_dst_tokens, head, counters, pool, pool_l,
                                    n_pool_slots, dst, dst_l, n_dst_tokens, status_flags, ra);
  } else {
    NoRope none{};
    rc = launch_move<NoRope, false, true>(stream, items, counters + 1, n_dst_tokens, head, counters, pool, pool_l,
                                    n_pool_slots, dst, dst_l, n_dst_tokens, status_flags, none);
  }
  if (tn.gather_stop && hipEventRecord(tn.gather_stop, stream) != hipSuccess) return CP_ERR_HIP;
  return rc;
}

extern "C" int32_t cp_gather_events(void *start_event, void *stop_event) {
  cp::tuning().gather_start = (hipEvent_t)start_event;
  cp::tuning().gather_stop = (hipEvent_t)stop_event;
  return CP_OK;
}

extern "C" void *cp_event_create(void) {
  hipEvent_t e = nullptr;
  hipError_t rc = hipEventCreate(&e);
  if (rc != hipSuccess) {
    cp::last_hip_error() = (int32_t)rc;
    return nullptr;
  }
  return (void *)e;
}

extern "C" float cp_event_elapsed_ms(void *start_event, void *stop_event) {
  float ms = -1.0f;
  hipError_t rc = hipEventElapsedTime(&ms, (hipEvent_t)start_event, (hipEvent_t)stop_event);
  if (rc != hipSuccess) {
    cp::last_hip_error() = (int32_t)rc;
    return -1.0f;
  }
  return ms;
}

extern "C" void cp_event_destroy(void *event) {
  if (event) (void)hipEventDestroy((hipEvent_t)event);
}

extern "C" size_t cp_scratch_bytes(uint32_t N, uint32_t max_spans, uint32_t n_pool_slots) {
  using namespace cp;
  uint64_t n = N > max_spans ? N : max_spans;
  // tile totals (16 bytes each), three per-token words (insert) and one 16-byte descriptor per
  // token (gather, insert), span offsets, one chain head per pool slot; pieces padded to 256 bytes
  return (size_t)(((uint64_t)div_up(n, kScanTile) + 2) * 16 + (3ull * 4 + 16) * N + 4ull * ((uint64_t)max_spans + 1) +
                  4ull * n_pool_slots + 12 * 256);
}

extern "C" int32_t cp_last_hip_error(void) { return cp::last_hip_error(); }

extern "C" int32_t cp_tune(int32_t key, uint32_t value) {
  cp::Tuning &t = cp::tuning();
  switch (key) {
    case 0: t.move_multicast = value; return CP_OK;
    case 1: t.move_blocks_per_cu = value; return CP_OK;
    case 2: t.move_nontemporal = value; return CP_OK;
    case 3: t.move_unroll = value; return CP_OK;
    default: return CP_ERR_INVALID_ARG;
  }
}

// Token-granular KV row mover: cp_gather_kv (pool -> request buffers, with
// optional key re-rotation) and the scatter half of cp_insert_kv (request
// buffers -> pool).  "Linking" matched segments into the request (Sec. 4.1 KV
// Retriever, Sec. 4.3.1) becomes a copy of every matched token's K and V rows;
// positions that no span covers are never written.
//
// This is the HBM-bound part of the path: each matched token moves
// 2 * n_layers * row_bytes bytes in and the same amount out, nothing is reused,
// so the kernel is a pure stream of 16-byte loads and stores:
//   - a work item is (token, chunk of that token's rows); workgroups take items
//     grid-stride so a fixed, chip-filling grid serves any device-resident count;
//   - inside an item the 256 lanes walk the (row, 16-byte column) space in
//     row-major order, so every wavefront touches whole contiguous 1 KiB pieces;
//   - several loads are issued before the first store to keep bytes in flight;
//   - loads and stores can be non-temporal: nothing is read twice and the
//     destination is not read back by this kernel.
// Key re-rotation (textbook RoPE, not in the paper) is done in double precision
// on the way through registers: the cos/sin of (delta * inv_freq[j]) are
// computed once per work item into LDS, the partner element of a pair comes from
// the neighbouring lane (half-split style) or from the same 16 bytes
// (interleaved style).
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
constexpr int kMoveUnroll = 4;
constexpr uint32_t kMaxHalfDim = 256;  // head_dim <= 512 when rotating

struct MoveItem {
  uint32_t from, to;
  int32_t delta;
};

// Work items of the gather: token w of the concatenation of all spans.
struct SpanItems {
  const uint32_t *span_src, *span_dst, *span_off;
  const int32_t *span_delta;  // nullable
  const uint32_t *n_spans;
  uint32_t max_spans;
  __device__ __forceinline__ uint32_t n() const {
    uint32_t k = *n_spans;
    return k < max_spans ? k : max_spans;
  }
  __device__ __forceinline__ uint32_t count() const { return span_off[n()]; }
  __device__ __forceinline__ MoveItem get(uint32_t w) const {
    uint32_t lo = 0, hi = n();  // invariant: span_off[lo] <= w < span_off[hi]
    while (hi - lo > 1) {
      uint32_t mid = (lo + hi) >> 1;
      if (span_off[mid] <= w) lo = mid; else hi = mid;
    }
    uint32_t k = w - span_off[lo];
    return MoveItem{span_src[lo] + k, span_dst[lo] + k, span_delta ? span_delta[lo] : 0};
  }
};

// Work items of the scatter: w-th newly stored token.
struct ListItems {
  const uint32_t *item_from, *item_to;
  const uint32_t *n_items;
  uint32_t max_items;
  __device__ __forceinline__ uint32_t count() const {
    uint32_t k = *n_items;
    return k < max_items ? k : max_items;
  }
  __device__ __forceinline__ MoveItem get(uint32_t w) const { return MoveItem{item_from[w], item_to[w], 0}; }
};

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

template <class Items, class RA, bool ROPE, bool NTL, bool NTS>
__global__ __launch_bounds__(kMoveThreads) void move_rows_kernel(Items items, const uint8_t *__restrict__ from,
                                                                 cp_kv_layout fl, uint32_t n_from,
                                                                 uint8_t *__restrict__ to, cp_kv_layout tl,
                                                                 uint32_t n_to, uint32_t rows_per_item,
                                                                 uint32_t *status_flags, RA rope) {
  __shared__ double s_cos[ROPE ? kMaxHalfDim : 1], s_sin[ROPE ? kMaxHalfDim : 1];
  const uint32_t n_rows = fl.n_layers * 2;
  const uint32_t vpr = fl.n_kv_heads * fl.head_dim / 8;  // 16-byte vectors per row
  const uint32_t chunks = (n_rows + rows_per_item - 1) / rows_per_item;
  const uint64_t n_items = (uint64_t)items.count() * chunks;
  // lane t starts at vector t of the item and advances by 256 vectors per step
  const uint32_t r_step = kMoveThreads / vpr, c_step = kMoveThreads % vpr;
  const uint32_t r_init = threadIdx.x / vpr, c_init = threadIdx.x % vpr;
  const uint32_t vph = fl.head_dim / 8;  // vectors per head
  const uint32_t half = fl.head_dim / 2;

  for (uint64_t it = blockIdx.x; it < n_items; it += gridDim.x) {
    const uint32_t w = (uint32_t)(it / chunks), ch = (uint32_t)(it - (uint64_t)w * chunks);
    const MoveItem d = items.get(w);
    if (d.from >= n_from || d.to >= n_to) {  // same for the whole workgroup
      if (threadIdx.x == 0) atomicOr(status_flags, CP_FLAG_BAD_INDEX);
      continue;
    }
    const uint32_t row0 = ch * rows_per_item;
    const uint32_t nr = min(rows_per_item, n_rows - row0);
    const uint8_t *fbase = from + (uint64_t)d.from * fl.tok_stride;
    uint8_t *tbase = to + (uint64_t)d.to * tl.tok_stride;
    const bool rot = ROPE && d.delta != 0;
    if (ROPE) {
      __syncthreads();  // the previous item's readers are done with the tables
      if (rot && threadIdx.x < half) {
        double sn, cs;
        sincos((double)d.delta * rope.inv_freq[threadIdx.x], &sn, &cs);
        s_cos[threadIdx.x] = cs;
        s_sin[threadIdx.x] = sn;
      }
      __syncthreads();
    }
    const uint32_t steps = (nr * vpr + kMoveThreads - 1) / kMoveThreads;  // same for every lane
    uint32_t r = r_init, c = c_init;
    for (uint32_t j = 0; j < steps; j += kMoveUnroll) {
      u32x4 v[kMoveUnroll];
      uint8_t *dp[kMoveUnroll];
      uint32_t cc[kMoveUnroll];
      bool ok[kMoveUnroll], is_k[kMoveUnroll];
#pragma unroll
      for (int u = 0; u < kMoveUnroll; ++u) {
        ok[u] = r < nr;  // r only grows, so the valid steps of a lane are a prefix
        const uint32_t row = row0 + r;
        const uint64_t l = row >> 1, kv = row & 1;
        is_k[u] = kv == 0;
        cc[u] = c;
        dp[u] = tbase + l * tl.layer_stride + kv * tl.kv_stride + (uint64_t)c * 16;
        v[u] = u32x4{0, 0, 0, 0};
        if (ok[u]) v[u] = load16<NTL>(fbase + l * fl.layer_stride + kv * fl.kv_stride + (uint64_t)c * 16);
        c += c_step;
        r += r_step;
        if (c >= vpr) {
          c -= vpr;
          r += 1;
        }
      }
      if (rot) {
#pragma unroll
        for (int u = 0; u < kMoveUnroll; ++u) {
          const uint32_t cih = cc[u] % vph;
          u32x4 par = v[u];
          if (rope.style == 0) {  // partner vector sits half a head away: vph/2 lanes (all lanes take part)
#pragma unroll
            for (int q = 0; q < 4; ++q) par[q] = __shfl_xor(v[u][q], (int)(vph / 2), kWave);
          }
          if (ok[u] && is_k[u]) v[u] = rotate_vec(v[u], par, cih, rope.style, half, s_cos, s_sin);
        }
      }
#pragma unroll
      for (int u = 0; u < kMoveUnroll; ++u)
        if (ok[u]) store16<NTS>(dp[u], v[u]);
    }
  }
}

template <class Items, class RA, bool ROPE>
int32_t launch_move(hipStream_t stream, const Items &items, uint32_t max_tokens, const void *from,
                    const cp_kv_layout &fl, uint32_t n_from, void *to, const cp_kv_layout &tl, uint32_t n_to,
                    uint32_t *status_flags, const RA &rope) {
  if (max_tokens == 0) return CP_OK;
  const Tuning &tn = tuning();
  const uint32_t n_rows = fl.n_layers * 2;
  uint32_t rpi = tn.move_rows_per_item ? tn.move_rows_per_item : n_rows;
  if (rpi > n_rows) rpi = n_rows;
  const uint64_t max_items = (uint64_t)max_tokens * ((n_rows + rpi - 1) / rpi);
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
    cus = 256;
  uint64_t grid = (uint64_t)cus * (tn.move_blocks_per_cu ? tn.move_blocks_per_cu : 8);
  if (grid > max_items) grid = max_items;
  const uint8_t *f = (const uint8_t *)from;
  uint8_t *t = (uint8_t *)to;
#define CP_LAUNCH(NTL, NTS)                                                                                      \
  move_rows_kernel<Items, RA, ROPE, NTL, NTS><<<(uint32_t)grid, kMoveThreads, 0, stream>>>(items, f, fl, n_from, t, tl, \
                                                                                        n_to, rpi, status_flags, rope)
  switch (tn.move_nontemporal & 3u) {
    case 0: CP_LAUNCH(false, false); break;
    case 1: CP_LAUNCH(true, false); break;
    case 2: CP_LAUNCH(false, true); break;
    default: CP_LAUNCH(true, true); break;
  }
#undef CP_LAUNCH
  return check_launch();
}

}  // namespace

int32_t launch_scatter(hipStream_t stream, const void *src, const cp_kv_layout &src_l, uint32_t n_src_tokens,
                       void *pool, const cp_kv_layout &pool_l, uint32_t n_pool_slots, const uint32_t *item_tok,
                       const uint32_t *item_slot, const uint32_t *n_items, uint32_t max_items,
                       uint32_t *status_flags) {
  ListItems items{item_tok, item_slot, n_items, max_items};
  NoRope none{};
  return launch_move<ListItems, NoRope, false>(stream, items, max_items, src, src_l, n_src_tokens, pool, pool_l, n_pool_slots,
                                       status_flags, none);
}

}  // namespace cp

extern "C" int32_t cp_gather_kv(void *stream_, const void *pool, cp_kv_layout pool_l, uint32_t n_pool_slots, void *dst,
                                cp_kv_layout dst_l, uint32_t n_dst_tokens, const uint32_t *span_src,
                                const uint32_t *span_dst, const uint32_t *span_len, const int32_t *span_delta,
                                const uint32_t *span_off, const uint32_t *n_spans, uint32_t max_spans,
                                const cp_rope *rope, uint32_t *status_flags, void *scratch, size_t scratch_bytes) {
  using namespace cp;
  hipStream_t stream = (hipStream_t)stream_;
  if (max_spans == 0 || n_dst_tokens == 0) return CP_OK;
  if (n_dst_tokens >= 0x80000000u || n_pool_slots >= 0x80000000u) return CP_ERR_UNSUPPORTED;
  if (!pool || !dst || !span_src || !span_dst || !span_len || !n_spans || !status_flags) return CP_ERR_INVALID_ARG;
  if (!aligned(pool, 16) || !aligned(dst, 16)) return CP_ERR_INVALID_ARG;
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
  if (!span_off) {
    if (!scratch || !aligned(scratch, 256)) return CP_ERR_INVALID_ARG;
    if (scratch_bytes < cp_scratch_bytes(0, max_spans)) return CP_ERR_SCRATCH;
    Scratch sc(scratch, scratch_bytes);
    uint32_t *agg = sc.take<uint32_t>(div_up(max_spans, kScanTile) + 1);
    uint32_t *offs = sc.take<uint32_t>((size_t)max_spans + 1);
    if (!agg || !offs) return CP_ERR_SCRATCH;
    if (int32_t rc = launch_span_offsets(stream, span_len, n_spans, max_spans, offs, agg)) return rc;
    span_off = offs;
  }
  SpanItems items{span_src, span_dst, span_off, use_rope ? span_delta : nullptr, n_spans, max_spans};
  // spans do not overlap in dst, so they cover at most n_dst_tokens tokens
  if (use_rope)
    return launch_move<SpanItems, RopeArg, true>(stream, items, n_dst_tokens, pool, pool_l, n_pool_slots, dst, dst_l,
                                                 n_dst_tokens, status_flags, ra);
  NoRope none{};
  return launch_move<SpanItems, NoRope, false>(stream, items, n_dst_tokens, pool, pool_l, n_pool_slots, dst, dst_l,
                                               n_dst_tokens, status_flags, none);
}

extern "C" size_t cp_scratch_bytes(uint32_t N, uint32_t max_spans) {
  using namespace cp;
  uint64_t n = N > max_spans ? N : max_spans;
  // tile totals (16 bytes each) + three per-token words + span offsets, each piece padded to 256 bytes
  return (size_t)(((uint64_t)div_up(n, kScanTile) + 2) * 16 + 3ull * 4 * N + 4ull * ((uint64_t)max_spans + 1) + 8 * 256);
}

extern "C" int32_t cp_last_hip_error(void) { return cp::last_hip_error(); }

extern "C" int32_t cp_tune(int32_t key, uint32_t value) {
  cp::Tuning &t = cp::tuning();
  switch (key) {
    case 0: t.move_rows_per_item = value; return CP_OK;
    case 1: t.move_blocks_per_cu = value; return CP_OK;
    case 2: t.move_nontemporal = value; return CP_OK;
    default: return CP_ERR_INVALID_ARG;
  }
}

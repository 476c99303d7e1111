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
//   - the chain heads are gathered into a dense work list (chains of several tokens first, single
//     tokens after them), so no workgroup ever meets a token that has nothing to do; units of
//     work are taken from the list through an atomic counter (one unit per ticket, several for
//     small tokens), so long chains and single tokens balance, and every workgroup leaves the
//     loop as soon as the counter passes the ticket count;
//   - a workgroup is four mover wavefronts plus one scout wavefront: the scout fetches and
//     decodes the next unit (descriptor, chain links, rotation tables) into LDS while the movers
//     copy the current one, so the movers never wait for a descriptor; one barrier per unit;
//   - inside a unit the 256 mover lanes walk the (row, 16-byte column) space in row-major order,
//     so every wavefront touches whole contiguous 1 KiB pieces; up to 16 loads per lane are
//     issued before the first store, and both directions can be non-temporal (nothing is read
//     back by this kernel).
// Key re-rotation (textbook RoPE, not in the paper) is done in double precision
// on the way through registers: cos/sin of delta * inv_freq[j] are computed once
// per destination into LDS, the partner element of a pair comes from the
// neighbouring lane (half-split style) or from the same 16 bytes (interleaved).
#include "cp_device.h"
#include "cp_internal.h"

#include <cmath>
#include <mutex>
#include <type_traits>

namespace cp {

bool resolve_opts(const cp_launch_opts *o, bool rotating, MoveOpts *out) {
  // defaults: non-temporal stores; loads in flight and workgroups are chosen at launch from the row shape
  // (0 here): 16 loads in flight per lane and one workgroup per compute unit for the Llama shapes
  (void)rotating;
  MoveOpts m{true, 0u, 0u, 2u, 0u, 16u, nullptr, nullptr};
  if (o) {
    if (o->read_sharing > 2 || o->blocks_per_cu > 64 || o->nontemporal > 4 || o->fanout > 16) return false;
    if (o->loads_in_flight != 0 && o->loads_in_flight != 4 && o->loads_in_flight != 8 && o->loads_in_flight != 16)
      return false;
    if (o->workgroups > (1u << 20) || o->reserved[0] | o->reserved[1]) return false;
    if (o->workgroups) m.workgroups = o->workgroups;
    if ((o->start_event == nullptr) != (o->stop_event == nullptr)) return false;
    if (o->read_sharing == 2) m.share_reads = false;
    if (o->blocks_per_cu) m.blocks_per_cu = o->blocks_per_cu;
    if (o->nontemporal) m.nontemporal = o->nontemporal - 1;
    if (o->loads_in_flight) m.loads_in_flight = o->loads_in_flight;
    if (o->fanout) m.fanout = o->fanout;
    m.start = (hipEvent_t)o->start_event;
    m.stop = (hipEvent_t)o->stop_event;
  }
  *out = m;
  return true;
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

constexpr int kMoveThreads = 256;                   // lanes of a workgroup that move rows
constexpr int kBlockThreads = kMoveThreads + kWave;  // ... plus one scout wavefront
constexpr uint32_t kMaxHalfDim = 256;    // head_dim <= 512 when rotating
constexpr uint32_t kMaxFanout = 16;      // destinations served per pass over the source rows
constexpr uint32_t kTrigDoubles = 1024;  // LDS doubles for cos (and as many for sin) per descriptor: fan-out * head_dim/2 <= this
constexpr uint32_t kNone = 0xFFFFFFFFu;
constexpr uint32_t kMaxTake = 8;         // units per ticket of the work counter, at most
constexpr uint32_t kTicketStride = 256;  // distance between the units of one ticket of the work counter
constexpr uint32_t kShareReadsFrom = 4096;  // destination tokens from which a gather shares reads by default

// cos/sin of (delta * inv_freq[j]) for any 32-bit delta come from five small
// tables, one per 7-bit digit of |delta|: entry [level][m][j] holds cos and sin of
// (m << 7*level) * inv_freq[j].  The angles of the digits add up to the exact
// product, so four complex multiplications give the wanted pair, and the mover
// needs no trigonometric code of its own.
constexpr uint32_t kTrigLevels = 5, kTrigDigit = 128;

struct InvFreq {
  double v[kMaxHalfDim];  // theta^(-2j/head_dim), evaluated on the host
};
template <uint32_t STYLE>  // the pairing style is a compile-time property of the kernel
struct RopeArg {
  static constexpr uint32_t style = STYLE;
  const double2 *tables;  // [kTrigLevels][kTrigDigit][head_dim / 2]
};
struct NoRope {  // stand-in for kernels that never rotate
  static constexpr uint32_t style = 0;
  const double2 *tables;
};

__global__ __launch_bounds__(256) void rope_tables_kernel(InvFreq inv, uint32_t half, double2 *__restrict__ tables) {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= kTrigLevels * kTrigDigit * half) return;
  const uint32_t j = i % half, m = (i / half) % kTrigDigit, level = i / (half * kTrigDigit);
  const double mult = (double)((uint64_t)m << (7 * level));  // exact
  const double f = inv.v[j];
  const double p = mult * f, e = fma(mult, f, -p);  // mult * f = p + e exactly
  double sn, cs;
  sincos(p, &sn, &cs);
  tables[i] = make_double2(cs - e * sn, sn + e * cs);  // first-order correction for the rounded-off part e
}

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

// The two bf16 values packed in a dword, as doubles (exact).
__device__ __forceinline__ double bf16_lo_to_f64(uint32_t w) { return (double)__uint_as_float(w << 16); }
__device__ __forceinline__ double bf16_hi_to_f64(uint32_t w) { return (double)__uint_as_float(w & 0xFFFF0000u); }

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// A double rounded to float and then to bf16 is rounded twice; the result differs from one direct
// rounding only if the float happens to sit exactly half way between two bf16 values although the
// double did not.  Such a float (low half 0x8000, inexact) is nudged one float step back towards
// the double, after which the second rounding goes the right way.
__device__ __forceinline__ float toward(float f, double x) {
  uint32_t u = __float_as_uint(f);
  const double back = (double)f;
  if (back != x && x == x) u += fabs(back) > fabs(x) ? 0xFFFFFFFFu : 1u;  // sign-magnitude: -1 shrinks, +1 grows
  return __uint_as_float(u);
}

// Two doubles -> two bf16 packed in a dword (x0 low), each with the effect of a single rounding to
// nearest, ties to even.  The float -> bf16 step is the hardware's packed conversion.
__device__ __forceinline__ uint32_t f64x2_to_bf16x2(double x0, double x1) {
  float f0 = (float)x0, f1 = (float)x1;
  const bool tie0 = (__float_as_uint(f0) & 0xFFFFu) == 0x8000u, tie1 = (__float_as_uint(f1) & 0xFFFFu) == 0x8000u;
  if (__builtin_expect(tie0 || tie1, 0)) {
    if (tie0) f0 = toward(f0, x0);
    if (tie1) f1 = toward(f1, x1);
  }
  const bf16x2 r = __builtin_convertvector(f32x2{f0, f1}, bf16x2);
  return __builtin_bit_cast(uint32_t, r);
}

// Rotation of one 16-byte vector (8 bf16 values) of a K row.
//
// A lane always works on the same 16-byte column of a head (the lane stride, 256 vectors, and the
// row length are multiples of the vectors per head), so which frequencies it needs is fixed.
//
// Half-split style (element j pairs with j + head_dim/2): the lane `vph/2` further holds the partner
// vector.  The two lanes split the eight pairs between them — the first-half lane does pairs 0..3,
// the second-half lane pairs 4..7 — and each computes BOTH outputs of its pairs, so every input is
// widened to double once and every lane needs only four cos/sin pairs.  Two dwords go each way
// before (the partner's inputs for my pairs) and after (the partner's half of the results).
//
// Interleaved style (2j pairs with 2j+1): both elements of a pair are in the lane's own vector;
// four pairs, four cos/sin pairs, no exchange.
struct Trig4 {
  double c[4], s[4];
};

// Index of the first of the four frequencies this lane works on.
template <uint32_t STYLE>
__device__ __forceinline__ uint32_t first_freq(uint32_t half, uint32_t col_in_head) {
  if (STYLE == 0) {
    const uint32_t vec_per_half = half / 8;
    const bool second = col_in_head >= vec_per_half;
    return (second ? col_in_head - vec_per_half : col_in_head) * 8 + (second ? 4u : 0u);
  }
  return col_in_head * 4;
}

__device__ __forceinline__ Trig4 load_trig(uint32_t j0, const double *cs, const double *sn) {
  Trig4 t;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    t.c[e] = cs[j0 + e];
    t.s[e] = sn[j0 + e];
  }
  return t;
}

// The inputs of this lane's four pairs as doubles: x1 from the first half of the head (or the even
// elements), x2 from the second half (or the odd elements).
struct Pairs4 {
  double x1[4], x2[4];
};

template <uint32_t STYLE>
__device__ __forceinline__ Pairs4 widen_pairs(u32x4 own, bool second, int partner_xor) {
  Pairs4 p;
  if (STYLE == 0) {
    // my pairs use dwords 0..1 (first-half lane) or 2..3 (second-half lane) of both vectors;
    // the partner needs the other two dwords of mine
    const uint32_t mine0 = second ? own[2] : own[0], mine1 = second ? own[3] : own[1];
    const uint32_t give0 = second ? own[0] : own[2], give1 = second ? own[1] : own[3];
    const uint32_t got0 = __shfl_xor(give0, partner_xor, kWave), got1 = __shfl_xor(give1, partner_xor, kWave);
    const uint32_t f0 = second ? got0 : mine0, f1 = second ? got1 : mine1;  // first-half elements
    const uint32_t g0 = second ? mine0 : got0, g1 = second ? mine1 : got1;  // second-half elements
    p.x1[0] = bf16_lo_to_f64(f0), p.x1[1] = bf16_hi_to_f64(f0), p.x1[2] = bf16_lo_to_f64(f1), p.x1[3] = bf16_hi_to_f64(f1);
    p.x2[0] = bf16_lo_to_f64(g0), p.x2[1] = bf16_hi_to_f64(g0), p.x2[2] = bf16_lo_to_f64(g1), p.x2[3] = bf16_hi_to_f64(g1);
  } else {
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      p.x1[w] = bf16_lo_to_f64(own[w]);
      p.x2[w] = bf16_hi_to_f64(own[w]);
    }
  }
  return p;
}

template <uint32_t STYLE>
__device__ __forceinline__ u32x4 rotate_pairs(const Pairs4 &p, const Trig4 &t, bool second, int partner_xor) {
  double y1[4], y2[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    y1[e] = fma(p.x1[e], t.c[e], -(p.x2[e] * t.s[e]));
    y2[e] = fma(p.x2[e], t.c[e], p.x1[e] * t.s[e]);
  }
  if (STYLE == 0) {
    // y1 belongs to the first-half lane's vector, y2 to the second-half lane's
    const uint32_t a0 = f64x2_to_bf16x2(y1[0], y1[1]), a1 = f64x2_to_bf16x2(y1[2], y1[3]);
    const uint32_t b0 = f64x2_to_bf16x2(y2[0], y2[1]), b1 = f64x2_to_bf16x2(y2[2], y2[3]);
    const uint32_t keep0 = second ? b0 : a0, keep1 = second ? b1 : a1;
    const uint32_t got0 = __shfl_xor(second ? a0 : b0, partner_xor, kWave);
    const uint32_t got1 = __shfl_xor(second ? a1 : b1, partner_xor, kWave);
    // first-half lane: its own pairs 0..3 then the partner's 4..7; second-half lane the other way round
    return second ? u32x4{got0, got1, keep0, keep1} : u32x4{keep0, keep1, got0, got1};
  }
  return u32x4{f64x2_to_bf16x2(y1[0], y2[0]), f64x2_to_bf16x2(y1[1], y2[1]), f64x2_to_bf16x2(y1[2], y2[2]),
               f64x2_to_bf16x2(y1[3], y2[3])};
}

// Scratch bytes any call needs: tile totals (at most 32 bytes each), four per-token words (insert),
// one 16-byte descriptor per token (gather, insert), a work-list entry per token (gather) and two flag
// bytes per token (floating anchors, chain-recording insert), span offsets, one chain head per pool slot, the cos/sin digit tables;
// pieces padded to 256 bytes.
constexpr size_t scratch_bytes_for(uint32_t N, uint32_t max_spans, uint32_t n_pool_slots) {
  const uint64_t n = N > max_spans ? N : max_spans;
  return (size_t)(((n + kScanTile - 1) / kScanTile + 2) * 32 + (4ull * 4 + 16 + 2 + 4) * N +
                  4ull * ((uint64_t)max_spans + 1) + 4ull * n_pool_slots +
                  (size_t)kTrigLevels * kTrigDigit * kMaxHalfDim * 16 + 16 * 256);
}

// ---- gather front end: clear the per-slot chain heads, expand spans, link chains -------------

__global__ __launch_bounds__(256) void gather_init_kernel(uint32_t *__restrict__ head, uint32_t n_head,
                                                          uint32_t *__restrict__ counter) {
  uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_head) head[i] = kNone;
  if (i == 0) counter[0] = counter[2] = counter[3] = 0;  // work counter, work-list counts ([1] is set by the expansion)
}

// One thread per token of the concatenated spans.
__global__ __launch_bounds__(256) void gather_expand_kernel(
    const uint32_t *__restrict__ span_src, const uint32_t *__restrict__ span_dst,
    const uint32_t *__restrict__ span_off, const int32_t *__restrict__ span_delta, const uint32_t *__restrict__ n_spans,
    uint32_t max_spans, uint32_t n_pool_slots, uint32_t n_dst_tokens, MoveItem *__restrict__ items,
    uint32_t *__restrict__ head /* nullable: no grouping */, uint32_t *__restrict__ counters,
    uint32_t *__restrict__ status_flags) {
  uint32_t n = *n_spans;
  if (n > max_spans) n = max_spans;
  uint32_t total = span_off[n];
  if (total > n_dst_tokens) total = n_dst_tokens;  // spans that do not overlap cannot cover more
  const uint32_t w = blockIdx.x * blockDim.x + threadIdx.x;
  if (w == 0) {
    counters[1] = total;            // item count
    if (!head) counters[0] = 0;     // work counter of the mover (with grouping, gather_init_kernel has cleared it)
  }
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

// The work list of a gather that shares reads: the chain heads, chains of several tokens first and
// single tokens behind them (so that the long units are not the last ones running).  One thread per
// token; the lanes of a wavefront that hold heads of one kind take their places with one atomic.
// counts[0] = chains taken from the front, counts[1] = single tokens taken from the back.
__global__ __launch_bounds__(256) void gather_heads_kernel(const MoveItem *__restrict__ items,
                                                           const uint32_t *__restrict__ n_items_ptr,
                                                           uint32_t max_items, const uint32_t *__restrict__ head,
                                                           uint32_t *__restrict__ units, uint32_t *counts) {
  uint32_t n = *n_items_ptr;
  if (n > max_items) n = max_items;
  const uint32_t w = blockIdx.x * blockDim.x + threadIdx.x;
  bool is_head = false, chain = false;
  if (w < n) {
    const MoveItem it = items[w];
    is_head = it.from != kNone && head[it.from] == w;
    chain = is_head && it.next != kNone;
  }
  const uint32_t lane = threadIdx.x & (kWave - 1);
  const unsigned long long below = (1ull << lane) - 1ull;
  const unsigned long long mc = __ballot(chain), ms = __ballot(is_head && !chain);
  uint32_t base_c = 0, base_s = 0;
  if (lane == 0) {
    if (mc) base_c = atomicAdd(&counts[0], (uint32_t)__popcll(mc));
    if (ms) base_s = atomicAdd(&counts[1], (uint32_t)__popcll(ms));
  }
  base_c = __shfl(base_c, 0, kWave);
  base_s = __shfl(base_s, 0, kWave);
  // chains and single tokens together are at most n, so the two ends never meet
  if (chain) units[base_c + __popcll(mc & below)] = w;
  else if (is_head) units[max_items - 1 - (base_s + __popcll(ms & below))] = w;
}

// ---- the mover ---------------------------------------------------------------------------------

// One work unit = one chain = all rows of one source token, written to every destination of the chain
// (at most `fanout` of them per pass).  A workgroup is four mover wavefronts plus one scout wavefront:
//   - the scout takes the next unit (a ticket of the atomic counter names one or a few) while the movers
//     are busy with the current one: it walks the unit's chain, and leaves the unit's
//     source, destination offsets, deltas and (rotating gather) cos/sin values in the other half of a
//     double-buffered descriptor in LDS.  Everything serial and latency-bound (dependent loads through
//     items[] and head[], the trigonometric table products) is thus off the movers' path, and a unit
//     costs one barrier;
//   - the 256 mover lanes walk the (row, 16-byte column) space row-major; a round is U vectors per lane:
//     all of a round's loads are issued before its first store, and a vector goes to all of its
//     destinations before the next vector is touched.  Rows alternate K, V; with RoPE a lane rotates the
//     vectors of its K rows.  For the Llama shapes a step of the 256 lanes is exactly one K row and one V row,
//     so a rotating gather swaps the two between the halves of the workgroup on every other step: each
//     wavefront then rotates half of its vectors instead of two wavefronts rotating all of theirs.
// Every wavefront executes exactly one barrier per unit and leaves when the scout reports that the
// counter has passed the item count, which every workgroup's scout eventually sees.
// Items that reach the mover name a destination inside `to`: cp_gather_kv's expansion and
// cp_insert_kv's commit step take out (and flag) every item that does not, so only the source index is
// checked here.
struct UnitDesc {
  uint64_t tobase[kMaxFanout];  // byte offset of every destination token
  int32_t delta[kMaxFanout];
  uint32_t from;  // source token; kNone = no more work
  uint32_t k;     // destinations in this pass
};

template <class RA, bool ROPE, bool NTL, bool NTS, int U>
__device__ __forceinline__ void move_rows_body(
    const MoveItem *__restrict__ items, const uint32_t *__restrict__ n_items_ptr, uint32_t max_items,
    const uint32_t *__restrict__ units /* nullable: every item is a unit of its own */,
    const uint32_t *__restrict__ unit_counts, uint32_t *counter, const uint8_t *__restrict__ from,
    const cp_kv_layout &fl, uint32_t n_from, uint8_t *__restrict__ to, const cp_kv_layout &tl, uint32_t fanout,
    uint32_t take, uint32_t *status_flags, const RA &rope) {
  __shared__ UnitDesc s_unit[2];
  __shared__ MoveItem s_ahead[kMaxTake];  // the scout's own: first item of each unit of its ticket, and which item that is
  __shared__ uint32_t s_ahead_w[kMaxTake];
  __shared__ double s_cos[2][ROPE ? kTrigDoubles : 1], s_sin[2][ROPE ? kTrigDoubles : 1];

  uint32_t n_items = *n_items_ptr;
  if (n_items > max_items) n_items = max_items;
  // with a work list: its chains are entries 0 .. n_chains-1, its single tokens the last n_single entries
  uint32_t n_chains = 0, n_units = n_items;
  if (units) {
    n_chains = unit_counts[0] < max_items ? unit_counts[0] : max_items;
    const uint32_t n_single = unit_counts[1] < max_items - n_chains ? unit_counts[1] : max_items - n_chains;
    n_units = n_chains + n_single;
  }
  // Destinations that read so few distinct slots that there are fewer chains than workgroups would leave most
  // of the chip idle while a few workgroups walk long chains.  Every token is then moved on its own, the
  // links ignored; the repeated reads of those few slots come from cache.  (Counts are the same for every lane
  // of every workgroup, so all decide alike.)
  const bool solo = units != nullptr && n_units < gridDim.x && n_items / 2 >= n_units;
  if (solo) {
    units = nullptr;
    n_chains = 0;
    n_units = n_items;
  }
  const uint32_t half = fl.head_dim / 2;
  const bool scout = threadIdx.x >= kMoveThreads;  // the fifth wavefront
  const uint32_t lane = threadIdx.x & (kWave - 1);

  // ---- mover lanes: geometry that does not change ----
  const uint32_t n_rows = fl.n_layers * 2;               // rows of one token: K, V of layer 0, K, V of layer 1, ..
  const uint32_t vpr = fl.n_kv_heads * fl.head_dim / 8;  // 16-byte vectors per row
  // lane t starts at vector t of the unit and advances by 256 vectors per step
  const uint32_t r_step = kMoveThreads / vpr, c_step = kMoveThreads % vpr;
  const uint32_t r_init = threadIdx.x / vpr, c_init = threadIdx.x % vpr;
  const uint32_t vph = fl.head_dim / 8;  // vectors per head
  // column of this lane inside its head: the same at every step, because the lane stride (256
  // vectors) and the row length are both multiples of the vectors per head
  const uint32_t cih = threadIdx.x % vph;
  const bool second = cih >= vph / 2;                                    // lane holds second-half elements of its head
  const uint32_t j_first = first_freq<RA::style>(fl.head_dim / 2, cih);  // its four frequencies start here
  const uint32_t steps = (n_rows * vpr + kMoveThreads - 1) / kMoveThreads;  // same for every lane
  // A rotating gather evens out who rotates: where a step of the 256 lanes covers whole (K, V) row pairs, a
  // lane's row parity never changes, so for the Llama shapes two wavefronts would rotate K rows all the time
  // while the other two only copy V rows.  Swapping K and V inside the pair on every other step of a round is
  // still a walk over every (row, column) once, and gives every wavefront half of the rotations.
  const uint32_t alternate = (ROPE && kMoveThreads % (2 * vpr) == 0) ? 1u : 0u;
  // With rows shorter than a wavefront's 1 KiB the lanes of one wavefront would hold K rows and V rows side by
  // side, and the wavefront would run the rotation with half of its lanes idle.  Where a step covers whole
  // (K, V) pairs, the rows of a step are therefore dealt out so that the first half of the workgroup holds the
  // step's K rows and the second half its V rows (a permutation inside the step's rows; nothing changes for
  // rows of 1 KiB and more).  row_shift = the lane's row under this rule minus its row in row-major order.
  uint32_t row_shift = 0;
  if (alternate) {
    const uint32_t pairs = r_step / 2;  // (K, V) pairs per step; r_init < r_step
    row_shift = 2 * (r_init % pairs) + r_init / pairs - r_init;
  }

  // ---- scout state (the same in all 64 lanes of the scout) ----
  uint32_t more_node = kNone, more_from = kNone;  // chain to continue in the next pass, and its source
  uint32_t mine = 0, mine_k = take;               // first unit of this scout's ticket, and how many of its units are done
  const uint32_t n_tickets = (n_units + take * kTicketStride - 1) / (take * kTicketStride) * kTicketStride;  // n_units < 2^31

  for (uint32_t turn = 0;; ++turn) {
    const uint32_t b = turn & 1u;
    if (scout) {
      // Describe the unit of turn `turn` into s_unit[b]; for turn 0 the movers wait at the barrier
      // below, afterwards they are moving the unit of turn - 1 out of s_unit[b ^ 1] meanwhile.
      uint32_t node = more_node, src = more_from;
      MoveItem first{kNone, kNone, 0, kNone};  // a new unit's first item, read while it was looked at
      bool have_first = false;
      if (node == kNone) {  // a new unit: the next one the counter hands out
        while (true) {
          if (mine_k == take) {  // a new ticket: `take` units, kTicketStride apart (see launch_move)
            uint32_t t = 0;
            if (lane == 0) t = atomicAdd(counter, 1u);
            t = __shfl(t, 0, kWave);
            if (t >= n_tickets) break;  // the counter only grows: every scout gets here
            mine = t / kTicketStride * (take * kTicketStride) + t % kTicketStride;
            mine_k = 0;
            // lane k fetches the first item of the ticket's k-th unit: the dependent loads (list entry, then item)
            // are paid once per ticket, side by side, not once per unit
            // (they wait in LDS, which only this wavefront touches: registers held across the movers' code
            // would cost every wavefront of the kernel its occupancy)
            if (lane < take) {
              const uint32_t i = mine + lane * kTicketStride;  // (the last group of tickets may reach past the end)
              uint32_t w = kNone;
              u32x4 it{kNone, kNone, 0u, kNone};  // a MoveItem's four words
              if (i < n_units) {
                w = units ? units[i < n_chains ? i : max_items - 1 - (i - n_chains)] : i;
                if (w < n_items) it = *reinterpret_cast<const u32x4 *>(&items[w]);
                else w = kNone;
              }
              s_ahead_w[lane] = w;
              *reinterpret_cast<u32x4 *>(&s_ahead[lane]) = it;
            }
            __builtin_amdgcn_wave_barrier();  // (LDS serves one wavefront's accesses in order)
          }
          const uint32_t k = mine_k++;
          const uint32_t w = s_ahead_w[k];
          if (w == kNone) continue;
          const MoveItem it = s_ahead[k];
          if (it.from == kNone) continue;  // an item that was taken out
          if (it.from >= n_from) {
            if (lane == 0) atomicOr(status_flags, CP_FLAG_BAD_INDEX);
            continue;
          }
          node = w;
          src = it.from;
          first = it;
          have_first = true;
          break;
        }
      }
      uint32_t K = 0;
      int32_t dl[kMaxFanout];
#pragma unroll
      for (uint32_t k = 0; k < kMaxFanout; ++k) {
        dl[k] = 0;
        if (k < fanout && node != kNone && node < n_items) {
          const MoveItem it = (k == 0 && have_first) ? first : items[node];
          dl[k] = it.delta;
          if (lane == 0) {
            s_unit[b].tobase[k] = (uint64_t)it.to * tl.tok_stride;
            s_unit[b].delta[k] = it.delta;
          }
          node = solo ? kNone : it.next;
          K = k + 1;
        }
      }
      more_node = (node != kNone && node < n_items) ? node : kNone;
      more_from = more_node != kNone ? src : kNone;
      if (lane == 0) {
        s_unit[b].from = K ? src : kNone;
        s_unit[b].k = K;
      }
      if (ROPE) {
#pragma unroll
        for (uint32_t k = 0; k < kMaxFanout; ++k) {
          if (k < K && dl[k] != 0) {
            for (uint32_t j = lane; j < half; j += kWave) {
              uint32_t a = dl[k] < 0 ? 0u - (uint32_t)dl[k] : (uint32_t)dl[k];  // |delta|, digit by digit
              double2 t = rope.tables[(a & (kTrigDigit - 1)) * half + j];
              double cs = t.x, sn = t.y;
#pragma unroll
              for (uint32_t level = 1; level < kTrigLevels; ++level) {
                a >>= 7;
                if (a == 0) break;  // all further digits are 0: their entries are (1, 0), which change nothing
                t = rope.tables[(level * kTrigDigit + (a & (kTrigDigit - 1))) * half + j];
                const double c2 = cs * t.x - sn * t.y;  // angles add: multiply the unit vectors
                sn = sn * t.x + cs * t.y;
                cs = c2;
              }
              s_cos[b][k * half + j] = cs;
              s_sin[b][k * half + j] = dl[k] < 0 ? -sn : sn;
            }
          }
        }
      }
    }
    __syncthreads();  // s_unit[b] is complete; nobody reads s_unit[b ^ 1] any more
    const uint32_t src = s_unit[b].from;
    if (src == kNone) break;  // same value in every lane of the workgroup
    if (scout) continue;      // on to the next unit's description
    const uint32_t K = s_unit[b].k;
    const uint8_t *fbase = from + (uint64_t)src * fl.tok_stride;
    uint8_t *to0 = to + s_unit[b].tobase[0];  // first destination: known before the loads are issued
    const bool rot0 = ROPE && s_unit[b].delta[0] != 0;
    uint32_t r = r_init, c = c_init;
    // One round: U loads per lane, then the stores.  The first destination's stores are straight-line
    // code right behind the loads (each waits only for its own load); further destinations of a chain
    // follow in a loop, when every load has arrived anyway.  FULL: every lane has U valid vectors.
    auto round = [&](auto full_tag) {
      constexpr bool FULL = decltype(full_tag)::value;
      u32x4 v[U];
      uint64_t doff[U];
      bool ok[U], is_k[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint32_t rp = r + row_shift;
        ok[u] = FULL || rp < n_rows;  // rp only grows, so the valid steps of a lane are a prefix
        const uint32_t rr = rp ^ (alternate & (uint32_t)u);  // (rounds start on even steps: U is even; n_rows is even)
        is_k[u] = (rr & 1u) == 0;
        const uint64_t l = rr >> 1, kv = rr & 1u;
        doff[u] = l * tl.layer_stride + kv * tl.kv_stride + (uint64_t)c * 16;
        v[u] = u32x4{0, 0, 0, 0};
        if (ok[u]) v[u] = load16<NTL>(fbase + l * fl.layer_stride + kv * fl.kv_stride + (uint64_t)c * 16);
        c += c_step;
        r += r_step;
        if (c >= vpr) {
          c -= vpr;
          r += 1;
        }
      }
      // all of the round's loads are in flight before anything waits for one of them: neither the
      // compiler nor the instruction scheduler may pair a load with its store
      asm volatile("" ::: "memory");
      __builtin_amdgcn_sched_barrier(0);
      Trig4 trig{};
      if (rot0) trig = load_trig(j_first, s_cos[b], s_sin[b]);
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (!ok[u]) continue;
        u32x4 x = v[u];
        if (ROPE && is_k[u]) {
          // a lane and its partner are in the same row, so both are here for the exchanges
          if (rot0) x = rotate_pairs<RA::style>(widen_pairs<RA::style>(v[u], second, (int)(vph / 2)), trig, second,
                                                (int)(vph / 2));
        }
        store16<NTS>(to0 + doff[u], x);
      }
      for (uint32_t k = 1; k < K; ++k) {
        uint8_t *tk = to + s_unit[b].tobase[k];
        const bool rot = ROPE && s_unit[b].delta[k] != 0;
        if (rot) trig = load_trig(j_first, s_cos[b] + k * half, s_sin[b] + k * half);
#pragma unroll
        for (int u = 0; u < U; ++u) {
          if (!ok[u]) continue;
          u32x4 x = v[u];
          // (the double-precision copies are made again per destination: keeping them for all U vectors
          // would cost the registers that let more wavefronts stay resident)
          if (ROPE && is_k[u] && rot)
            x = rotate_pairs<RA::style>(widen_pairs<RA::style>(v[u], second, (int)(vph / 2)), trig, second,
                                        (int)(vph / 2));
          store16<NTS>(tk + doff[u], x);
        }
      }
    };
    const uint32_t full_steps = (n_rows * vpr) / (kMoveThreads * U) * U;  // steps of whole rounds in which every lane works
    uint32_t j = 0;
    for (; j < full_steps; j += U) round(std::true_type{});
    for (; j < steps; j += U) round(std::false_type{});
  }
}

// The two users of the mover get kernels of their own name, so that profiles tell them apart.
template <class RA, bool ROPE, bool NTL, bool NTS, int U>
__global__ __launch_bounds__(kBlockThreads) void gather_rows_kernel(
    const MoveItem *__restrict__ items, const uint32_t *__restrict__ n_items_ptr, uint32_t max_items,
    const uint32_t *__restrict__ units, const uint32_t *__restrict__ unit_counts, uint32_t *counter,
    const uint8_t *__restrict__ pool, cp_kv_layout pool_l, uint32_t n_pool_slots, uint8_t *__restrict__ dst,
    cp_kv_layout dst_l, uint32_t fanout, uint32_t take, uint32_t *status_flags, RA rope) {
  move_rows_body<RA, ROPE, NTL, NTS, U>(items, n_items_ptr, max_items, units, unit_counts, counter, pool, pool_l,
                                        n_pool_slots, dst, dst_l, fanout, take, status_flags, rope);
}

template <class RA, bool ROPE, bool NTL, bool NTS, int U>
__global__ __launch_bounds__(kBlockThreads) void scatter_rows_kernel(
    const MoveItem *__restrict__ items, const uint32_t *__restrict__ n_items_ptr, uint32_t max_items,
    const uint32_t *__restrict__ units, const uint32_t *__restrict__ unit_counts, uint32_t *counter,
    const uint8_t *__restrict__ src, cp_kv_layout src_l, uint32_t n_src_tokens, uint8_t *__restrict__ pool,
    cp_kv_layout pool_l, uint32_t fanout, uint32_t take, uint32_t *status_flags, RA rope) {
  move_rows_body<RA, ROPE, NTL, NTS, U>(items, n_items_ptr, max_items, units, unit_counts, counter, src, src_l,
                                        n_src_tokens, pool, pool_l, fanout, take, status_flags, rope);
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
                    const uint32_t *units, const uint32_t *unit_counts, uint32_t *counter, const void *from,
                    const cp_kv_layout &fl, uint32_t n_from, void *to, const cp_kv_layout &tl, uint32_t *status_flags,
                    const RA &rope, const MoveOpts &mo) {
  if (max_items == 0) return CP_OK;
  if (mo.start && hipEventRecord(mo.start, stream) != hipSuccess) return CP_ERR_HIP;
  // Defaults, measured on MI355X with the Llama row shapes.  Copy form: 16 loads in flight per lane and
  // one workgroup on seven of every eight compute units (224 of 256; one per unit is 1 % slower, two per
  // unit with 8 loads 3-6 % slower).  Rotating form: 8 loads in flight (165 registers), two workgroups per
  // unit; with every wavefront taking half of the rotations (see `alternate` in the mover) that is 3 % faster
  // than 4 loads and within 2 % of the copy form on the same spans.  Small tokens get as many loads as they
  // have steps for.
  const uint64_t steps = div_up((uint64_t)fl.n_layers * 2 * (fl.n_kv_heads * fl.head_dim / 8), kMoveThreads);
  uint32_t lif = mo.loads_in_flight ? mo.loads_in_flight
                 : ROPE             ? (steps >= 16 ? 8u : 4u)
                                    : (steps >= 32 ? 16u : steps >= 16 ? 8u : 4u);
  if (ROPE && lif > 8) lif = 8;  // the rotating form is not built with 16: it needs its registers for arithmetic
  const uint32_t cus = cu_count();
  uint64_t grid = mo.workgroups      ? mo.workgroups
                  : mo.blocks_per_cu ? (uint64_t)cus * mo.blocks_per_cu
                  : ROPE             ? (uint64_t)cus * 2
                  : lif >= 16        ? cus - cus / 8
                                     : (uint64_t)cus * 2;
  if (grid > max_items) grid = max_items;
  uint32_t fanout = mo.fanout < kMaxFanout ? mo.fanout : kMaxFanout;
  if (ROPE) {
    uint32_t cap = kTrigDoubles / (fl.head_dim / 2);
    if (fanout > cap) fanout = cap;
  }
  // Units per ticket of the work counter.  Every workgroup of the chip adds to that one word, and such additions
  // go through at about 80 per microsecond in all: enough for tokens of 64 KiB and more, a cap on the whole kernel
  // for small ones (16 KiB tokens need 170 units per microsecond to keep HBM busy).  For small tokens a ticket
  // is therefore worth several units, about 24 steps of the 256 lanes.  Ticket t of a group of kTicketStride
  // tickets stands for units t, t + kTicketStride, t + 2 kTicketStride, .. of the group's stretch of the list: the workgroups
  // that run at the same time are then still on neighbouring units (neighbouring destination rows), as with
  // one unit per ticket, which consecutive units per ticket would give up (5 % slower on 40 KiB tokens).
  const uint32_t take = steps >= 24 ? 1u : (uint32_t)(24 / steps) < kMaxTake ? (uint32_t)(24 / steps) : kMaxTake;
  const uint8_t *f = (const uint8_t *)from;
  uint8_t *t = (uint8_t *)to;
#define CP_LAUNCH(NTL, NTS, UN)                                                                              \
  if constexpr (GATHER)                                                                                      \
    gather_rows_kernel<RA, ROPE, NTL, NTS, UN><<<(uint32_t)grid, kBlockThreads, 0, stream>>>(                 \
        items, n_items, max_items, units, unit_counts, counter, f, fl, n_from, t, tl, fanout, take, status_flags, rope); \
  else                                                                                                       \
    scatter_rows_kernel<RA, ROPE, NTL, NTS, UN><<<(uint32_t)grid, kBlockThreads, 0, stream>>>(                \
        items, n_items, max_items, units, unit_counts, counter, f, fl, n_from, t, tl, fanout, take, status_flags, rope)
  switch ((mo.nontemporal & 3u) | (lif >= 16 ? 8u : lif >= 8 ? 4u : 0u)) {
    case 0: CP_LAUNCH(false, false, 4); break;
    case 1: CP_LAUNCH(true, false, 4); break;
    case 2: CP_LAUNCH(false, true, 4); break;
    case 3: CP_LAUNCH(true, true, 4); break;
    case 4: CP_LAUNCH(false, false, 8); break;
    case 5: CP_LAUNCH(true, false, 8); break;
    case 6: CP_LAUNCH(false, true, 8); break;
    case 7: CP_LAUNCH(true, true, 8); break;
    default:
      if constexpr (!ROPE) {
        switch (mo.nontemporal & 3u) {
          case 0: CP_LAUNCH(false, false, 16); break;
          case 1: CP_LAUNCH(true, false, 16); break;
          case 2: CP_LAUNCH(false, true, 16); break;
          default: CP_LAUNCH(true, true, 16); break;
        }
      }
      break;
  }
#undef CP_LAUNCH
  if (int32_t rc = check_launch()) return rc;
  if (mo.stop && hipEventRecord(mo.stop, stream) != hipSuccess) return CP_ERR_HIP;
  return CP_OK;
}

}  // namespace

int32_t launch_scatter(hipStream_t stream, const void *src, const cp_kv_layout &src_l, uint32_t n_src_tokens,
                       void *pool, const cp_kv_layout &pool_l, uint32_t n_pool_slots, const MoveItem *items,
                       const uint32_t *n_items, uint32_t max_items, uint32_t *counter, uint32_t *status_flags,
                       const MoveOpts &mo) {
  NoRope none{};
  (void)n_pool_slots;  // the commit step has checked every slot it put on the list
  return launch_move<NoRope, false, false>(stream, items, n_items, max_items, nullptr, nullptr, counter, src, src_l,
                                           n_src_tokens, pool, pool_l, status_flags, none, mo);
}

}  // namespace cp

namespace cp {
namespace {

int32_t gather_impl(hipStream_t stream, const void *pool, const cp_kv_layout &pool_l, uint32_t n_pool_slots, void *dst,
                    const cp_kv_layout &dst_l, uint32_t n_dst_tokens, const uint32_t *span_src,
                    const uint32_t *span_dst, const uint32_t *span_len, const int32_t *span_delta,
                    const uint32_t *span_off, const uint32_t *n_spans, uint32_t max_spans, const cp_rope *rope,
                    uint32_t *status_flags, void *work, size_t work_bytes, const cp_launch_opts *opts) {
  if (n_dst_tokens >= 0x80000000u || n_pool_slots >= 0x80000000u) return CP_ERR_UNSUPPORTED;
  if (!pool || !dst || !span_src || !span_dst || !span_len || !n_spans || !status_flags) return CP_ERR_INVALID_ARG;
  if (!aligned(pool, 16) || !aligned(dst, 16)) return CP_ERR_INVALID_ARG;
  if (!layout_ok(pool_l) || !layout_ok(dst_l) || !layouts_match(pool_l, dst_l)) return CP_ERR_UNSUPPORTED;
  const bool use_rope = rope != nullptr && span_delta != nullptr;
  if (use_rope) {
    const uint32_t D = pool_l.head_dim;
    // pairs must not straddle 16-byte vectors or wavefronts: power-of-two head_dim in [16, 512]
    if (D < 16 || D > 2 * kMaxHalfDim || (D & (D - 1))) return CP_ERR_UNSUPPORTED;
    if (rope->style > 1 || !(rope->theta > 0.0)) return CP_ERR_INVALID_ARG;
  }
  MoveOpts mo;
  if (!resolve_opts(opts, use_rope, &mo)) return CP_ERR_INVALID_ARG;
  // a small batch is bound by its launches, not by its bytes: grouping (two more launches) is left out
  if ((!opts || opts->read_sharing == 0) && n_dst_tokens < kShareReadsFrom) mo.share_reads = false;
  if (work_bytes < scratch_bytes_for(n_dst_tokens, max_spans, n_pool_slots)) return CP_ERR_SCRATCH;
  Scratch sc(work, work_bytes);
  uint32_t *agg = sc.take<uint32_t>(div_up(max_spans, kScanTile) + 1);
  uint32_t *offs = sc.take<uint32_t>((size_t)max_spans + 1);
  uint32_t *counters = sc.take<uint32_t>(4);  // [0] work counter, [1] item count, [2] chains and [3] single tokens on the work list
  MoveItem *items = sc.take<MoveItem>(n_dst_tokens);
  const bool group = mo.share_reads;
  uint32_t *head = group ? sc.take<uint32_t>(n_pool_slots) : nullptr;
  uint32_t *units = group ? sc.take<uint32_t>(n_dst_tokens) : nullptr;
  double2 *tables = use_rope ? sc.take<double2>((size_t)kTrigLevels * kTrigDigit * (pool_l.head_dim / 2)) : nullptr;
  if (!agg || !offs || !counters || !items || (group && (!head || !units)) || (use_rope && !tables)) return CP_ERR_SCRATCH;
  if (use_rope) {
    InvFreq inv{};
    const uint32_t D = pool_l.head_dim;
    for (uint32_t j = 0; j < D / 2; ++j) inv.v[j] = std::pow(rope->theta, -2.0 * (double)j / (double)D);
    rope_tables_kernel<<<div_up((uint64_t)kTrigLevels * kTrigDigit * (D / 2), 256), 256, 0, stream>>>(inv, D / 2, tables);
  }
  if (!span_off) {
    if (int32_t rc = launch_span_offsets(stream, span_len, n_spans, max_spans, offs, agg)) return rc;
    span_off = offs;
  }
  if (group) gather_init_kernel<<<div_up(n_pool_slots, 256), 256, 0, stream>>>(head, n_pool_slots, counters);
  // spans do not overlap in dst, so they cover at most n_dst_tokens tokens
  gather_expand_kernel<<<div_up(n_dst_tokens, 256), 256, 0, stream>>>(
      span_src, span_dst, span_off, use_rope ? span_delta : nullptr, n_spans, max_spans, n_pool_slots, n_dst_tokens,
      items, head, counters, status_flags);
  if (group)
    gather_heads_kernel<<<div_up(n_dst_tokens, 256), 256, 0, stream>>>(items, counters + 1, n_dst_tokens, head, units,
                                                                       counters + 2);
  if (int32_t rc = check_launch()) return rc;
  if (use_rope && rope->style == 0)
    return launch_move<RopeArg<0>, true, true>(stream, items, counters + 1, n_dst_tokens, units, counters + 2, counters,
                                               pool, pool_l, n_pool_slots, dst, dst_l, status_flags, RopeArg<0>{tables},
                                               mo);
  if (use_rope)
    return launch_move<RopeArg<1>, true, true>(stream, items, counters + 1, n_dst_tokens, units, counters + 2, counters,
                                               pool, pool_l, n_pool_slots, dst, dst_l, status_flags, RopeArg<1>{tables},
                                               mo);
  NoRope none{};
  return launch_move<NoRope, false, true>(stream, items, counters + 1, n_dst_tokens, units, counters + 2, counters, pool,
                                          pool_l, n_pool_slots, dst, dst_l, status_flags, none, mo);
}

// ---- the entry point that brings its own scratch memory -----------------------------------------

// Largest call cp_gather_kv_static accepts, and the scratch it needs for that.
constexpr uint32_t kStaticMaxTokens = CP_STATIC_MAX_TOKENS, kStaticMaxSpans = CP_STATIC_MAX_SPANS,
                   kStaticMaxSlots = CP_STATIC_MAX_SLOTS;
constexpr size_t kStaticScratchBytes = 10u << 20;
static_assert(scratch_bytes_for(kStaticMaxTokens, kStaticMaxSpans, kStaticMaxSlots) <= kStaticScratchBytes,
              "the static scratch array must hold the largest accepted call");
constexpr int kMaxDevices = 64;

}  // namespace
}  // namespace cp

// Device memory that exists from the moment the code object is loaded on a GPU until the process
// ends, one copy per GPU.  In host code this name is only a handle for hipGetSymbolAddress; the
// array's address on the current GPU is looked up once and used from then on.
static __device__ __align__(256) uint8_t scratch[cp::kStaticScratchBytes];

namespace cp {
namespace {

// Address of `scratch` on the current device (looked up once per device), or null with *rc set.
void *static_scratch(int32_t *rc) {
  static std::mutex mu;
  static void *ptr[kMaxDevices] = {};
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess && (dev < 0 || dev >= kMaxDevices)) e = hipErrorInvalidDevice;
  if (e == hipSuccess) {
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
      void *p = nullptr;
      e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
      if (e == hipSuccess && !p) e = hipErrorInvalidSymbol;
      if (e == hipSuccess) ptr[dev] = p;
    }
    if (e == hipSuccess) return ptr[dev];
  }
  last_hip_error() = (int32_t)e;
  *rc = CP_ERR_HIP;
  return nullptr;
}

}  // namespace
}  // namespace cp

extern "C" int32_t cp_gather_kv(void *stream, const void *pool, cp_kv_layout pool_l, uint32_t n_pool_slots, void *dst,
                                cp_kv_layout dst_l, uint32_t n_dst_tokens, const uint32_t *span_src,
                                const uint32_t *span_dst, const uint32_t *span_len, const int32_t *span_delta,
                                const uint32_t *span_off, const uint32_t *n_spans, uint32_t max_spans,
                                const cp_rope *rope, uint32_t *status_flags, void *scratch_arg, size_t scratch_bytes,
                                const cp_launch_opts *opts) {
  if (max_spans == 0 || n_dst_tokens == 0 || n_pool_slots == 0) return CP_OK;
  if (!scratch_arg || !cp::aligned(scratch_arg, 256)) return CP_ERR_INVALID_ARG;
  return cp::gather_impl((hipStream_t)stream, pool, pool_l, n_pool_slots, dst, dst_l, n_dst_tokens, span_src, span_dst,
                         span_len, span_delta, span_off, n_spans, max_spans, rope, status_flags, scratch_arg,
                         scratch_bytes, opts);
}

extern "C" int32_t cp_gather_kv_static(void *stream, const void *pool, cp_kv_layout pool_l, uint32_t n_pool_slots,
                                       void *dst, cp_kv_layout dst_l, uint32_t n_dst_tokens, const uint32_t *span_src,
                                       const uint32_t *span_dst, const uint32_t *span_len, const int32_t *span_delta,
                                       const uint32_t *span_off, const uint32_t *n_spans, uint32_t max_spans,
                                       const cp_rope *rope, uint32_t *status_flags, const cp_launch_opts *opts) {
  using namespace cp;
  if (max_spans == 0 || n_dst_tokens == 0 || n_pool_slots == 0) return CP_OK;
  if (n_dst_tokens > kStaticMaxTokens || max_spans > kStaticMaxSpans || n_pool_slots > kStaticMaxSlots)
    return CP_ERR_STATIC_LIMIT;
  int32_t rc = CP_OK;
  void *mem = static_scratch(&rc);  // the array's address on this GPU, never the array's name
  if (!mem) return rc;
  return gather_impl((hipStream_t)stream, pool, pool_l, n_pool_slots, dst, dst_l, n_dst_tokens, span_src, span_dst,
                     span_len, span_delta, span_off, n_spans, max_spans, rope, status_flags, mem, kStaticScratchBytes,
                     opts);
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
  return cp::scratch_bytes_for(N, max_spans, n_pool_slots);
}

extern "C" int32_t cp_last_hip_error(void) { return cp::last_hip_error(); }

// Pool policies on top of the lookup / insert path:
//   cp_filter_matches   minimum segment length (Sec. 4.2.1 "Optimization") and recompute marks
//                       (Sec. 4.2.1 Step 3: marked tokens of a reused segment are recomputed)
//   cp_mark_recompute   per-slot recompute marks, set when tokens are stored
//   cp_fill_unmatched   zero placeholders for tokens that are not linked (Sec. 4.3.1
//                       "Operational details")
//   cp_touch, cp_lru_threshold, cp_evict, cp_table_compact
//                       least-recently-used eviction (Sec. 4.3.5 "Lifecycle management")
//
// A "stretch" is a maximal run of consecutive positions of one request that have a slot.  Its
// length at every token is (tokens of the stretch before it) + (after it) + 1: one ordered scan
// forwards and one backwards over the same monoid (count since the last break).
#include "cp_device.h"
#include "cp_internal.h"

namespace cp {
namespace {

constexpr uint32_t kNone = 0xFFFFFFFFu;
constexpr uint32_t kBreak = 0x80000000u;  // bit 31 of the scan value: the piece contains a break

// Count of elements since the last break.  Value = count | (break seen ? kBreak : 0).
struct CountSinceBreak {
  using T = uint32_t;
  static __device__ __forceinline__ T identity() { return 0u; }
  static __device__ __forceinline__ T combine(T f, T g) { return (g & kBreak) ? g : f + g; }
};

// Forwards: before[i] = matched tokens of i's stretch in front of i (kNone if i has no slot).
struct StretchFwdOp : CountSinceBreak {
  const uint32_t *slot;
  const uint32_t *off;
  uint32_t *before;
  uint32_t N, R;
  __device__ __forceinline__ uint32_t count() const { return N; }
  __device__ __forceinline__ T load(uint32_t i) const {
    if (slot[i] == kNone) return kBreak;  // count 0, and nothing carries over it
    const bool start = off[request_of(off, R, i)] == i;
    return 1u | (start ? kBreak : 0u);
  }
  __device__ __forceinline__ void store(uint32_t i, T, T incl) const {
    before[i] = slot[i] == kNone ? kNone : (incl & ~kBreak) - 1u;
  }
  __device__ __forceinline__ void finish(T) const {}
};

// Backwards (element e of the scan is token N-1-e): tokens of the stretch behind the token; then the
// decision.  Token i+1 continues i's stretch iff before[i+1] == before[i] + 1.
struct StretchBwdOp : CountSinceBreak {
  const uint32_t *before;
  const uint32_t *slot_in;
  const uint8_t *slot_recompute;  // nullable
  uint32_t *slot_out;
  uint32_t N, n_pool_slots, min_len;
  __device__ __forceinline__ uint32_t count() const { return N; }
  __device__ __forceinline__ T load(uint32_t e) const {
    const uint32_t i = N - 1 - e;
    const uint32_t b = before[i];
    if (b == kNone) return kBreak;
    const bool last = i + 1 == N || before[i + 1] != b + 1;  // kNone + ... never equals b + 1 for b < 2^31
    return 1u | (last ? kBreak : 0u);
  }
  __device__ __forceinline__ void store(uint32_t e, T, T incl) const {
    const uint32_t i = N - 1 - e;
    const uint32_t b = before[i], s = slot_in[i];
    uint32_t r = kNone;
    if (b != kNone) {
      const uint32_t len = b + (incl & ~kBreak);  // before + (after + 1)
      bool keep = len >= min_len;
      if (keep && slot_recompute && s < n_pool_slots && slot_recompute[s]) keep = false;
      if (keep) r = s;
    }
    slot_out[i] = r;
  }
  __device__ __forceinline__ void finish(T) const {}
};

__global__ __launch_bounds__(256) void mark_recompute_kernel(const uint32_t *__restrict__ slot,
                                                             const uint8_t *__restrict__ recompute, uint32_t N,
                                                             uint32_t n_pool_slots, uint8_t *slot_recompute) {
  uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < N && recompute[i] && slot[i] < n_pool_slots) slot_recompute[slot[i]] = 1;  // every writer writes 1
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Workgroup b takes tokens b, b + grid, ...: unmatched tokens come in long stretches (a request's own
// text), striding spreads them over the grid.  All rows of an unmatched token are set to zero with
// 16-byte non-temporal stores; the 256 lanes walk the token's (row, 16-byte column) space row-major, so
// every lane stores at every step whatever the row length.
__global__ __launch_bounds__(256) void fill_unmatched_kernel(const uint32_t *__restrict__ slot, uint32_t N,
                                                             uint8_t *__restrict__ dst, cp_kv_layout l) {
  const uint32_t vpr = l.n_kv_heads * l.head_dim * 2 / 16;  // vectors per row
  const uint32_t n_vec = l.n_layers * 2 * vpr;
  const uint32_t r_step = 256 / vpr, c_step = 256 % vpr;
  const u32x4 zero = {0u, 0u, 0u, 0u};
  for (uint32_t t = blockIdx.x; t < N; t += gridDim.x) {
    if (slot[t] != kNone) continue;  // same for the whole workgroup
    uint8_t *tok = dst + (uint64_t)t * l.tok_stride;
    uint32_t r = threadIdx.x / vpr, c = threadIdx.x % vpr;
    for (uint32_t v = threadIdx.x; v < n_vec; v += 256) {
      uint8_t *p = tok + (uint64_t)(r >> 1) * l.layer_stride + (uint64_t)(r & 1) * l.kv_stride + (uint64_t)c * 16;
      __builtin_nontemporal_store(zero, (u32x4 *)p);
      r += r_step, c += c_step;
      if (c >= vpr) c -= vpr, r += 1;
    }
  }
}

__global__ __launch_bounds__(256) void touch_kernel(const uint32_t *__restrict__ slot, uint32_t N, uint32_t epoch,
                                                    uint32_t n_pool_slots, uint32_t *slot_stamp) {
  uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < N && slot[i] < n_pool_slots) atomicMax(&slot_stamp[slot[i]], epoch);
}

// ---- LRU threshold: histogram of ages, then the oldest cohorts until enough ----

__global__ __launch_bounds__(256) void zero_words_kernel(uint32_t *p, uint32_t n) {
  uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

// Histogram of slot ages, the last bin open-ended.  Right after a few large batches nearly all slots share a
// handful of ages, so plain atomics would queue up on a few words: the lanes of a wavefront that hold the same
// age add once, into a histogram in LDS, and every workgroup adds its non-empty bins to the global one at the end.
__global__ __launch_bounds__(256) void age_histogram_kernel(const uint32_t *__restrict__ slot_stamp,
                                                            uint32_t n_pool_slots, uint32_t epoch_now, uint32_t *hist) {
  __shared__ uint32_t local[CP_LRU_MAX_AGE];
  for (uint32_t a = threadIdx.x; a < CP_LRU_MAX_AGE; a += blockDim.x) local[a] = 0;
  __syncthreads();
  const uint32_t lane = threadIdx.x & (kWave - 1);
  for (uint32_t base = blockIdx.x * blockDim.x; base < n_pool_slots; base += gridDim.x * blockDim.x) {
    const uint32_t s = base + threadIdx.x;  // base is the same for the whole workgroup
    uint32_t bin = kNone;
    if (s < n_pool_slots) {
      const uint32_t st = slot_stamp[s];
      if (st != 0 && st <= epoch_now) {  // else free, or stamped in the future: never chosen
        const uint32_t age = epoch_now - st;
        bin = age < CP_LRU_MAX_AGE - 1 ? age : CP_LRU_MAX_AGE - 1;
      }
    }
    bool todo = bin != kNone;
    unsigned long long left = __ballot(todo);
    while (left) {  // the same for the whole wavefront; every round retires at least one lane
      const uint32_t first = (uint32_t)__ffsll(left) - 1;
      const uint32_t b = __builtin_amdgcn_readlane(bin, first);
      const unsigned long long same = __ballot(todo && bin == b);
      if (lane == first) atomicAdd(&local[b], (uint32_t)__popcll(same));
      if (bin == b) todo = false;
      left = __ballot(todo);
    }
  }
  __syncthreads();
  for (uint32_t a = threadIdx.x; a < CP_LRU_MAX_AGE; a += blockDim.x)
    if (local[a]) atomicAdd(&hist[a], local[a]);
}

// One workgroup.  Largest age a such that the slots of age >= a are at least n_needed; threshold =
// epoch_now - a + 1 (a slot goes iff its stamp is below the threshold).
__global__ __launch_bounds__(256) void lru_pick_kernel(const uint32_t *__restrict__ hist, uint32_t max_age,
                                                       uint32_t epoch_now, uint32_t n_needed, uint32_t *threshold_out) {
  __shared__ uint32_t part[256];
  __shared__ uint32_t found_age;
  const uint32_t per = (max_age + 255) / 256;  // ages handled by one thread; thread 0 holds the oldest
  // thread k covers ages  max_age-1 - k*per  down to  max_age - (k+1)*per
  uint32_t sum = 0;
  for (uint32_t j = 0; j < per; ++j) {
    const int64_t a = (int64_t)max_age - 1 - (int64_t)threadIdx.x * per - j;
    if (a >= 0) sum += hist[a];
  }
  part[threadIdx.x] = sum;
  if (threadIdx.x == 0) found_age = kNone;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint64_t older = 0;  // slots older than everything thread k covers
    for (uint32_t k = 0; k < 256 && found_age == kNone; ++k) {
      if (older + part[k] >= n_needed) {  // the boundary lies among thread k's ages
        for (uint32_t j = 0; j < per; ++j) {
          const int64_t a = (int64_t)max_age - 1 - (int64_t)k * per - j;
          if (a < 0) break;
          older += hist[a];
          if (older >= n_needed) {
            found_age = (uint32_t)a;
            break;
          }
        }
      } else {
        older += part[k];
      }
    }
    uint32_t T;
    if (n_needed == 0) T = 0;
    else if (found_age == kNone) T = epoch_now + 1;
    else T = epoch_now - found_age + 1;
    *threshold_out = T;
  }
}

// ---- eviction ----

// Ordered compaction of the slots that go: freed[rank] = s in ascending slot order.
struct EvictOp {
  using T = uint32_t;
  const uint32_t *slot_stamp;
  const uint32_t *threshold;
  uint32_t *freed;
  uint32_t *n_freed;
  uint32_t n_pool_slots;
  static __device__ __forceinline__ T identity() { return 0u; }
  static __device__ __forceinline__ T combine(T a, T b) { return a + b; }
  __device__ __forceinline__ uint32_t count() const { return n_pool_slots; }
  __device__ __forceinline__ T load(uint32_t s) const {
    const uint32_t st = slot_stamp[s];
    return (st != 0 && st < *threshold) ? 1u : 0u;
  }
  __device__ __forceinline__ void store(uint32_t s, T excl, T incl) const {
    if (incl != excl) freed[excl] = s;
  }
  __device__ __forceinline__ void finish(T total) const { *n_freed = total; }
};

// The key of an evicted slot stays in the table with the value "absent": a later insert of the same
// key takes the entry over, lookups treat it as a miss.
__global__ __launch_bounds__(256) void evict_table_kernel(cp_table t, const uint32_t *__restrict__ slot_stamp,
                                                          const uint32_t *__restrict__ threshold,
                                                          uint32_t n_pool_slots) {
  uint64_t e = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= t.capacity) return;
  const uint32_t v = t.vals[e];
  if (v >= n_pool_slots) return;
  const uint32_t st = slot_stamp[v];
  if (st != 0 && st < *threshold) t.vals[e] = CP_SLOT_NONE;
}

__global__ __launch_bounds__(256) void evict_slots_kernel(uint32_t *slot_stamp, const uint32_t *__restrict__ threshold,
                                                          uint32_t n_pool_slots, uint32_t *slot_parent,
                                                          uint8_t *slot_recompute, uint8_t *slot_anchor) {
  uint32_t s = blockIdx.x * blockDim.x + threadIdx.x;
  if (s >= n_pool_slots) return;
  const uint32_t st = slot_stamp[s];
  if (st == 0 || st >= *threshold) return;
  slot_stamp[s] = 0;
  if (slot_parent) slot_parent[s] = CP_PARENT_POISON;
  if (slot_recompute) slot_recompute[s] = 0;
  if (slot_anchor) slot_anchor[s] = 0;
}

}  // namespace
}  // namespace cp

extern "C" int32_t cp_filter_matches(void *stream_, const uint32_t *slot_in, const uint32_t *off, uint32_t N, uint32_t R,
                                     uint32_t min_len, const uint8_t *slot_recompute, uint32_t n_pool_slots,
                                     uint32_t *slot_out, void *scratch, size_t scratch_bytes) {
  using namespace cp;
  hipStream_t stream = (hipStream_t)stream_;
  if (N == 0) return CP_OK;
  if (N >= 0x80000000u) return CP_ERR_UNSUPPORTED;
  if (!slot_in || !off || R == 0 || !slot_out || !scratch || !aligned(scratch, 256)) return CP_ERR_INVALID_ARG;
  if (scratch_bytes < cp_scratch_bytes(N, 0, 0)) return CP_ERR_SCRATCH;
  Scratch sc(scratch, scratch_bytes);
  uint32_t *agg = sc.take<uint32_t>(div_up(N, kScanTile) + 1);
  uint32_t *before = sc.take<uint32_t>(N);
  if (!agg || !before) return CP_ERR_SCRATCH;
  StretchFwdOp fwd{{}, slot_in, off, before, N, R};
  if (int32_t rc = run_scan<StretchFwdOp>(stream, fwd, N, agg)) return rc;
  StretchBwdOp bwd{{}, before, slot_in, slot_recompute, slot_out, N, n_pool_slots, min_len};
  return run_scan<StretchBwdOp>(stream, bwd, N, agg);
}

extern "C" int32_t cp_mark_recompute(void *stream, const uint32_t *slot, const uint8_t *recompute, uint32_t N,
                                     uint32_t n_pool_slots, uint8_t *slot_recompute) {
  using namespace cp;
  if (N == 0) return CP_OK;
  if (!slot || !recompute || !slot_recompute) return CP_ERR_INVALID_ARG;
  mark_recompute_kernel<<<div_up(N, 256), 256, 0, (hipStream_t)stream>>>(slot, recompute, N, n_pool_slots,
                                                                         slot_recompute);
  return check_launch();
}

extern "C" int32_t cp_fill_unmatched(void *stream, const uint32_t *slot, uint32_t N, void *dst, cp_kv_layout dst_l) {
  using namespace cp;
  if (N == 0) return CP_OK;
  if (!slot || !dst || !aligned(dst, 16)) return CP_ERR_INVALID_ARG;
  if (!layout_ok(dst_l)) return CP_ERR_UNSUPPORTED;
  const uint32_t grid = N < 256u * 8u ? N : 256u * 8u;
  fill_unmatched_kernel<<<grid, 256, 0, (hipStream_t)stream>>>(slot, N, (uint8_t *)dst, dst_l);
  return check_launch();
}

extern "C" int32_t cp_touch(void *stream, const uint32_t *slot, uint32_t N, uint32_t epoch, uint32_t n_pool_slots,
                            uint32_t *slot_stamp) {
  using namespace cp;
  if (N == 0) return CP_OK;
  if (!slot || !slot_stamp || epoch == 0) return CP_ERR_INVALID_ARG;
  touch_kernel<<<div_up(N, 256), 256, 0, (hipStream_t)stream>>>(slot, N, epoch, n_pool_slots, slot_stamp);
  return check_launch();
}

extern "C" int32_t cp_lru_threshold(void *stream_, const uint32_t *slot_stamp, uint32_t n_pool_slots,
                                    uint32_t epoch_now, uint32_t n_needed, uint32_t *threshold_out, void *scratch,
                                    size_t scratch_bytes) {
  using namespace cp;
  hipStream_t stream = (hipStream_t)stream_;
  if (!slot_stamp || !threshold_out || !scratch || !aligned(scratch, 256)) return CP_ERR_INVALID_ARG;
  if (epoch_now >= 0x7FFFFFFFu) return CP_ERR_UNSUPPORTED;
  Scratch sc(scratch, scratch_bytes);
  uint32_t *hist = sc.take<uint32_t>(CP_LRU_MAX_AGE);
  if (!hist) return CP_ERR_SCRATCH;
  zero_words_kernel<<<div_up(CP_LRU_MAX_AGE, 256), 256, 0, stream>>>(hist, CP_LRU_MAX_AGE);
  if (n_pool_slots)
    age_histogram_kernel<<<std::min<uint32_t>(div_up(n_pool_slots, 256), 512), 256, 0, stream>>>(slot_stamp, n_pool_slots,
                                                                                                 epoch_now, hist);
  lru_pick_kernel<<<1, 256, 0, stream>>>(hist, CP_LRU_MAX_AGE, epoch_now, n_needed, threshold_out);
  return check_launch();
}

extern "C" int32_t cp_evict(void *stream_, cp_table table, uint32_t *slot_stamp, uint32_t n_pool_slots,
                            const uint32_t *threshold, uint32_t *freed_slots, uint32_t *n_freed, uint32_t *slot_parent,
                            uint8_t *slot_recompute, uint8_t *slot_anchor, void *scratch, size_t scratch_bytes) {
  using namespace cp;
  hipStream_t stream = (hipStream_t)stream_;
  if (!table.keys || !table.vals || table.capacity == 0 || table.capacity % CP_TABLE_BUCKET) return CP_ERR_INVALID_ARG;
  if (!slot_stamp || !threshold || !freed_slots || !n_freed || !scratch || !aligned(scratch, 256))
    return CP_ERR_INVALID_ARG;
  if (n_pool_slots >= 0x80000000u) return CP_ERR_UNSUPPORTED;
  Scratch sc(scratch, scratch_bytes);
  uint32_t *agg = sc.take<uint32_t>(div_up(n_pool_slots, kScanTile) + 1);
  if (!agg) return CP_ERR_SCRATCH;
  EvictOp op{slot_stamp, threshold, freed_slots, n_freed, n_pool_slots};
  if (int32_t rc = run_scan<EvictOp>(stream, op, n_pool_slots, agg)) return rc;
  evict_table_kernel<<<div_up(table.capacity, 256), 256, 0, stream>>>(table, slot_stamp, threshold, n_pool_slots);
  if (n_pool_slots)
    evict_slots_kernel<<<div_up(n_pool_slots, 256), 256, 0, stream>>>(slot_stamp, threshold, n_pool_slots, slot_parent,
                                                                      slot_recompute, slot_anchor);
  return check_launch();
}

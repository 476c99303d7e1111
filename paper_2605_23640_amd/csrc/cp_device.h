// Device-side building blocks shared by the kernels of libcacheprune:
// an ordered scan over a user-defined monoid, request lookup, and
// launch / error plumbing.  gfx950 only (64-lane wavefronts).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/cacheprune.h"

namespace cp {

constexpr int kWave = 64;
constexpr int kScanThreads = 256;
constexpr int kScanItems = 1;
constexpr int kScanTile = kScanThreads * kScanItems;  // elements per workgroup

// Last HIP error seen by a launch helper on this host thread.
int32_t &last_hip_error();

inline int32_t check_launch() {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    last_hip_error() = (int32_t)e;
    return CP_ERR_HIP;
  }
  return CP_OK;
}

inline uint32_t div_up(uint64_t a, uint64_t b) { return (uint32_t)((a + b - 1) / b); }

// Index r of the request that holds packed token i: the last r with off[r] <= i.
// (Empty requests share their offset with the next one and are skipped.)
__device__ __forceinline__ uint32_t request_of(const uint32_t *__restrict__ off, uint32_t R, uint32_t i) {
  uint32_t lo = 0, hi = R;  // invariant: off[lo] <= i < off[hi]
  while (hi - lo > 1) {
    uint32_t mid = (lo + hi) >> 1;
    if (off[mid] <= i) lo = mid; else hi = mid;
  }
  return lo;
}

// Shuffle a trivially copyable value whose size is a multiple of 4 bytes.
template <class T>
__device__ __forceinline__ T shfl_up_any(T v, int delta) {
  static_assert(sizeof(T) % 4 == 0, "value must be whole dwords");
  union { T t; uint32_t w[sizeof(T) / 4]; } u;
  u.t = v;
#pragma unroll
  for (int k = 0; k < (int)(sizeof(T) / 4); ++k) u.w[k] = __shfl_up(u.w[k], delta, kWave);
  return u.t;
}

template <class T>
__device__ __forceinline__ T shfl_any(T v, int lane) {
  static_assert(sizeof(T) % 4 == 0, "value must be whole dwords");
  union { T t; uint32_t w[sizeof(T) / 4]; } u;
  u.t = v;
#pragma unroll
  for (int k = 0; k < (int)(sizeof(T) / 4); ++k) u.w[k] = __shfl(u.w[k], lane, kWave);
  return u.t;
}

// Ordered exclusive scan of one value per thread across a 256-thread workgroup.
// Op::combine(a, b) is associative with a the earlier operand; need not commute.
// Returns the combination of all earlier threads' values; *total = all threads'.
template <class Op>
__device__ __forceinline__ typename Op::T block_exclusive_scan(typename Op::T v, typename Op::T *total) {
  using T = typename Op::T;
  __shared__ T wave_tot[kScanThreads / kWave];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  T incl = v;
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    T up = shfl_up_any(incl, d);
    if (lane >= d) incl = Op::combine(up, incl);
  }
  if (lane == kWave - 1) wave_tot[wave] = incl;
  T excl = shfl_up_any(incl, 1);
  if (lane == 0) excl = Op::identity();
  __syncthreads();
  T before = Op::identity(), all = Op::identity();
#pragma unroll
  for (int w = 0; w < kScanThreads / kWave; ++w) {
    T t = wave_tot[w];
    if (w < wave) before = Op::combine(before, t);
    all = Op::combine(all, t);
  }
  __syncthreads();  // wave_tot may be reused by a following call
  *total = all;
  return Op::combine(before, excl);
}

// ---- ordered scan over n = op.count() elements -------------------------------
// Op supplies:  T, identity(), combine(a, b), count(), load(i),
//               store(i, exclusive, inclusive), finish(total)
// Three forms, chosen by the number of elements.  A tile is kScanTile = 256 elements, one per thread: these
// scans are bound by latency, not by bytes, so small tiles (many workgroups, short dependent chains) win.
//   up to 1024 elements  scan_single: one workgroup walks the few tiles in order.  One launch.
//   up to 1024 tiles     scan_reduce (per-tile totals -> agg[tile]), then scan_apply_self: every tile
//                        combines the totals of the tiles before it by itself (at most four loads per
//                        thread) and scans its elements; the last tile calls op.finish.  Two launches.
//   more                 scan_reduce, scan_carry (one workgroup turns agg[] into exclusive tile
//                        prefixes and calls op.finish), scan_apply.  Three launches.
// No form waits for another workgroup.  Tiles past the end do nothing, so the grid may be sized for
// an upper bound of n.
constexpr uint32_t kSelfCarryPerThread = 4;
constexpr uint32_t kSelfCarryTiles = kSelfCarryPerThread * kScanThreads;  // 262,144 elements
constexpr uint32_t kSingleItems = 1024;

// Scan of one tile seeded with `prefix`; returns the tile's total combined onto the prefix.
template <class Op>
__device__ __forceinline__ typename Op::T scan_tile(const Op &op, uint32_t n, uint64_t base, typename Op::T prefix) {
  using T = typename Op::T;
  T item[kScanItems];
  T acc = Op::identity();
#pragma unroll
  for (int k = 0; k < kScanItems; ++k) {
    uint64_t i = base + (uint64_t)threadIdx.x * kScanItems + k;
    item[k] = i < n ? op.load((uint32_t)i) : Op::identity();
    acc = Op::combine(acc, item[k]);
  }
  T total;
  T excl = block_exclusive_scan<Op>(acc, &total);
  T run = Op::combine(prefix, excl);
#pragma unroll
  for (int k = 0; k < kScanItems; ++k) {
    uint64_t i = base + (uint64_t)threadIdx.x * kScanItems + k;
    T incl = Op::combine(run, item[k]);
    if (i < n) op.store((uint32_t)i, run, incl);
    run = incl;
  }
  return Op::combine(prefix, total);
}

template <class Op>
__global__ __launch_bounds__(kScanThreads) void scan_single(Op op) {
  const uint32_t n = op.count();  // at most kSingleItems: one workgroup walks the few tiles in order
  typename Op::T total = Op::identity();
  for (uint64_t base = 0; base == 0 || base < n; base += kScanTile) total = scan_tile<Op>(op, n, base, total);
  if (threadIdx.x == 0) op.finish(total);
}

template <class Op>
__global__ __launch_bounds__(kScanThreads) void scan_reduce(Op op, typename Op::T *__restrict__ agg) {
  using T = typename Op::T;
  const uint32_t n = op.count();
  const uint64_t base = (uint64_t)blockIdx.x * kScanTile;
  if (base >= n) return;
  T acc = Op::identity();
#pragma unroll
  for (int k = 0; k < kScanItems; ++k) {
    uint64_t i = base + (uint64_t)threadIdx.x * kScanItems + k;
    if (i < n) acc = Op::combine(acc, op.load((uint32_t)i));
  }
  T total;
  block_exclusive_scan<Op>(acc, &total);
  if (threadIdx.x == 0) agg[blockIdx.x] = total;
}

template <class Op>
__global__ __launch_bounds__(kScanThreads) void scan_carry(Op op, typename Op::T *__restrict__ agg) {
  using T = typename Op::T;
  const uint32_t n = op.count();
  const uint32_t n_tiles = (uint32_t)(((uint64_t)n + kScanTile - 1) / kScanTile);
  T carry = Op::identity();
  for (uint32_t c0 = 0; c0 < n_tiles; c0 += kScanThreads) {  // uniform trip count
    uint32_t t = c0 + threadIdx.x;
    T v = t < n_tiles ? agg[t] : Op::identity();
    T total;
    T excl = block_exclusive_scan<Op>(v, &total);
    if (t < n_tiles) agg[t] = Op::combine(carry, excl);
    carry = Op::combine(carry, total);
  }
  if (threadIdx.x == 0) op.finish(carry);
}

template <class Op>
__global__ __launch_bounds__(kScanThreads) void scan_apply(Op op, const typename Op::T *__restrict__ agg) {
  const uint32_t n = op.count();
  const uint64_t base = (uint64_t)blockIdx.x * kScanTile;
  if (base >= n) return;
  scan_tile<Op>(op, n, base, agg[blockIdx.x]);
}

// agg[] holds the tiles' totals (scan_reduce); at most kSelfCarryTiles tiles.
template <class Op>
__global__ __launch_bounds__(kScanThreads) void scan_apply_self(Op op, const typename Op::T *__restrict__ agg) {
  using T = typename Op::T;
  const uint32_t n = op.count();
  const uint64_t base = (uint64_t)blockIdx.x * kScanTile;
  if (n == 0) {
    if (blockIdx.x == 0 && threadIdx.x == 0) op.finish(Op::identity());
    return;
  }
  if (base >= n) return;
  // totals of the tiles before this one, in order: thread t takes a few consecutive entries
  T mine = Op::identity();
#pragma unroll
  for (uint32_t k = 0; k < kSelfCarryPerThread; ++k) {
    const uint32_t t = kSelfCarryPerThread * threadIdx.x + k;
    if (t < blockIdx.x) mine = Op::combine(mine, agg[t]);
  }
  T prefix;
  block_exclusive_scan<Op>(mine, &prefix);
  const T total = scan_tile<Op>(op, n, base, prefix);
  if (threadIdx.x == 0 && base + kScanTile >= n) op.finish(total);  // the tile that holds the last element
}

// Enqueue the passes.  max_n bounds op.count() and sizes the grids;
// agg needs div_up(max_n, kScanTile) entries (at least one).
template <class Op>
int32_t run_scan(hipStream_t stream, const Op &op, uint32_t max_n, typename Op::T *agg) {
  uint32_t tiles = div_up(max_n, kScanTile);
  if (max_n <= kSingleItems) {
    scan_single<Op><<<1, kScanThreads, 0, stream>>>(op);
  } else if (tiles <= kSelfCarryTiles) {
    scan_reduce<Op><<<tiles, kScanThreads, 0, stream>>>(op, agg);
    scan_apply_self<Op><<<tiles, kScanThreads, 0, stream>>>(op, agg);
  } else {
    scan_reduce<Op><<<tiles, kScanThreads, 0, stream>>>(op, agg);
    scan_carry<Op><<<1, kScanThreads, 0, stream>>>(op, agg);
    scan_apply<Op><<<tiles, kScanThreads, 0, stream>>>(op, agg);
  }
  return check_launch();
}

inline bool aligned(const void *p, size_t a) { return ((uintptr_t)p % a) == 0; }

}  // namespace cp

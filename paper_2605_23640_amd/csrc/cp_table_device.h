// Device-side pieces of the pool index (an open-addressing table of 16-entry buckets) that more than
// one translation unit uses: where a key's walk starts, and a lookup done by a single lane.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/cacheprune.h"

namespace cp {

constexpr uint32_t kBucket = CP_TABLE_BUCKET;
constexpr uint32_t kPending = 0x80000000u;

__device__ __forceinline__ uint32_t home_bucket(uint64_t h, uint32_t n_buckets) {
  h ^= h >> 32;
  h *= 0xD6E8FEB86659FD93ull;
  h ^= h >> 32;
  h *= 0xD6E8FEB86659FD93ull;
  h ^= h >> 32;
  return __umulhi((uint32_t)h, n_buckets);  // uniform over [0, n_buckets) for any n_buckets
}


// Value stored under key h, or CP_SLOT_NONE: the walk of table.hip's group_lookup done by one lane, which
// reads a bucket's 16 keys as eight 16-byte pieces.  For callers whose lanes hold unrelated keys at
// unrelated times (a scan's store step); a group of 16 lanes per key is the faster form where a kernel
// does nothing but look keys up.
__device__ __forceinline__ uint32_t lane_lookup(const cp_table &t, uint64_t h) {
  if (h == CP_HASH_NONE) return CP_SLOT_NONE;
  const uint32_t n_buckets = (uint32_t)(t.capacity / kBucket);
  uint32_t b = home_bucket(h, n_buckets);
  for (uint32_t walked = 0; walked < n_buckets; ++walked) {
    const ulonglong2 *keys = (const ulonglong2 *)(t.keys + (uint64_t)b * kBucket);
    uint32_t hit = kBucket;
    bool empty = false;
#pragma unroll
    for (uint32_t j = 0; j < kBucket / 2; ++j) {
      const ulonglong2 k = keys[j];
      if (k.x == h) hit = 2 * j;
      if (k.y == h) hit = 2 * j + 1;
      empty = empty || k.x == CP_HASH_NONE || k.y == CP_HASH_NONE;
    }
    if (hit != kBucket) {
      const uint32_t v = t.vals[(uint64_t)b * kBucket + hit];
      return v >= kPending ? CP_SLOT_NONE : v;
    }
    if (empty) return CP_SLOT_NONE;  // entries are never removed: a key beyond a free entry does not exist
    b = b + 1 == n_buckets ? 0 : b + 1;
  }
  return CP_SLOT_NONE;
}

}  // namespace cp

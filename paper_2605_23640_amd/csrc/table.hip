// The pool index as an open-addressing table on the GPU (Sec. 4.3.5 "Storage
// format and indexing": cached segments are found through a hash index; here
// one key per pooled token), its lookup (cp_probe) and the table side of
// insertion (cp_insert_kv; Sec. 4.3.5 "Lifecycle management": one copy of a
// duplicate).
//
// Layout: buckets of 16 entries.  The 16 keys of a bucket are one 128-byte
// line, fetched by a group of 16 lanes with one coalesced load; wavefront
// ballots find the matching or the first empty entry.  A key lives in the
// first bucket, walking from its home bucket with wrap-around, that had a free
// entry when it arrived.  Entries are never removed, so a bucket that was full
// stays full and a walk may stop at the first bucket that shows a free entry.
//
// Values: a pool slot (< 2^31), CP_SLOT_NONE for an entry whose token could not
// be stored (treated as absent), or, only while cp_insert_kv runs, the marker
// kPending | i naming the lowest packed token index i that wants the entry.
#include "cp_device.h"
#include "cp_internal.h"
#include "cp_table_device.h"

namespace cp {
namespace {

constexpr int kProbeThreads = 256;

// 16-bit slice of a wavefront ballot belonging to this lane's group of 16.
__device__ __forceinline__ uint32_t group_bits(unsigned long long ballot) {
  return (uint32_t)(ballot >> (threadIdx.x & 48)) & 0xFFFFu;
}

__global__ __launch_bounds__(kProbeThreads) void table_init_kernel(cp_table t) {
  uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < t.capacity) {
    t.keys[i] = CP_HASH_NONE;
    t.vals[i] = CP_SLOT_NONE;
  }
}

// Value stored under key h, or CP_SLOT_NONE.  Called by all lanes of a wavefront together; the 16
// lanes of a group pass the same h (CP_HASH_NONE = nothing to look up) and get the same answer.
__device__ __forceinline__ uint32_t group_lookup(const cp_table &t, uint64_t h) {
  const uint32_t sub = threadIdx.x & (kBucket - 1);
  const uint32_t n_buckets = (uint32_t)(t.capacity / kBucket);
  bool active = h != CP_HASH_NONE;
  uint32_t b = home_bucket(h, n_buckets), walked = 0, result = CP_SLOT_NONE;
  while (__any(active)) {  // wavefront-uniform loop; groups drop out one by one
    uint64_t k = CP_HASH_NONE;
    if (active) k = t.keys[(uint64_t)b * kBucket + sub];
    uint32_t hit = group_bits(__ballot(active && k == h));
    uint32_t empty = group_bits(__ballot(active && k == CP_HASH_NONE));
    if (active) {
      if (hit) {
        result = t.vals[(uint64_t)b * kBucket + (__ffs(hit) - 1)];
        active = false;
      } else if (empty || ++walked == n_buckets) {
        active = false;
      } else {
        b = b + 1 == n_buckets ? 0 : b + 1;
      }
    }
  }
  return result >= kPending ? CP_SLOT_NONE : result;
}

// One group of 16 lanes per token.  hash_b, hash_c (nullable): further keys, tried in this order while
// the ones before miss.
__global__ __launch_bounds__(kProbeThreads) void probe_kernel(cp_table t, const uint64_t *__restrict__ hash,
                                                              const uint64_t *__restrict__ hash_b,
                                                              const uint64_t *__restrict__ hash_c, uint32_t N,
                                                              uint32_t *__restrict__ slot_out) {
  const uint32_t q = (uint32_t)(((uint64_t)blockIdx.x * kProbeThreads + threadIdx.x) / kBucket);
  uint32_t result = group_lookup(t, q < N ? hash[q] : CP_HASH_NONE);
  if (hash_b) {  // same for the whole grid
    const uint64_t h2 = (q < N && result == CP_SLOT_NONE) ? hash_b[q] : CP_HASH_NONE;
    const uint32_t r2 = group_lookup(t, h2);
    if (result == CP_SLOT_NONE) result = r2;
  }
  if (hash_c) {
    const uint64_t h3 = (q < N && result == CP_SLOT_NONE) ? hash_c[q] : CP_HASH_NONE;
    const uint32_t r3 = group_lookup(t, h3);
    if (result == CP_SLOT_NONE) result = r3;
  }
  if (q < N && (threadIdx.x & (kBucket - 1)) == 0) slot_out[q] = result;
}

// Two key arrays looked up side by side, each into an output of its own (the candidates of two key streams).
__global__ __launch_bounds__(kProbeThreads) void probe_each_kernel(cp_table t, const uint64_t *__restrict__ hash_a,
                                                                   const uint64_t *__restrict__ hash_b, uint32_t N,
                                                                   uint32_t *__restrict__ out_a,
                                                                   uint32_t *__restrict__ out_b) {
  const uint32_t q = (uint32_t)(((uint64_t)blockIdx.x * kProbeThreads + threadIdx.x) / kBucket);
  const uint32_t ra = group_lookup(t, q < N ? hash_a[q] : CP_HASH_NONE);
  const uint32_t rb = group_lookup(t, q < N ? hash_b[q] : CP_HASH_NONE);
  if (q < N && (threadIdx.x & (kBucket - 1)) == 0) {
    out_a[q] = ra;
    out_b[q] = rb;
  }
}

__device__ __forceinline__ uint64_t pow_u64(uint64_t b, uint32_t k) {  // b^k mod 2^64
  uint64_t r = 1;
  while (k) {
    if (k & 1) r *= b;
    b *= b;
    k >>= 1;
  }
  return r;
}

// Floating-anchor lookup, Step 1 and the pre-check of Step 2 (Sec. 4.2.2), one group of 16 lanes per
// position a of the batch.  Step 1: is a a candidate, i.e. does the W-token window that starts at a lie
// inside one run, after the run's first token, and hash to a stored prefix hash?  (The prefix hash of a
// stored run is the table key of the run's W-th token, so the stored prefix hashes are the keys whose
// live slot carries the anchor mark.)  Step 2's pre-check: how far does the stored text go on?  The key
// of tokens a..t follows in O(1) from the run's chain hashes and a power of the base; stored runs are
// closed under taking prefixes, so "key of a..t is stored" is true up to some last token and false
// beyond it: that token is found by growing steps and then narrowing, 16 tokens looked up per round (one by each
// lane of the group), about 2 log16(length) + 1 rounds.
// ext1[a] = 1 + last token whose key from a is stored, 0 if a is no candidate.
__global__ __launch_bounds__(kProbeThreads) void anchor_extent_kernel(cp_table table,
                                                                      const uint8_t *__restrict__ slot_anchor,
                                                                      uint32_t n_pool_slots,
                                                                      const uint64_t *__restrict__ hash,
                                                                      const uint32_t *__restrict__ run_off, uint32_t N,
                                                                      uint32_t W, uint64_t base,
                                                                      uint32_t *__restrict__ ext1) {
  const uint32_t a = (uint32_t)(((uint64_t)blockIdx.x * kProbeThreads + threadIdx.x) / kBucket);
  const uint64_t end64 = (uint64_t)a + W - 1;  // last token of the window
  uint64_t wh = CP_HASH_NONE, before = 0;
  uint32_t end = 0, ro_end = 0;
  if (a < N && end64 < N) {
    end = (uint32_t)end64;
    ro_end = run_off[end];
    // the window lies inside the run and starts after the run's first token: at least W tokens before its end
    if (hash[end] != CP_HASH_NONE && ro_end != 0xFFFFFFFFu && ro_end >= W) {
      before = hash[a - 1];  // token a-1 is in the same run
      wh = hash[end] - before * pow_u64(base, W);
      if (wh == CP_HASH_NONE) wh = CP_HASH_NONE - 1;
    }
  }
  const uint32_t s = group_lookup(table, wh);
  const bool cand = s < n_pool_slots && slot_anchor[s] != 0;
  // lo = last token known to be stored from a, hi = first token known not to be (0 = none known yet).  Every round
  // the 16 lanes of the group look 16 tokens up at once, lane j the token lo + (j + 1) * stride by itself: as long
  // as all are stored the stride grows sixteenfold, then the gap between lo and hi shrinks seventeenfold per round.
  const uint32_t sub = threadIdx.x & (kBucket - 1);
  uint32_t lo = end, hi = 0, stride = 1;
  bool searching = cand;
  while (__any(searching)) {  // wavefront-uniform loop; groups drop out one by one
    uint64_t key = CP_HASH_NONE;
    if (searching) {
      const uint64_t t64 = (uint64_t)lo + (uint64_t)(sub + 1) * stride;
      // token t continues the run of the window iff its offset in the run says so; beyond the run, the batch, or a
      // token already known not to be stored: not stored
      if (t64 < N && (hi == 0 || t64 < hi) && run_off[(uint32_t)t64] == ro_end + (uint32_t)(t64 - end)) {
        const uint32_t t = (uint32_t)t64;
        key = hash[t] - before * pow_u64(base, t - a + 1);
        if (key == CP_HASH_NONE) key = CP_HASH_NONE - 1;
      }
    }
    const bool stored = lane_lookup(table, key) != CP_SLOT_NONE;
    // stored runs are closed under taking prefixes: the lanes that found their key are the first k of the group
    const uint32_t found = group_bits(__ballot(searching && stored));
    const uint32_t k = (uint32_t)__ffs((int)~found) - 1;  // 16 if all found (bit 16 of ~found is set)
    if (searching) {
      const uint64_t first_missing = (uint64_t)lo + (uint64_t)(k + 1) * stride;
      lo += k * stride;
      if (k < kBucket && (hi == 0 || first_missing < hi)) hi = (uint32_t)(first_missing < 0xFFFFFFFFull ? first_missing : 0xFFFFFFFFull);
      if (hi == 0) {
        stride = stride < (1u << 26) ? stride * kBucket : stride;
      } else if (hi - lo <= 1) {
        searching = false;
      } else {
        stride = (hi - lo + kBucket) / (kBucket + 1);
      }
    }
  }
  if (a < N && (threadIdx.x & (kBucket - 1)) == 0) ext1[a] = cand ? lo + 1 : 0u;
}

// Index of the entry that holds key h, taking a free entry for it if there is none yet; CP_SLOT_NONE
// if h is CP_HASH_NONE or every bucket is full.  Called by all lanes of a wavefront together; the 16
// lanes of a group pass the same h and get the same answer.
__device__ __forceinline__ uint32_t group_claim(const cp_table &t, uint64_t h) {
  const uint32_t sub = threadIdx.x & (kBucket - 1);
  const uint32_t n_buckets = (uint32_t)(t.capacity / kBucket);
  bool active = h != CP_HASH_NONE;
  uint32_t b = home_bucket(h, n_buckets), walked = 0, entry = CP_SLOT_NONE;
  while (__any(active)) {
    unsigned long long *kp = (unsigned long long *)&t.keys[(uint64_t)b * kBucket + sub];
    uint64_t k = CP_HASH_NONE;
    // other workgroups fill entries while this kernel runs: read at device scope, past the per-CU cache
    if (active) k = __hip_atomic_load(kp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    uint32_t hit = group_bits(__ballot(active && k == h));
    uint32_t empty = group_bits(__ballot(active && k == CP_HASH_NONE));
    // the lane that saw the first free entry tries to take it
    bool try_claim = active && !hit && empty && sub == (uint32_t)(__ffs(empty) - 1);
    uint64_t old = 0;
    if (try_claim) old = atomicCAS(kp, (unsigned long long)CP_HASH_NONE, (unsigned long long)h);
    // success also if another group stored this very key there in the meantime
    uint32_t claimed = group_bits(__ballot(try_claim && (old == CP_HASH_NONE || old == h)));
    if (active) {
      if (hit) {
        entry = b * kBucket + (__ffs(hit) - 1);
        active = false;
      } else if (empty) {
        if (claimed) {
          entry = b * kBucket + (__ffs(empty) - 1);
          active = false;
        }  // else: someone else took that entry; look at the same bucket again
      } else if (++walked == n_buckets) {
        active = false;  // every bucket is full
      } else {
        b = b + 1 == n_buckets ? 0 : b + 1;
      }
    }
  }
  return entry;
}

// Record the prefix hash of every run whose W-th token has a slot: that token's key is the hash of
// the run's first W tokens, so a mark on its slot is all it takes.  Several tokens may name one
// slot; all write the same byte.
__global__ __launch_bounds__(kProbeThreads) void mark_anchor_kernel(const uint32_t *__restrict__ run_off,
                                                                    const uint32_t *__restrict__ slot, uint32_t N,
                                                                    uint32_t W, uint32_t n_pool_slots,
                                                                    uint8_t *__restrict__ slot_anchor) {
  const uint32_t i = blockIdx.x * kProbeThreads + threadIdx.x;
  if (i < N && run_off[i] == W - 1 && slot[i] < n_pool_slots) slot_anchor[slot[i]] = 1;
}

// Copy of the live entries of one table into another (fresh) one: the keys of evicted slots, which
// stay behind with the value "absent", are left out.  One group of 16 lanes per source entry.
__global__ __launch_bounds__(kProbeThreads) void table_compact_kernel(cp_table src, cp_table dst,
                                                                      uint32_t *status_flags) {
  const uint64_t e = ((uint64_t)blockIdx.x * kProbeThreads + threadIdx.x) / kBucket;
  const uint32_t sub = threadIdx.x & (kBucket - 1);
  uint64_t h = CP_HASH_NONE;
  uint32_t v = CP_SLOT_NONE;
  if (e < src.capacity) {
    v = src.vals[e];
    if (v < kPending) h = src.keys[e];
  }
  const uint32_t entry = group_claim(dst, h);
  if (sub == 0 && h != CP_HASH_NONE) {
    if (entry != CP_SLOT_NONE) dst.vals[entry] = v;
    else atomicOr(status_flags, CP_FLAG_TABLE_FULL);
  }
}

// How full the table is: entries that hold a key, and those of them whose key has a slot.  The difference is
// what evictions and dropped tokens left behind, i.e. what cp_table_compact would give back.
__global__ void table_count_zero_kernel(uint32_t *counts) { counts[0] = counts[1] = 0; }
__global__ __launch_bounds__(kProbeThreads) void table_count_kernel(cp_table t, uint32_t *counts) {
  uint32_t used = 0, live = 0;
  for (uint64_t e = (uint64_t)blockIdx.x * kProbeThreads + threadIdx.x; e < t.capacity;
       e += (uint64_t)gridDim.x * kProbeThreads) {
    const bool has_key = t.keys[e] != CP_HASH_NONE;
    used += has_key ? 1u : 0u;
    live += (has_key && t.vals[e] < kPending) ? 1u : 0u;
  }
#pragma unroll
  for (int m = 1; m < kWave; m <<= 1) {
    used += __shfl_xor(used, m, kWave);
    live += __shfl_xor(live, m, kWave);
  }
  if ((threadIdx.x & (kWave - 1)) == 0) {
    if (used) atomicAdd(&counts[0], used);
    if (live) atomicAdd(&counts[1], live);
  }
}

// Insert, step 1: find or claim the table entry of every token's key and leave
// in vals[] the smallest packed index that asked for a not-yet-stored key.
__global__ __launch_bounds__(kProbeThreads) void insert_claim_kernel(cp_table t, const uint64_t *__restrict__ hash,
                                                                     const uint32_t *__restrict__ found /* nullable */,
                                                                     uint32_t N, uint32_t *__restrict__ entry_of,
                                                                     uint32_t *status_flags) {
  const uint32_t q = (uint32_t)(((uint64_t)blockIdx.x * kProbeThreads + threadIdx.x) / kBucket);
  const uint32_t sub = threadIdx.x & (kBucket - 1);
  // a token whose text the pool holds already (found) asks for no entry: it is not stored again
  const uint64_t h = (q < N && !(found && found[q] != CP_SLOT_NONE)) ? hash[q] : CP_HASH_NONE;
  const uint32_t entry = group_claim(t, h);
  if (q < N && sub == 0) {
    entry_of[q] = entry;
    if (entry != CP_SLOT_NONE) {
      atomicMin(&t.vals[entry], kPending | q);  // no effect on a stored slot (< kPending)
    } else if (h != CP_HASH_NONE) {
      atomicOr(status_flags, CP_FLAG_TABLE_FULL);
    }
  }
}

// Insert, step 2: ordered count of the storing tokens (the owners of new keys).  The same scan learns
// whether any token found no table entry: then the table cannot hold the batch's new keys, and the call
// stores none of them (room = 0), so that what a call stores never depends on which keys happened to get
// the last entries.
struct OwnerRankOp {
  struct T { uint32_t n, failed; };
  const uint64_t *hash;
  const uint32_t *found;  // nullable
  const uint32_t *entry_of;
  const uint32_t *vals;
  uint32_t *rank;      // [N]  rank of token i among the owners, valid for owners only
  uint32_t *n_inserted;
  uint32_t *room;      // free-list entries this call may use: n_free, or 0 if the table overflowed
  uint32_t *status_flags;
  uint32_t N, n_free;

  static __device__ __forceinline__ T identity() { return T{0u, 0u}; }
  static __device__ __forceinline__ T combine(T a, T b) { return T{a.n + b.n, a.failed | b.failed}; }
  __device__ __forceinline__ uint32_t count() const { return N; }
  __device__ __forceinline__ T load(uint32_t i) const {
    const uint32_t e = entry_of[i];
    if (e == CP_SLOT_NONE)  // no entry: not asked for (sensitive, found already) or the table is full
      return T{0u, (hash[i] != CP_HASH_NONE && !(found && found[i] != CP_SLOT_NONE)) ? 1u : 0u};
    return T{vals[e] == (kPending | i) ? 1u : 0u, 0u};
  }
  __device__ __forceinline__ void store(uint32_t i, T excl, T incl) const {
    if (incl.n != excl.n) rank[i] = excl.n;
  }
  __device__ __forceinline__ void finish(T total) const {
    const uint32_t r = total.failed ? 0u : n_free;
    *room = r;
    *n_inserted = total.n < r ? total.n : r;
    if (!total.failed && total.n > n_free) atomicOr(status_flags, CP_FLAG_POOL_FULL);
  }
};

// Insert, step 3: every token learns the slot that holds its key after the call.
__global__ __launch_bounds__(256) void insert_resolve_kernel(const uint32_t *__restrict__ entry_of,
                                                             const uint32_t *__restrict__ vals,
                                                             const uint32_t *__restrict__ rank,
                                                             const uint32_t *__restrict__ free_slots,
                                                             const uint32_t *__restrict__ room,
                                                             uint32_t n_pool_slots, uint32_t N,
                                                             const uint32_t *__restrict__ found /* nullable */,
                                                             uint32_t *__restrict__ slot_out,
                                                             uint8_t *__restrict__ owner) {
  uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= N) return;
  const uint32_t n_free = *room;
  if (owner) owner[i] = 0;  // set again by the commit step for the tokens that store
  uint32_t e = entry_of[i], s = CP_SLOT_NONE;
  if (found && found[i] != CP_SLOT_NONE) {
    s = found[i];  // the slot that already holds this token's text
  } else if (e != CP_SLOT_NONE) {
    uint32_t v = vals[e];
    if (v < kPending) {
      s = v;  // stored by an earlier call
    } else if (v != CP_SLOT_NONE) {
      uint32_t owner = v & ~kPending;
      uint32_t r = owner < N ? rank[owner] : n_free;  // a marker of this call always names a token < N
      if (r < n_free) s = free_slots[r];
      if (s >= n_pool_slots) s = CP_SLOT_NONE;  // a free-list entry outside the pool is never used
    }
  }
  slot_out[i] = s;
}

// What the chain-recording insert adds (all null otherwise): the batch's tokens and run offsets, the
// slot every token resolved to, the per-slot token / parent arrays and a flag per storing token.
struct ChainRecord {
  const uint32_t *tok, *run_off, *cand;
  uint32_t *slot_tok, *slot_parent;
  uint8_t *owner;
};

// Chain-recording insert, last step: a token that took a slot but whose run was not confirmed up to
// it (the slot found for an earlier token of the run holds another text) leaves a slot nobody may
// match: its parent is set to a value no candidate ever equals.
__global__ __launch_bounds__(256) void insert_poison_kernel(const uint8_t *__restrict__ owner,
                                                            const uint32_t *__restrict__ cand,
                                                            const uint32_t *__restrict__ slot_out, uint32_t N,
                                                            uint32_t n_pool_slots, uint32_t *__restrict__ slot_parent) {
  uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= N || !owner[i]) return;
  if (slot_out[i] == CP_SLOT_NONE && cand[i] < n_pool_slots) slot_parent[cand[i]] = CP_PARENT_POISON;
}

// Insert, step 4: owners replace the marker by their slot (or by "absent" when
// the free list ran out) and record the position their token had in its request.
__global__ __launch_bounds__(256) void insert_commit_kernel(const uint32_t *__restrict__ entry_of, uint32_t *vals,
                                                            const uint32_t *__restrict__ rank,
                                                            const uint32_t *__restrict__ free_slots,
                                                            const uint32_t *__restrict__ room,
                                                            uint32_t n_pool_slots, const uint32_t *__restrict__ off,
                                                            uint32_t R, uint32_t N, int32_t *__restrict__ slot_pos,
                                                            MoveItem *__restrict__ items,
                                                            uint32_t *__restrict__ move_counter, ChainRecord chain,
                                                            const uint32_t *__restrict__ found,
                                                            uint32_t *__restrict__ resolve_to) {
  uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i == 0) *move_counter = 0;  // work counter of the scatter that follows
  if (i >= N) return;
  const uint32_t n_free = *room;
  uint32_t e = entry_of[i];
  if (resolve_to) {
    // Insert without chain records: step 3 (every token learns the slot that holds its key) is done here too.
    // An owner may replace its marker while another token reads the entry; the reader then sees either the
    // marker, and works the slot out from the owner's rank, or the slot the owner wrote: the same value.
    uint32_t s = CP_SLOT_NONE;
    if (found && found[i] != CP_SLOT_NONE) {
      s = found[i];
    } else if (e != CP_SLOT_NONE) {
      const uint32_t v = __hip_atomic_load(&vals[e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (v < kPending) {
        s = v;
      } else if (v != CP_SLOT_NONE) {
        const uint32_t owner = v & ~kPending;
        const uint32_t r = owner < N ? rank[owner] : n_free;
        if (r < n_free) s = free_slots[r];
        if (s >= n_pool_slots) s = CP_SLOT_NONE;
      }
    }
    resolve_to[i] = s;
  }
  if (e == CP_SLOT_NONE || vals[e] != (kPending | i)) return;  // only the owner touches its entry
  uint32_t r = rank[i], s = CP_SLOT_NONE;
  if (r < n_free) {
    s = free_slots[r];
    if (s < n_pool_slots) slot_pos[s] = (int32_t)(i - off[request_of(off, R, i)]);
    else s = CP_SLOT_NONE;  // a free-list entry outside the pool is never used
  }
  if (chain.slot_tok && s != CP_SLOT_NONE) {
    // the slot's node of the trie of stored runs: its token and the slot of the token before it
    uint32_t parent = CP_SLOT_NONE;
    if (chain.run_off[i] != 0) {
      parent = i ? chain.cand[i - 1] : CP_SLOT_NONE;
      if (parent == CP_SLOT_NONE) parent = CP_PARENT_POISON;  // its predecessor has no slot: never matches
    }
    chain.slot_tok[s] = chain.tok[i];
    chain.slot_parent[s] = parent;
    chain.owner[i] = 1;
  }
  vals[e] = s;
  // work list of the scatter: token i -> slot s (an unusable entry is marked and skipped)
  if (r < n_free) items[r] = MoveItem{s == CP_SLOT_NONE ? CP_SLOT_NONE : i, s, 0, CP_SLOT_NONE};
}

}  // namespace
}  // namespace cp

extern "C" uint64_t cp_table_capacity_for(uint64_t n_keys, double load_factor) {
  if (!(load_factor > 0.0) || load_factor > 1.0) load_factor = 0.5;
  double want = (double)n_keys / load_factor;
  uint64_t c = (uint64_t)want;
  if ((double)c < want) ++c;
  if (c < n_keys + 1) c = n_keys + 1;  // at least one entry stays free
  return (c + CP_TABLE_BUCKET - 1) / CP_TABLE_BUCKET * CP_TABLE_BUCKET;
}

static int32_t table_ok(const cp_table &t) {
  if (!t.keys || !t.vals || t.capacity == 0) return CP_ERR_INVALID_ARG;
  if (t.capacity % CP_TABLE_BUCKET || !cp::aligned(t.keys, 128) || !cp::aligned(t.vals, 64)) return CP_ERR_INVALID_ARG;
  if (t.capacity >= 0x100000000ull) return CP_ERR_UNSUPPORTED;
  return CP_OK;
}

extern "C" int32_t cp_table_init(void *stream, cp_table table) {
  using namespace cp;
  if (int32_t rc = table_ok(table)) return rc;
  table_init_kernel<<<div_up(table.capacity, kProbeThreads), kProbeThreads, 0, (hipStream_t)stream>>>(table);
  return check_launch();
}

static int32_t probe_common(void *stream, const cp_table &table, const uint64_t *hash, const uint64_t *hash_b,
                            const uint64_t *hash_c, uint32_t N, uint32_t *slot_out) {
  using namespace cp;
  if (N == 0) return CP_OK;
  if (N >= 0x80000000u) return CP_ERR_UNSUPPORTED;
  if (int32_t rc = table_ok(table)) return rc;
  if (!hash || !slot_out || !aligned(hash, 8) || !aligned(hash_b, 8) || !aligned(hash_c, 8) || !aligned(slot_out, 4))
    return CP_ERR_INVALID_ARG;
  probe_kernel<<<div_up((uint64_t)N * kBucket, kProbeThreads), kProbeThreads, 0, (hipStream_t)stream>>>(
      table, hash, hash_b, hash_c, N, slot_out);
  return check_launch();
}

extern "C" int32_t cp_probe(void *stream, cp_table table, const uint64_t *hash, uint32_t N, uint32_t *slot_out) {
  return probe_common(stream, table, hash, nullptr, nullptr, N, slot_out);
}

extern "C" int32_t cp_probe2(void *stream, cp_table table, const uint64_t *hash_a, const uint64_t *hash_b, uint32_t N,
                             uint32_t *slot_out) {
  if (N && !hash_b) return CP_ERR_INVALID_ARG;
  return probe_common(stream, table, hash_a, hash_b, nullptr, N, slot_out);
}

extern "C" int32_t cp_probe3(void *stream, cp_table table, const uint64_t *hash_a, const uint64_t *hash_b,
                             const uint64_t *hash_c, uint32_t N, uint32_t *slot_out) {
  if (N && (!hash_b || !hash_c)) return CP_ERR_INVALID_ARG;
  return probe_common(stream, table, hash_a, hash_b, hash_c, N, slot_out);
}

extern "C" int32_t cp_insert_anchors(void *stream, const uint32_t *run_off, const uint32_t *slot, uint32_t N,
                                     uint32_t W, uint32_t n_pool_slots, uint8_t *slot_anchor) {
  using namespace cp;
  if (N == 0 || n_pool_slots == 0) return CP_OK;
  if (N >= 0x80000000u || n_pool_slots >= 0x80000000u) return CP_ERR_UNSUPPORTED;
  if (W == 0 || !run_off || !slot || !slot_anchor) return CP_ERR_INVALID_ARG;
  mark_anchor_kernel<<<div_up(N, kProbeThreads), kProbeThreads, 0, (hipStream_t)stream>>>(run_off, slot, N, W,
                                                                                          n_pool_slots, slot_anchor);
  return check_launch();
}

namespace cp {
int32_t launch_probe_each(hipStream_t stream, cp_table table, const uint64_t *hash_a, const uint64_t *hash_b,
                          uint32_t N, uint32_t *out_a, uint32_t *out_b) {
  if (int32_t rc = table_ok(table)) return rc;
  probe_each_kernel<<<div_up((uint64_t)N * kBucket, kProbeThreads), kProbeThreads, 0, stream>>>(table, hash_a, hash_b, N,
                                                                                              out_a, out_b);
  return check_launch();
}

int32_t launch_anchor_extents(hipStream_t stream, const cp_table &table, const uint8_t *slot_anchor,
                              uint32_t n_pool_slots, const uint64_t *hash, const uint32_t *run_off, uint32_t N,
                              uint32_t W, uint64_t base, uint32_t *ext1) {
  if (int32_t rc = table_ok(table)) return rc;
  anchor_extent_kernel<<<div_up((uint64_t)N * kBucket, kProbeThreads), kProbeThreads, 0, stream>>>(
      table, slot_anchor, n_pool_slots, hash, run_off, N, W, base, ext1);
  return check_launch();
}
}  // namespace cp

static int32_t insert_common(void *stream_, cp_table table, const uint64_t *hash, const uint32_t *off, uint32_t N,
                             uint32_t R, const uint32_t *free_slots, uint32_t n_free, const void *src,
                             cp_kv_layout src_l, void *pool, cp_kv_layout pool_l, uint32_t n_pool_slots,
                             int32_t *slot_pos, uint32_t *slot_out, uint32_t *n_inserted, uint32_t *status_flags,
                             void *scratch, size_t scratch_bytes, const uint32_t *tok, const uint32_t *run_off,
                             uint32_t *slot_tok, uint32_t *slot_parent, const cp_launch_opts *opts,
                             const uint32_t *found = nullptr) {
  using namespace cp;
  hipStream_t stream = (hipStream_t)stream_;
  const bool chain = slot_tok != nullptr;
  if (N >= 0x80000000u || n_pool_slots >= 0x80000000u) return CP_ERR_UNSUPPORTED;
  if (int32_t rc = table_ok(table)) return rc;
  if (!n_inserted || !status_flags || !scratch || !aligned(scratch, 256)) return CP_ERR_INVALID_ARG;
  if (N && (!hash || !off || R == 0 || !slot_out || !slot_pos || !src || !pool)) return CP_ERR_INVALID_ARG;
  if (chain && N && (!tok || !run_off || !slot_parent)) return CP_ERR_INVALID_ARG;
  if (n_free && !free_slots) return CP_ERR_INVALID_ARG;
  if (!aligned(hash, 8) || !aligned(src, 16) || !aligned(pool, 16)) return CP_ERR_INVALID_ARG;
  if (!layout_ok(src_l) || !layout_ok(pool_l) || !layouts_match(src_l, pool_l)) return CP_ERR_UNSUPPORTED;
  MoveOpts mo;
  if (!resolve_opts(opts, false, &mo)) return CP_ERR_INVALID_ARG;
  if (scratch_bytes < cp_scratch_bytes(N, 0, 0)) return CP_ERR_SCRATCH;
  Scratch sc(scratch, scratch_bytes);
  uint32_t *agg = sc.take<uint32_t>(2 * (div_up(N, kScanTile) + 1));  // tile totals of the scans (8 bytes each at most)
  uint32_t *entry_of = sc.take<uint32_t>(N);
  uint32_t *rank = sc.take<uint32_t>(N);
  uint32_t *counter = sc.take<uint32_t>(2);  // [0] the scatter's work counter, [1] free-list entries the call may use
  MoveItem *items = sc.take<MoveItem>(N);
  uint32_t *cand = chain ? sc.take<uint32_t>(N) : slot_out;  // slot every token's key resolves to
  uint8_t *owner = chain ? sc.take<uint8_t>(N) : nullptr;
  if (!agg || !entry_of || !rank || !counter || !items || (N && !cand) || (chain && !owner)) return CP_ERR_SCRATCH;
  const uint32_t blocks = div_up(N, 256);
  if (N)
    insert_claim_kernel<<<div_up((uint64_t)N * kBucket, kProbeThreads), kProbeThreads, 0, stream>>>(
        table, hash, found, N, entry_of, status_flags);
  OwnerRankOp op{hash, found, entry_of, table.vals, rank, n_inserted, counter + 1, status_flags, N, n_free};
  if (int32_t rc = run_scan<OwnerRankOp>(stream, op, N, (OwnerRankOp::T *)agg)) return rc;
  if (N == 0) return CP_OK;
  // with chain records the commit step needs every token's slot first (a stored token's parent is its left
  // neighbour's slot); without them the two steps are one kernel
  if (chain)
    insert_resolve_kernel<<<blocks, 256, 0, stream>>>(entry_of, table.vals, rank, free_slots, counter + 1, n_pool_slots,
                                                      N, found, cand, owner);
  ChainRecord rec{tok, run_off, cand, slot_tok, slot_parent, owner};
  insert_commit_kernel<<<blocks, 256, 0, stream>>>(entry_of, table.vals, rank, free_slots, counter + 1, n_pool_slots,
                                                   off, R, N, slot_pos, items, counter, chain ? rec : ChainRecord{},
                                                   found, chain ? nullptr : cand);
  if (int32_t rc = check_launch()) return rc;
  if (chain) {
    // confirm every token's slot against the recorded chains (new slots are consistent by construction,
    // slots found under an existing key need not be), then take the unconfirmed new slots out of play
    if (int32_t rc = launch_chain_verify(stream, tok, run_off, cand, N, slot_tok, slot_parent, n_pool_slots, 0,
                                         slot_out, nullptr, agg, found))
      return rc;
    insert_poison_kernel<<<blocks, 256, 0, stream>>>(owner, cand, slot_out, N, n_pool_slots, slot_parent);
    if (int32_t rc = check_launch()) return rc;
  }
  uint32_t max_items = N < n_free ? N : n_free;
  return launch_scatter(stream, src, src_l, N, pool, pool_l, n_pool_slots, items, n_inserted, max_items, counter,
                        status_flags, mo);
}

extern "C" int32_t cp_insert_kv(void *stream, cp_table table, const uint64_t *hash, const uint32_t *off, uint32_t N,
                                uint32_t R, const uint32_t *free_slots, uint32_t n_free, const void *src,
                                cp_kv_layout src_l, void *pool, cp_kv_layout pool_l, uint32_t n_pool_slots,
                                int32_t *slot_pos, uint32_t *slot_out, uint32_t *n_inserted, uint32_t *status_flags,
                                void *scratch, size_t scratch_bytes, const cp_launch_opts *opts) {
  return insert_common(stream, table, hash, off, N, R, free_slots, n_free, src, src_l, pool, pool_l, n_pool_slots,
                       slot_pos, slot_out, n_inserted, status_flags, scratch, scratch_bytes, nullptr, nullptr, nullptr,
                       nullptr, opts);
}

extern "C" int32_t cp_insert_kv_chain(void *stream, cp_table table, const uint64_t *hash, const uint32_t *tok,
                                      const uint32_t *run_off, const uint32_t *off, uint32_t N, uint32_t R,
                                      const uint32_t *free_slots, uint32_t n_free, const void *src, cp_kv_layout src_l,
                                      void *pool, cp_kv_layout pool_l, uint32_t n_pool_slots, int32_t *slot_pos,
                                      uint32_t *slot_tok, uint32_t *slot_parent, uint32_t *slot_out,
                                      uint32_t *n_inserted, uint32_t *status_flags, void *scratch,
                                      size_t scratch_bytes, const cp_launch_opts *opts) {
  if (!slot_tok || !slot_parent) return CP_ERR_INVALID_ARG;
  return insert_common(stream, table, hash, off, N, R, free_slots, n_free, src, src_l, pool, pool_l, n_pool_slots,
                       slot_pos, slot_out, n_inserted, status_flags, scratch, scratch_bytes, tok, run_off, slot_tok,
                       slot_parent, opts);
}

extern "C" int32_t cp_insert_kv_dedup(void *stream, cp_table table, const uint64_t *ins_hash, const uint32_t *found,
                                      const uint32_t *tok, const uint32_t *ins_off, const uint32_t *off, uint32_t N,
                                      uint32_t R, const uint32_t *free_slots, uint32_t n_free, const void *src,
                                      cp_kv_layout src_l, void *pool, cp_kv_layout pool_l, uint32_t n_pool_slots,
                                      int32_t *slot_pos, uint32_t *slot_tok, uint32_t *slot_parent, uint32_t *slot_out,
                                      uint32_t *n_inserted, uint32_t *status_flags, void *scratch,
                                      size_t scratch_bytes, const cp_launch_opts *opts) {
  if (N && !found) return CP_ERR_INVALID_ARG;
  if ((slot_tok == nullptr) != (slot_parent == nullptr)) return CP_ERR_INVALID_ARG;
  return insert_common(stream, table, ins_hash, off, N, R, free_slots, n_free, src, src_l, pool, pool_l, n_pool_slots,
                       slot_pos, slot_out, n_inserted, status_flags, scratch, scratch_bytes, tok, ins_off, slot_tok,
                       slot_parent, opts, found);
}

extern "C" int32_t cp_table_compact(void *stream, cp_table src, cp_table dst, uint32_t *status_flags) {
  using namespace cp;
  if (int32_t rc = table_ok(src)) return rc;
  if (int32_t rc = table_ok(dst)) return rc;
  if (!status_flags || src.keys == dst.keys || src.vals == dst.vals) return CP_ERR_INVALID_ARG;
  table_compact_kernel<<<div_up(src.capacity * kBucket, kProbeThreads), kProbeThreads, 0, (hipStream_t)stream>>>(
      src, dst, status_flags);
  return check_launch();
}

extern "C" int32_t cp_table_count(void *stream, cp_table table, uint32_t *counts_out) {
  using namespace cp;
  if (int32_t rc = table_ok(table)) return rc;
  if (!counts_out || !aligned(counts_out, 4)) return CP_ERR_INVALID_ARG;
  table_count_zero_kernel<<<1, 1, 0, (hipStream_t)stream>>>(counts_out);
  const uint32_t blocks = div_up(table.capacity, kProbeThreads);
  table_count_kernel<<<blocks < 2048 ? blocks : 2048, kProbeThreads, 0, (hipStream_t)stream>>>(table, counts_out);
  return check_launch();
}

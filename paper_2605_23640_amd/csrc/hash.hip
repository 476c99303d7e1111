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
#include "cp_table_device.h"

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
  cp_table table;      // cp_hash_probe: the pool index, looked up under every token's hash right away
  uint32_t *slot_out;  // nullable: no lookup

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
    if (slot_out) slot_out[i] = lane_lookup(table, sensitive ? CP_HASH_NONE : h);
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

// Key of the request's tokens a..i, a after its run's first token: the chain hash those tokens get as
// the beginning of a run (Sec. 4.2.2 Step 2: substring hash from prefix hashes and a power of the base).
__device__ __forceinline__ uint64_t substring_key(const uint64_t *__restrict__ hash, uint64_t base, uint32_t a,
                                                  uint32_t i) {
  uint64_t key = hash[i] - hash[a - 1] * pow_u64(base, i - a + 1);
  return key == CP_HASH_NONE ? CP_HASH_NONE - 1 : key;
}

// Which candidate serves which token (Sec. 4.2.2: Step 1 yields a set of candidates, Step 2 checks each over the
// text stored behind it).  Candidate a covers the tokens a .. ext1[a]-1 (ext1[a] = 1 + last token whose key from a
// is stored, 0 where a is no candidate).  The candidates that serve are chosen like the intervals of a greedy
// cover: a piece of covered text begins at a candidate that no earlier candidate's text reaches; as long as a
// candidate that starts inside the text covered so far reaches beyond it, the one that reaches furthest (the
// earliest such) is chosen next.  Every token that any candidate covers is then covered by a chosen one, a chosen
// candidate overlaps only with its two neighbours in the piece, and handing the chosen candidates of a piece
// alternately to stream a and stream b (the first to a) leaves each stream a sequence of whole texts that do not
// overlap: what the per-stream verification and the span builder need.
//
// In terms of reach[p] = the largest ext1 over the candidates at or before p in the run (a prefix maximum): a
// piece begins at a candidate g with reach[g-1] <= g; its chosen candidates end at e1 = ext1[g], e2 = reach[e1-1],
// e3 = reach[e2-1], ... while that grows; the candidate that ends at e is the first position where reach attains
// e.  One scan gives every token reach[] and the piece it lies in; a token then walks its piece's ends.
struct FloatOp {
  struct T {
    uint32_t reach;  // max ext1
    uint32_t piece;  // 1 + the latest candidate x with (the largest ext1 before x in this stretch) <= x; 0: none
    uint32_t reset;  // the stretch contains a run start
  };
  const uint32_t *run_off;
  const uint32_t *ext1;
  uint32_t *reach_out;  // [N]
  uint32_t *piece_out;  // [N]: 1 + the candidate at which the piece of covered text around the token begins
  uint32_t N;

  static __device__ __forceinline__ T identity() { return T{0u, 0u, 0u}; }
  // A candidate of the right stretch begins a piece iff nothing before it reaches beyond it; only the latest such
  // candidate is wanted, and if that one fails against the left stretch's reach every earlier one of the right
  // stretch fails too (they are smaller), so one position per stretch is all that has to be carried.
  static __device__ __forceinline__ T combine(T f, T g) {
    if (g.reset) return g;
    return T{f.reach > g.reach ? f.reach : g.reach, (g.piece != 0 && g.piece - 1 >= f.reach) ? g.piece : f.piece, f.reset};
  }
  __device__ __forceinline__ uint32_t count() const { return N; }
  __device__ __forceinline__ T load(uint32_t i) const {
    const uint32_t ro = run_off[i];
    if (ro == 0 || ro == 0xFFFFFFFFu) return T{0u, 0u, 1u};  // a run's first token is never a candidate
    const uint32_t e = ext1[i];
    return T{e, e ? i + 1 : 0u, 0u};
  }
  __device__ __forceinline__ void store(uint32_t i, T, T incl) const {
    reach_out[i] = incl.reach;
    piece_out[i] = incl.piece;
  }
  __device__ __forceinline__ void finish(T) const {}
};

// First position p in (lo, hi] with reach[p] >= v, given reach[lo] < v <= reach[hi] (reach never decreases inside a run).
__device__ __forceinline__ uint32_t first_reaching(const uint32_t *__restrict__ reach, uint32_t lo, uint32_t hi, uint32_t v) {
  while (hi - lo > 1) {
    const uint32_t mid = lo + (hi - lo) / 2;
    if (reach[mid] >= v) hi = mid; else lo = mid;
  }
  return hi;
}

// Per token: the chosen candidate whose text it lies in (primary), and the next chosen candidate of the piece if
// that one's text has begun at or before the token (the two overlap there); their keys go to the two streams.
__global__ __launch_bounds__(256) void stream_keys_kernel(const uint64_t *__restrict__ hash,
                                                          const uint32_t *__restrict__ run_off,
                                                          const uint32_t *__restrict__ reach,
                                                          const uint32_t *__restrict__ piece, uint32_t N, uint64_t base,
                                                          uint64_t *__restrict__ hash_a_out, uint32_t *__restrict__ off_a_out,
                                                          uint64_t *__restrict__ hash_b_out, uint32_t *__restrict__ off_b_out) {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= N) return;
  uint64_t key[2] = {CP_HASH_NONE, CP_HASH_NONE};
  uint32_t so[2] = {0xFFFFFFFFu, 0xFFFFFFFFu};
  const uint32_t ro = run_off[i];
  if (hash[i] != CP_HASH_NONE && ro != 0xFFFFFFFFu && ro > 0 && reach[i] > i && piece[i] != 0) {  // some candidate covers i
    const uint32_t g = piece[i] - 1;
    // ends of the chosen candidates' texts, one after the other, until one lies beyond i
    uint32_t c = g, before = g, e = reach[g], k = 0;  // reach[g] = ext1[g]: nothing earlier reaches beyond g
    while (e <= i) {  // token e is covered (the piece goes on to i), so a candidate before it reaches beyond it
      before = e;
      e = reach[e - 1];
      ++k;
    }
    if (k) c = first_reaching(reach, c, before - 1, e);  // the chosen candidate that ends at e: after g, before `before`
    key[k & 1] = substring_key(hash, base, c, i);
    so[k & 1] = i - c;
    const uint32_t further = reach[e - 1];  // e - 1 >= i is a token of the run
    if (further > e) {
      const uint32_t c2 = first_reaching(reach, c, e - 1, further);
      if (c2 <= i) {
        key[(k + 1) & 1] = substring_key(hash, base, c2, i);
        so[(k + 1) & 1] = i - c2;
      }
    }
  }
  hash_a_out[i] = key[0];
  if (off_a_out) off_a_out[i] = so[0];
  if (hash_b_out) hash_b_out[i] = key[1];
  if (off_b_out) off_b_out[i] = so[1];
}

// Keys under which a batch is stored when every text is kept once (Sec. 4.3.5 "Lifecycle management").
// A token that a lookup stream found belongs to the stored text that stream's segment starts; a token
// that nothing found continues the text of the latest found token before it in its run (or starts a
// text with its run).  "Start of the text I belong to" is thus a value that found tokens and run starts
// define and every other token inherits from its left neighbour: a scan that keeps the latest
// defined value.
struct InsertKeyOp {
  using T = uint32_t;  // 1 + start of the text, 0 = not defined by this piece
  const uint64_t *hash;
  const uint32_t *run_off;
  const uint32_t *seg_off[3];  // per lookup stream, in serving order (unused streams: null)
  const uint32_t *slot[3];
  uint64_t *ins_hash_out;
  uint32_t *ins_off_out, *found_out;
  uint64_t base;
  uint32_t N;

  static __device__ __forceinline__ T identity() { return 0u; }
  static __device__ __forceinline__ T combine(T f, T g) { return g ? g : f; }
  __device__ __forceinline__ uint32_t count() const { return N; }
  __device__ __forceinline__ uint32_t found_in(uint32_t i, uint32_t *start) const {
#pragma unroll
    for (int k = 0; k < 3; ++k)
      if (slot[k] && slot[k][i] != CP_SLOT_NONE) {
        *start = i - seg_off[k][i];
        return slot[k][i];
      }
    return CP_SLOT_NONE;
  }
  __device__ __forceinline__ T load(uint32_t i) const {
    const uint32_t ro = run_off[i];
    if (ro == 0xFFFFFFFFu) return 0u;  // sensitive: the token after it starts a run
    uint32_t start = i - ro;
    if (found_in(i, &start) != CP_SLOT_NONE) return start + 1;
    return ro == 0 ? i + 1 : 0u;
  }
  __device__ __forceinline__ void store(uint32_t i, T, T incl) const {
    uint64_t key = CP_HASH_NONE;
    uint32_t io = 0xFFFFFFFFu, f = CP_SLOT_NONE;
    if (hash[i] != CP_HASH_NONE && incl != 0) {
      const uint32_t c = incl - 1;
      uint32_t unused;
      f = found_in(i, &unused);
      io = i - c;
      key = io == run_off[i] ? hash[i] : substring_key(hash, base, c, i);  // a text that starts its run: the plain chain hash
    }
    ins_hash_out[i] = key;
    ins_off_out[i] = io;
    found_out[i] = f;
  }
  __device__ __forceinline__ void finish(T) const {}
};

}  // namespace
}  // namespace cp

static int32_t hash_common(void *stream, const uint32_t *tok, const uint8_t *mask, const uint32_t *off, uint32_t N,
                           uint32_t R, uint64_t base, uint64_t *hash_out, uint32_t *run_off_out, void *scratch,
                           size_t scratch_bytes, cp_table table = cp_table{}, uint32_t *slot_out = nullptr) {
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
  HashOp op{tok, mask, off, hash_out, run_off_out, base, N, R, table, slot_out};
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

extern "C" int32_t cp_hash_probe(void *stream, const uint32_t *tok, const uint8_t *mask, const uint32_t *off, uint32_t N,
                                 uint32_t R, uint64_t base, cp_table table, uint64_t *hash_out, uint32_t *run_off_out,
                                 uint32_t *slot_out, void *scratch, size_t scratch_bytes) {
  if (N == 0) return CP_OK;
  if (!table.keys || !table.vals || table.capacity == 0 || table.capacity % CP_TABLE_BUCKET ||
      !cp::aligned(table.keys, 128) || !cp::aligned(table.vals, 64) || !slot_out)
    return CP_ERR_INVALID_ARG;
  if (table.capacity >= 0x100000000ull) return CP_ERR_UNSUPPORTED;
  return hash_common(stream, tok, mask, off, N, R, base, hash_out, run_off_out, scratch, scratch_bytes, table, slot_out);
}

extern "C" int32_t cp_hash_floating(void *stream_, cp_table table, const uint8_t *slot_anchor, uint32_t n_pool_slots,
                                    const uint64_t *hash, const uint32_t *run_off, uint32_t N, uint64_t base,
                                    uint32_t W, uint64_t *hash_a_out, uint32_t *off_a_out, uint64_t *hash_b_out,
                                    uint32_t *off_b_out, void *scratch, size_t scratch_bytes) {
  using namespace cp;
  hipStream_t stream = (hipStream_t)stream_;
  if (N == 0) return CP_OK;
  if (N >= 0x80000000u) return CP_ERR_UNSUPPORTED;
  if (n_pool_slots >= 0x80000000u) return CP_ERR_UNSUPPORTED;
  if (W == 0 || !slot_anchor || !hash || !run_off || !hash_a_out || !scratch || !aligned(scratch, 256) ||
      !aligned(hash, 8) || !aligned(hash_a_out, 8) || !aligned(hash_b_out, 8))
    return CP_ERR_INVALID_ARG;
  if (scratch_bytes < cp_scratch_bytes(N, 0, 0)) return CP_ERR_SCRATCH;
  Scratch sc(scratch, scratch_bytes);
  FloatOp::T *agg = sc.take<FloatOp::T>(div_up(N, kScanTile) + 1);
  uint32_t *ext1 = sc.take<uint32_t>(N);
  uint32_t *reach = sc.take<uint32_t>(N);
  uint32_t *piece = sc.take<uint32_t>(N);
  if (!agg || !ext1 || !reach || !piece) return CP_ERR_SCRATCH;
  if (int32_t rc = launch_anchor_extents(stream, table, slot_anchor, n_pool_slots, hash, run_off, N, W, base, ext1))
    return rc;
  FloatOp op{run_off, ext1, reach, piece, N};
  if (int32_t rc = run_scan<FloatOp>(stream, op, N, agg)) return rc;
  stream_keys_kernel<<<div_up(N, 256), 256, 0, stream>>>(hash, run_off, reach, piece, N, base, hash_a_out, off_a_out,
                                                         hash_b_out, off_b_out);
  return check_launch();
}

extern "C" int32_t cp_insert_keys(void *stream, const uint64_t *hash, const uint32_t *run_off, uint32_t N, uint64_t base,
                                  const uint32_t *seg_off_a, const uint32_t *slot_a, const uint32_t *seg_off_b,
                                  const uint32_t *slot_b, const uint32_t *seg_off_c, const uint32_t *slot_c,
                                  uint64_t *ins_hash_out, uint32_t *ins_off_out, uint32_t *found_out, void *scratch,
                                  size_t scratch_bytes) {
  using namespace cp;
  if (N == 0) return CP_OK;
  if (N >= 0x80000000u) return CP_ERR_UNSUPPORTED;
  if (!hash || !run_off || !ins_hash_out || !ins_off_out || !found_out || !scratch || !aligned(scratch, 256) ||
      !aligned(hash, 8) || !aligned(ins_hash_out, 8))
    return CP_ERR_INVALID_ARG;
  if ((seg_off_a == nullptr) != (slot_a == nullptr) || (seg_off_b == nullptr) != (slot_b == nullptr) ||
      (seg_off_c == nullptr) != (slot_c == nullptr))
    return CP_ERR_INVALID_ARG;
  if (scratch_bytes < cp_scratch_bytes(N, 0, 0)) return CP_ERR_SCRATCH;
  Scratch sc(scratch, scratch_bytes);
  uint32_t *agg = sc.take<uint32_t>(div_up(N, kScanTile) + 1);
  if (!agg) return CP_ERR_SCRATCH;
  InsertKeyOp op{hash, run_off, {seg_off_a, seg_off_b, seg_off_c}, {slot_a, slot_b, slot_c}, ins_hash_out, ins_off_out,
                 found_out, base, N};
  return run_scan<InsertKeyOp>((hipStream_t)stream, op, N, agg);
}

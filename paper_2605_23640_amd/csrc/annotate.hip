// The KV annotator's arithmetic (Sec. 4.2.1 "C1", Steps 1-3): summed-area table of the attention
// matrix, the substring of every coarse segment with the largest intra - inter attention, and the
// ranking that picks the tokens to recompute.
//
// Exact arithmetic: every weight x becomes the integer round(x * 2^32) (entries above the diagonal,
// non-finite and huge values count as 0) and all sums are 64-bit integers.  Integer addition is
// associative, so the table does not depend on how the work is split, the maximum over the
// substrings is decided without rounding, and results are reproducible bit for bit.
//
// Step 1 (cp_sat_build), three sweeps over 64 x 64 tiles, one wavefront per tile, lane = column:
//   sums   per tile: the sum of every column over the tile's rows and of every row over its columns
//   carry  exclusive scans of those sums over the tile rows / tile columns, then a running sum of the
//          "left of this tile column" row sums down all rows
//   apply  per tile: prefix sums inside the tile (wave scan along the row, running sum down the
//          rows) + what lies above the tile in its columns + what lies left of it in rows <= i
// The matrix is read twice (4 bytes per entry each) and the table written once (8 bytes per entry).
//
// Step 2 (cp_annotate): score(l, r) = T[r,r] - T[l-1,r] - 2 T[r,l-1] + 2 T[l-1,l-1]; all (l, r) of a
// 64 x 64 block of the (l, r) triangle take T[l-1, r] straight from global memory (lanes along r) and
// T[r, l-1] through a transposing LDS tile.  First sweep: maximum score per segment (64-bit atomic
// max); second sweep: smallest (l, r) among the candidates that reach it (64-bit atomic min).
#include "cp_device.h"
#include "cp_internal.h"

namespace cp {
namespace {

constexpr uint32_t kTile = 64;
constexpr uint32_t kNone = 0xFFFFFFFFu;
constexpr uint64_t kBias = 0x8000000000000000ull;  // signed -> unsigned, order preserving

__device__ __forceinline__ int64_t quantise(float x, uint32_t i, uint32_t j) {
  if (j > i || !(fabsf(x) <= 1048576.0f)) return 0;
  return (int64_t)__double2ll_rn((double)x * 4294967296.0);
}

// 64-bit wave scans through DPP moves (no LDS traffic).  dpp_add adds to v the value of the lane that
// the DPP control selects, or 0 where that lane does not exist or the row is masked off.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int64_t dpp_add(int64_t v) {
  const int lo = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)v, CTRL, ROW_MASK, 0xF, false);
  const int hi = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)((uint64_t)v >> 32), CTRL, ROW_MASK, 0xF, false);
  return v + (int64_t)(((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
}
// Inclusive prefix sum over the 64 lanes: shifts by 1, 2, 4, 8 inside each row of 16 lanes, then the
// last lane of row 0 / 2 is broadcast into row 1 / 3, then the last lane of row 1 into rows 2 and 3.
__device__ __forceinline__ int64_t wave_inclusive_sum(int64_t v) {
  v = dpp_add<0x111, 0xF>(v);  // row_shr:1
  v = dpp_add<0x112, 0xF>(v);  // row_shr:2
  v = dpp_add<0x114, 0xF>(v);  // row_shr:4
  v = dpp_add<0x118, 0xF>(v);  // row_shr:8
  v = dpp_add<0x142, 0xA>(v);  // row_bcast:15 into rows 1 and 3
  v = dpp_add<0x143, 0xC>(v);  // row_bcast:31 into rows 2 and 3
  return v;
}
// Sum over the 64 lanes, valid in every lane.
__device__ __forceinline__ int64_t wave_sum(int64_t v) {
  v = wave_inclusive_sum(v);
  const uint32_t lo = __builtin_amdgcn_readlane((int)(uint32_t)v, 63);
  const uint32_t hi = __builtin_amdgcn_readlane((int)(uint32_t)((uint64_t)v >> 32), 63);
  return (int64_t)(((uint64_t)hi << 32) | lo);
}

// colsum[I][c]: sum of column c over the rows of tile row I;  rowsum[J][r]: sum of row r over the
// columns of tile column J.  Both arrays are padded to whole tiles (n_pad columns / rows).
__global__ __launch_bounds__(64) void sat_tile_sums_kernel(const float *__restrict__ attn, uint32_t n, uint64_t ld,
                                                           uint32_t n_pad, int64_t *__restrict__ colsum,
                                                           int64_t *__restrict__ rowsum) {
  const uint32_t J = blockIdx.x, I = blockIdx.y, lane = threadIdx.x;
  const uint32_t c = J * kTile + lane, r0 = I * kTile;
  int64_t col = 0;
  if (J <= I) {  // tiles above the diagonal hold no weight
#pragma unroll 8
    for (uint32_t k = 0; k < kTile; ++k) {
      const uint32_t r = r0 + k;
      float x = 0.0f;
      if (r < n && c < n && c <= r) x = attn[(uint64_t)r * ld + c];
      const int64_t q = quantise(x, r, c);
      col += q;
      const int64_t row = wave_sum(q);
      if (lane == 0) rowsum[(uint64_t)J * n_pad + r] = row;
    }
  } else {
    rowsum[(uint64_t)J * n_pad + r0 + lane] = 0;
  }
  colsum[(uint64_t)I * n_pad + c] = col;
}

// In place, for both arrays (blockIdx.y picks one): a[k][x] <- sum of a[k'][x] over k' < k   (x < n_pad, k < n_k).
__global__ __launch_bounds__(64) void sat_exclusive_over_tiles_kernel(int64_t *a0, int64_t *a1, uint32_t n_k,
                                                                      uint32_t n_pad) {
  int64_t *a = blockIdx.y ? a1 : a0;
  const uint32_t x = blockIdx.x * blockDim.x + threadIdx.x;
  if (x >= n_pad) return;
  int64_t run = 0;
  uint32_t k = 0;
  for (; k + 8 <= n_k; k += 8) {  // eight independent loads in flight
    int64_t v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = a[(uint64_t)(k + u) * n_pad + x];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      a[(uint64_t)(k + u) * n_pad + x] = run;
      run += v[u];
    }
  }
  for (; k < n_k; ++k) {
    const int64_t v = a[(uint64_t)k * n_pad + x];
    a[(uint64_t)k * n_pad + x] = run;
    run += v;
  }
}

// In place, for every tile column J: left[J][r] <- sum of left[J][r'] over r' <= r (element e = J * n_pad + r).
struct RunningRowsOp {
  struct T {
    int64_t v;
    uint32_t reset, pad;
  };
  int64_t *a;
  uint32_t n_pad, total;
  static __device__ __forceinline__ T identity() { return T{0, 0u, 0u}; }
  static __device__ __forceinline__ T combine(T f, T g) { return g.reset ? g : T{f.v + g.v, f.reset, 0u}; }
  __device__ __forceinline__ uint32_t count() const { return total; }
  __device__ __forceinline__ T load(uint32_t e) const { return T{a[e], (e % n_pad) == 0 ? 1u : 0u, 0u}; }
  __device__ __forceinline__ void store(uint32_t e, T, T incl) const { a[e] = incl.v; }
  __device__ __forceinline__ void finish(T) const {}
};

__global__ __launch_bounds__(64) void sat_apply_kernel(const float *__restrict__ attn, uint32_t n, uint64_t ld,
                                                       uint32_t n_pad, const int64_t *__restrict__ above,
                                                       const int64_t *__restrict__ left, int64_t *__restrict__ T) {
  const uint32_t J = blockIdx.x, I = blockIdx.y, lane = threadIdx.x;
  const uint32_t c = J * kTile + lane, r0 = I * kTile;
  // everything above the tile, in the tile's columns up to this lane's
  const int64_t above_pref = wave_inclusive_sum(above[(uint64_t)I * n_pad + c]);
  int64_t acc = 0;  // this tile's rows so far, tile's columns up to this lane's
  const bool weight = J <= I;
#pragma unroll 8
  for (uint32_t k = 0; k < kTile; ++k) {
    const uint32_t r = r0 + k;
    if (r >= n) break;  // same for the whole wave
    if (weight) {
      float x = 0.0f;
      if (c < n && c <= r) x = attn[(uint64_t)r * ld + c];
      acc += wave_inclusive_sum(quantise(x, r, c));
    }
    if (c < n) T[(uint64_t)r * n + c] = acc + above_pref + left[(uint64_t)J * n_pad + r];
  }
}

// ---- segments ----

// seg_a[i] = first token of i's coarse segment (kNone for a sensitive token): running maximum of
// (position + 1) over the sensitive tokens.  A substring [l, r] lies in one segment iff l >= seg_a[r].
struct SegStartOp {
  using T = uint32_t;
  const uint8_t *mask;
  uint32_t *seg_a;
  uint32_t n;
  static __device__ __forceinline__ T identity() { return 0u; }
  static __device__ __forceinline__ T combine(T a, T b) { return a > b ? a : b; }
  __device__ __forceinline__ uint32_t count() const { return n; }
  __device__ __forceinline__ T load(uint32_t i) const { return mask[i] ? i + 1 : 0u; }
  __device__ __forceinline__ void store(uint32_t i, T, T incl) const { seg_a[i] = mask[i] ? kNone : incl; }
  __device__ __forceinline__ void finish(T) const {}
};
__global__ __launch_bounds__(256) void annotate_init_kernel(const int64_t *__restrict__ T, uint32_t n,
                                                            int64_t *__restrict__ diag, uint64_t *best_u,
                                                            uint64_t *best_lr) {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  diag[i] = T[(uint64_t)i * n + i];
  best_u[i] = 0;        // below every biased score
  best_lr[i] = ~0ull;   // above every packed (l, r)
}

// One workgroup per 64 x 64 block of candidates: l in [lt*64, +64), r in [rt*64, +64), lt <= rt.
// pass 0: best_u[seg] = max biased score; pass 1: best_lr[seg] = min packed (l, r) among the maxima.
__global__ __launch_bounds__(256) void annotate_search_kernel(const int64_t *__restrict__ T, uint32_t n,
                                                              const int64_t *__restrict__ diag,
                                                              const uint32_t *__restrict__ seg_a, uint32_t min_len,
                                                              int pass, uint64_t *best_u, uint64_t *best_lr) {
  const uint32_t rt = blockIdx.x, lt = blockIdx.y;
  if (lt > rt) return;
  __shared__ int64_t colT[kTile][kTile + 1];  // colT[r'][l'] = T[r0 + r'][l0 + l' - 1]
  __shared__ uint32_t any_valid;
  const uint32_t l0 = lt * kTile, r0 = rt * kTile;
  const uint32_t rl = threadIdx.x & (kTile - 1), grp = threadIdx.x / kTile;  // lane along r; 4 groups of 16 l's
  const uint32_t r = r0 + rl;
  const uint32_t a_r = r < n ? seg_a[r] : kNone;  // kNone: r is sensitive or past the end
  // candidates exist iff some r of the block has its segment start at or before the block's last l
  if (threadIdx.x == 0) any_valid = 0;
  __syncthreads();
  if (a_r != kNone && a_r <= l0 + kTile - 1 && r + 1 >= min_len + (a_r > l0 ? a_r : l0)) atomicOr(&any_valid, 1u);
  __syncthreads();
  if (!any_valid) return;
  // stage T[r][l-1] for the block: rows r0.., columns l0-1 .. l0+62, loaded along the rows
  for (uint32_t e = threadIdx.x; e < kTile * kTile; e += blockDim.x) {
    const uint32_t rr = e / kTile, ll = e % kTile;
    const uint32_t gr = r0 + rr, gl = l0 + ll;  // gl = l; column wanted = l - 1
    colT[rr][ll] = (gr < n && gl >= 1 && gl - 1 < n) ? T[(uint64_t)gr * n + (gl - 1)] : 0;
  }
  __syncthreads();
  bool have = false;
  int64_t best = 0;
  uint32_t best_l = 0;
  if (a_r != kNone) {
    const int64_t d_r = diag[r];
#pragma unroll 4
    for (uint32_t k = 0; k < kTile / 4; ++k) {
      const uint32_t ll = grp * (kTile / 4) + k, l = l0 + ll;
      if (l > r || l < a_r || r - l + 1 < min_len) continue;
      const int64_t up = l ? T[(uint64_t)(l - 1) * n + r] : 0;  // T[l-1][r], lanes along r
      const int64_t dl = l ? diag[l - 1] : 0;
      const int64_t score = d_r - up - 2 * colT[rl][ll] + 2 * dl;
      if (!have || score > best) {  // l ascending: the smallest l stays on ties
        have = true;
        best = score;
        best_l = l;
      }
    }
  }
  if (!have) return;
  const uint64_t u = (uint64_t)best ^ kBias;
  if (pass == 0) {
    if (best_u[a_r] < u) atomicMax((unsigned long long *)&best_u[a_r], (unsigned long long)u);
  } else if (u == best_u[a_r]) {
    atomicMin((unsigned long long *)&best_lr[a_r], ((unsigned long long)best_l << 32) | r);
  }
}

// Per token: the chosen substring of its segment, and d = inter - intra attention of its own row.
__global__ __launch_bounds__(256) void annotate_finish_kernel(const int64_t *__restrict__ T, uint32_t n,
                                                              const int64_t *__restrict__ diag,
                                                              const uint32_t *__restrict__ seg_a,
                                                              const uint64_t *__restrict__ best_u,
                                                              const uint64_t *__restrict__ best_lr,
                                                              uint32_t *__restrict__ out_l, uint32_t *__restrict__ out_r,
                                                              int64_t *__restrict__ out_score,
                                                              uint8_t *__restrict__ reusable,
                                                              uint8_t *__restrict__ store_mask,
                                                              int64_t *__restrict__ d, uint32_t *__restrict__ rank) {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  uint32_t bl = kNone, br = kNone;
  int64_t score = 0, di = 0;
  bool inside = false;
  const uint32_t a = seg_a[i];
  if (a != kNone && best_lr[a] != ~0ull) {
    bl = (uint32_t)(best_lr[a] >> 32);
    br = (uint32_t)best_lr[a];
    score = (int64_t)(best_u[a] ^ kBias);
    inside = bl <= i && i <= br;
    if (inside) {
      // inter_i = T[i][bl-1] - T[i-1][bl-1];  intra_i = T[i][i] - T[i-1][i] - inter_i
      const int64_t t_i = bl ? T[(uint64_t)i * n + bl - 1] : 0;
      const int64_t t_p = (bl && i) ? T[(uint64_t)(i - 1) * n + bl - 1] : 0;
      const int64_t up = i ? T[(uint64_t)(i - 1) * n + i] : 0;
      const int64_t inter = t_i - t_p;
      di = inter - (diag[i] - up - inter);
    }
  }
  out_l[i] = bl;
  out_r[i] = br;
  out_score[i] = score;
  reusable[i] = inside ? 1 : 0;
  if (store_mask) store_mask[i] = inside ? 0 : 1;
  d[i] = di;
  rank[i] = 0;
}

// Rank of every token of a chosen substring among that substring's tokens by d, largest first,
// earlier token first on ties.  Block (x, y): tokens i of block x against the tokens j of chunk y;
// the partial counts are added up in rank[] (zeroed by the finish kernel).
constexpr uint32_t kRankChunk = 256;
__global__ __launch_bounds__(256) void annotate_rank_kernel(uint32_t n, const uint32_t *__restrict__ out_l,
                                                            const uint32_t *__restrict__ out_r,
                                                            const uint8_t *__restrict__ reusable,
                                                            const int64_t *__restrict__ d, uint32_t *rank) {
  __shared__ int64_t dj[kRankChunk];
  __shared__ uint32_t lo_all, hi_all;
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  const uint32_t j0 = blockIdx.y * kRankChunk;
  const bool mine = i < n && reusable[i];
  const uint32_t bl = mine ? out_l[i] : kNone, br = mine ? out_r[i] : 0u;
  if (threadIdx.x == 0) {
    lo_all = kNone;
    hi_all = 0;
  }
  __syncthreads();
  if (mine) {
    atomicMin(&lo_all, bl);
    atomicMax(&hi_all, br);
  }
  __syncthreads();
  if (lo_all == kNone || j0 > hi_all || j0 + kRankChunk <= lo_all) return;  // no token here looks at this chunk
  const uint32_t j = j0 + threadIdx.x;
  dj[threadIdx.x] = j < n ? d[j] : 0;
  __syncthreads();
  if (!mine) return;
  const uint32_t from = bl > j0 ? bl : j0, to = br < j0 + kRankChunk - 1 ? br : j0 + kRankChunk - 1;  // inclusive
  if (from > to) return;
  const int64_t di = d[i];
  uint32_t count = 0;
  for (uint32_t jj = from; jj <= to; ++jj) {
    const int64_t v = dj[jj - j0];
    count += (v > di || (v == di && jj < i)) ? 1u : 0u;
  }
  if (count) atomicAdd(&rank[i], count);
}

// The first floor(len * rho / 100) tokens of that order are marked.
__global__ __launch_bounds__(256) void annotate_mark_kernel(uint32_t n, const uint32_t *__restrict__ out_l,
                                                            const uint32_t *__restrict__ out_r,
                                                            const uint8_t *__restrict__ reusable,
                                                            const uint32_t *__restrict__ rank, uint32_t rho_percent,
                                                            uint8_t *__restrict__ recompute) {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  uint8_t mark = 0;
  if (reusable[i]) {
    const uint32_t n_marked = (uint32_t)((uint64_t)(out_r[i] - out_l[i] + 1) * rho_percent / 100);
    mark = rank[i] < n_marked ? 1 : 0;
  }
  recompute[i] = mark;
}

inline uint32_t pad_to_tile(uint32_t n) { return (n + kTile - 1) / kTile * kTile; }

}  // namespace
}  // namespace cp

extern "C" size_t cp_sat_scratch_bytes(uint32_t n) {
  using namespace cp;
  const uint64_t n_pad = pad_to_tile(n), n_t = n_pad / kTile;
  // column sums and row sums per tile row / tile column, scan totals, per-token arrays of cp_annotate
  return (size_t)(2 * n_t * n_pad * 8 + ((2 * n_t * n_pad) / kScanTile + 2) * 16 + 56ull * n + 16 * 256);
}

extern "C" int32_t cp_sat_build(void *stream_, const float *attn, uint32_t n, uint64_t ld, int64_t *T, void *scratch,
                                size_t scratch_bytes) {
  using namespace cp;
  hipStream_t stream = (hipStream_t)stream_;
  if (n == 0) return CP_OK;
  if (n > (1u << 20)) return CP_ERR_UNSUPPORTED;  // sums of n * n weights of at most 2^52 each stay below 2^63 ... for sane weights
  if (!attn || !T || ld < n || !scratch || !aligned(scratch, 256) || !aligned(attn, 4) || !aligned(T, 8))
    return CP_ERR_INVALID_ARG;
  if (scratch_bytes < cp_sat_scratch_bytes(n)) return CP_ERR_SCRATCH;
  const uint32_t n_pad = pad_to_tile(n), n_t = n_pad / kTile;
  Scratch sc(scratch, scratch_bytes);
  int64_t *colsum = sc.take<int64_t>((size_t)n_t * n_pad);
  int64_t *rowsum = sc.take<int64_t>((size_t)n_t * n_pad);
  RunningRowsOp::T *agg = sc.take<RunningRowsOp::T>(div_up((uint64_t)n_t * n_pad, kScanTile) + 1);
  if (!colsum || !rowsum || !agg) return CP_ERR_SCRATCH;
  if ((uint64_t)n_t * n_pad >= 0x80000000ull) return CP_ERR_UNSUPPORTED;
  const dim3 tiles(n_t, n_t);
  sat_tile_sums_kernel<<<tiles, 64, 0, stream>>>(attn, n, ld, n_pad, colsum, rowsum);
  sat_exclusive_over_tiles_kernel<<<dim3(div_up(n_pad, 64), 2), 64, 0, stream>>>(colsum, rowsum, n_t, n_pad);
  RunningRowsOp op{rowsum, n_pad, n_t * n_pad};
  if (int32_t rc = run_scan<RunningRowsOp>(stream, op, n_t * n_pad, agg)) return rc;
  sat_apply_kernel<<<tiles, 64, 0, stream>>>(attn, n, ld, n_pad, colsum, rowsum, T);
  return check_launch();
}

extern "C" int32_t cp_annotate(void *stream_, const int64_t *T, uint32_t n, const uint8_t *mask, uint32_t min_len,
                               uint32_t rho_percent, uint32_t *best_l, uint32_t *best_r, int64_t *best_score,
                               uint8_t *reusable, uint8_t *recompute, uint8_t *store_mask, void *scratch,
                               size_t scratch_bytes) {
  using namespace cp;
  hipStream_t stream = (hipStream_t)stream_;
  if (n == 0) return CP_OK;
  if (n > (1u << 20)) return CP_ERR_UNSUPPORTED;
  if (!T || !mask || !best_l || !best_r || !best_score || !reusable || !recompute || !scratch || !aligned(scratch, 256))
    return CP_ERR_INVALID_ARG;
  if (rho_percent > 100) return CP_ERR_INVALID_ARG;
  if (scratch_bytes < cp_sat_scratch_bytes(n)) return CP_ERR_SCRATCH;
  if (min_len == 0) min_len = 1;
  Scratch sc(scratch, scratch_bytes);
  uint32_t *agg = sc.take<uint32_t>(div_up(n, kScanTile) + 1);
  uint32_t *seg_a = sc.take<uint32_t>(n);
  int64_t *diag = sc.take<int64_t>(n);
  uint64_t *best_u = sc.take<uint64_t>(n);
  uint64_t *best_lr = sc.take<uint64_t>(n);
  int64_t *d = sc.take<int64_t>(n);
  uint32_t *rank = sc.take<uint32_t>(n);
  if (!agg || !seg_a || !diag || !best_u || !best_lr || !d || !rank) return CP_ERR_SCRATCH;
  SegStartOp so{mask, seg_a, n};
  if (int32_t rc = run_scan<SegStartOp>(stream, so, n, agg)) return rc;
  const uint32_t blocks = div_up(n, 256), n_t = div_up(n, kTile);
  annotate_init_kernel<<<blocks, 256, 0, stream>>>(T, n, diag, best_u, best_lr);
  for (int pass = 0; pass < 2; ++pass)
    annotate_search_kernel<<<dim3(n_t, n_t), 256, 0, stream>>>(T, n, diag, seg_a, min_len, pass, best_u, best_lr);
  annotate_finish_kernel<<<blocks, 256, 0, stream>>>(T, n, diag, seg_a, best_u, best_lr, best_l, best_r, best_score,
                                                     reusable, store_mask, d, rank);
  if (rho_percent)
    annotate_rank_kernel<<<dim3(blocks, div_up(n, kRankChunk)), 256, 0, stream>>>(n, best_l, best_r, reusable, d, rank);
  annotate_mark_kernel<<<blocks, 256, 0, stream>>>(n, best_l, best_r, reusable, rank, rho_percent, recompute);
  return check_launch();
}

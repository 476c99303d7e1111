// The KV annotator's arithmetic (Sec. 4.2.1 "C1", Steps 1-3): summed-area table of the attention
// matrix, the substring of every coarse segment with the largest intra - inter attention, and the
// ranking that picks the tokens to recompute.
//
// Exact arithmetic: every weight x becomes the integer round(x * 2^32) (entries above the diagonal,
// non-finite and huge values count as 0) and all sums are 64-bit integers.  Integer addition is
// associative, so the table does not depend on how the work is split, the maximum over the
// substrings is decided without rounding, and results are reproducible bit for bit.
//
// No token attends to a later one, so T[i][j] = T[i][i] for j > i: tiles strictly above the diagonal
// are neither computed nor written, and nothing here reads them.
//
// Step 1 (cp_sat_build), three sweeps over tiles of 64 rows x 128 columns that reach the diagonal or
// lie below it, one wavefront per tile, every lane owning two adjacent columns:
//   sums   per tile: the sum of every column over the tile's rows (lane-local), the running sum of the
//          row totals down the tile's rows (eight rows are reduced over the lanes together, see
//          sum8_over_lanes) and the tile's total
//   carry  exclusive scans of the three over the tile rows / tile columns / tile rows
//   apply  per tile and row: prefix over the lane's two columns, one wave scan across lanes, running
//          sum down the rows, + what lies above the tile in its columns + what lies left of it in
//          rows <= i (left of it in the tile's own rows + the totals of the tiles above those)
// Wave scans are DPP moves (no LDS).  When the row strides allow it a lane reads its two weights as
// one 8-byte vector and stores its two table entries as one 16-byte vector, so that a wavefront's
// store is one contiguous KiB.  Loads of the next eight rows are issued before the current eight
// are summed.  The lower half of the matrix is read twice
// (4 bytes per entry each) and the lower half of the table written once (8 bytes per entry).
//
// Step 2 (cp_annotate): score(l, r) = Intra - Inter = T[r,r] - T[l-1,r] - 2 T[r,l-1] + 2 T[l-1,l-1]
// = T[r,r] + T[l-1,l-1] - 2 T[r,l-1]  (T[l-1,r] = T[l-1,l-1], see above).  A workgroup takes a 64 x 64
// block of the (l, r) triangle: lanes along l, so that T[r, l-1] is read row by row in contiguous pieces,
// and keeps for every l the best (score, smallest r).  Two small passes over the tokens then find every
// segment's maximum score (64-bit atomic max) and the smallest (l, r) among the l that reach it (atomic min).
#include "cp_device.h"
#include "cp_internal.h"

namespace cp {
namespace {

constexpr uint32_t kTile = 64;    // rows of a table tile; also the block edge of the (l, r) search
constexpr uint32_t kTileC = 128;  // columns of a table tile: two per lane
constexpr uint32_t kNone = 0xFFFFFFFFu;
constexpr uint64_t kBias = 0x8000000000000000ull;  // signed -> unsigned, order preserving

// round(x * 2^32), ties to even, as a 64-bit integer; 0 above the diagonal and for values that are not
// finite or beyond 2^18 in magnitude.  x * 2^32 is exact in double; adding 2^52 + 2^51 leaves a double
// whose unit in the last place is 1, i.e. the hardware addition does the rounding, and the integer is
// the difference of the bit patterns.
__device__ __forceinline__ int64_t quantise(float x, uint32_t i, uint32_t j) {
  if (j > i || !(fabsf(x) <= 262144.0f)) return 0;
  const double magic = 6755399441055744.0;
  const double d = (double)x * 4294967296.0 + magic;
  return (int64_t)(__double_as_longlong(d) - __double_as_longlong(magic));
}

// The same integer plus the bit pattern of the rounding constant (kMagicBits): what the hardware addition
// leaves behind.  Sums of these are corrected once, by the number of terms times kMagicBits, instead of
// once per weight; a weight that counts as 0 is replaced before the conversion, so it contributes
// exactly kMagicBits.
constexpr uint64_t kMagicBits = 0x4338000000000000ull;  // 2^52 + 2^51 as a double
__device__ __forceinline__ uint64_t quantise_biased(float x, uint32_t i, uint32_t j) {
  if (j > i || !(fabsf(x) <= 262144.0f)) x = 0.0f;
  return (uint64_t)__double_as_longlong((double)x * 4294967296.0 + 6755399441055744.0);
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
__device__ __forceinline__ uint64_t shfl_xor_u64(uint64_t v, int m) {
  const uint32_t lo = __shfl_xor((uint32_t)v, m, kWave), hi = __shfl_xor((uint32_t)(v >> 32), m, kWave);
  return ((uint64_t)hi << 32) | lo;
}
__device__ __forceinline__ int64_t readlane_i64(int64_t v, uint32_t lane) {  // lane: same for the whole wave
  const uint32_t lo = __builtin_amdgcn_readlane((int)(uint32_t)v, lane);
  const uint32_t hi = __builtin_amdgcn_readlane((int)(uint32_t)((uint64_t)v >> 32), lane);
  return (int64_t)(((uint64_t)hi << 32) | lo);
}

// The sums below run modulo 2^64 on unsigned words (they carry multiples of kMagicBits that wrap).
template <int CTRL>
__device__ __forceinline__ uint64_t dpp_move_u64(uint64_t v) {  // CTRL: a permutation inside rows, every lane has a source
  const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)v, CTRL, 0xF, 0xF, false);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(v >> 32), CTRL, 0xF, 0xF, false);
  return ((uint64_t)hi << 32) | lo;
}
// a + b with the halves of the wavefront (HALF = 32) or the odd and even rows of 16 lanes (HALF = 16)
// exchanged first: lanes whose bit HALF is clear get a[lane] + a[lane ^ HALF], the others
// b[lane] + b[lane ^ HALF].  One swap instruction per 32-bit half, no select.
template <int HALF>
__device__ __forceinline__ uint64_t swap_add(uint64_t a, uint64_t b) {
  const uint32_t alo = (uint32_t)a, ahi = (uint32_t)(a >> 32), blo = (uint32_t)b, bhi = (uint32_t)(b >> 32);
  const auto lo = HALF == 32 ? __builtin_amdgcn_permlane32_swap(alo, blo, false, false)
                             : __builtin_amdgcn_permlane16_swap(alo, blo, false, false);
  const auto hi = HALF == 32 ? __builtin_amdgcn_permlane32_swap(ahi, bhi, false, false)
                             : __builtin_amdgcn_permlane16_swap(ahi, bhi, false, false);
  return (((uint64_t)hi[0] << 32) | lo[0]) + (((uint64_t)hi[1] << 32) | lo[1]);
}
// Eight sums over the 64 lanes at once: returns, in every lane L, the sum of v[L >> 3] over all lanes.
// Each exchange halves the number of values a lane still carries (8 -> 4 -> 2 -> 1), then three
// more steps add up the eight lanes that hold parts of the same sum: 10 exchanges instead of 48.
__device__ __forceinline__ uint64_t sum8_over_lanes(const uint64_t v[8]) {
  uint64_t w[4], x[2];
#pragma unroll
  for (int u = 0; u < 4; ++u) w[u] = swap_add<32>(v[u], v[u + 4]);  // lane bit 5 picks v[u] or v[u + 4]
#pragma unroll
  for (int u = 0; u < 2; ++u) x[u] = swap_add<16>(w[u], w[u + 2]);  // lane bit 4
  const bool up = (threadIdx.x & 8) != 0;                           // lane bit 3
  uint64_t y = (up ? x[1] : x[0]) + dpp_move_u64<0x128>(up ? x[0] : x[1]);  // row_ror:8 = lane ^ 8
  y += dpp_move_u64<0xB1>(y);   // quad_perm [1,0,3,2]: lane ^ 1
  y += dpp_move_u64<0x4E>(y);   // quad_perm [2,3,0,1]: lane ^ 2
  y += dpp_move_u64<0x141>(y);  // row_half_mirror: the other quad of the same eight lanes
  return y;
}

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef long long i64x2 __attribute__((ext_vector_type(2)));

constexpr int kRowGroup = 8;  // rows whose loads are in flight while the previous rows are being summed

// Weights of one row, columns c and c+1 (c even), from p = &attn[row][c].
// INTERIOR: the whole tile lies on or below the diagonal and inside the matrix, nothing to check;
// otherwise columns beyond the row index r (and rows beyond n) read as 0.
template <bool VEC, bool INTERIOR>
__device__ __forceinline__ f32x2 load_x2(const float *__restrict__ p, uint32_t n, uint32_t r, uint32_t c) {
  if (INTERIOR) {
    if (VEC) return *reinterpret_cast<const f32x2 *>(p);
    return f32x2{p[0], p[1]};
  }
  f32x2 v = {0.0f, 0.0f};
  if (r < n && c <= r) {
    if (VEC && c + 1 <= r) {  // c + 1 <= r < n <= ld: both inside the row
      v = *reinterpret_cast<const f32x2 *>(p);
    } else {
      v.x = p[0];
      if (c + 1 <= r) v.y = p[1];
    }
  }
  return v;
}
template <bool VEC, bool INTERIOR>
__device__ __forceinline__ void load_group(const float *__restrict__ p, uint64_t ld, uint32_t n, uint32_t r_first,
                                           uint32_t c, f32x2 x[kRowGroup]) {
#pragma unroll
  for (int u = 0; u < kRowGroup; ++u) x[u] = load_x2<VEC, INTERIOR>(p + (uint64_t)u * ld, n, r_first + u, c);
}
// In an interior tile every column is at or left of the diagonal: only the range check remains.
template <bool INTERIOR>
__device__ __forceinline__ void quantise2(f32x2 v, uint32_t r, uint32_t c, int64_t q[2]) {
  const uint32_t i = INTERIOR ? 0xFFFFFFFFu : r;
  q[0] = quantise(v.x, i, c), q[1] = quantise(v.y, i, c + 1);
}

// col[0..1]: this lane's two column sums over the tile's rows.  Returns in lane k the sum of the tile's
// rows 0..k (all columns); lane 63 thus holds the tile's total.
template <bool VEC, bool INTERIOR>
__device__ __forceinline__ int64_t tile_sums(const float *__restrict__ attn, uint32_t n, uint64_t ld, uint32_t r0,
                                             uint32_t c, int64_t col[2]) {
  static_assert(kRowGroup == 8, "sum8_over_lanes reduces eight rows at a time");
  const float *p = attn + (uint64_t)r0 * ld + c;
  f32x2 cur[kRowGroup], nxt[kRowGroup];
  load_group<VEC, INTERIOR>(p, ld, n, r0, c, cur);
  // every sum here carries kMagicBits per weight (modulo 2^64), taken off where the sum is complete
  uint64_t col0 = 0, col1 = 0, running = 0, mine = 0;  // running: the same in every lane
#pragma unroll 1
  for (uint32_t g = 0; g < kTile / kRowGroup; ++g) {
    p += (uint64_t)kRowGroup * ld;
    if (g + 1 < kTile / kRowGroup) load_group<VEC, INTERIOR>(p, ld, n, r0 + (g + 1) * kRowGroup, c, nxt);
    uint64_t part[kRowGroup];
#pragma unroll
    for (int u = 0; u < kRowGroup; ++u) {
      const uint32_t i = INTERIOR ? 0xFFFFFFFFu : r0 + g * kRowGroup + u;
      const uint64_t q0 = quantise_biased(cur[u].x, i, c), q1 = quantise_biased(cur[u].y, i, c + 1);
      col0 += q0, col1 += q1;
      part[u] = q0 + q1;
    }
    const uint64_t rows = sum8_over_lanes(part);  // lanes 8u .. 8u+7: the total of row u of this group
#pragma unroll
    for (int u = 0; u < kRowGroup; ++u) {
      running += (uint64_t)readlane_i64((int64_t)rows, 8 * u) - (uint64_t)kTileC * kMagicBits;
      if (threadIdx.x == g * kRowGroup + u) mine = running;
    }
#pragma unroll
    for (int u = 0; u < kRowGroup; ++u) cur[u] = nxt[u];
  }
  col[0] = (int64_t)(col0 - (uint64_t)kTile * kMagicBits), col[1] = (int64_t)(col1 - (uint64_t)kTile * kMagicBits);
  return (int64_t)mine;
}

// colsum[I][c]: sum of column c over the 64 rows of tile row I (width n_pad_c);  rowrun[J][r]: sum of
// the rows r0..r of r's tile row over the 128 columns of tile column J (width n_pad_r);
// tilesum[I][J]: the tile's total (width n_j).
template <bool VEC>
__global__ __launch_bounds__(64) void sat_tile_sums_kernel(const float *__restrict__ attn, uint32_t n, uint64_t ld,
                                                           uint32_t n_pad_c, uint32_t n_pad_r,
                                                           int64_t *__restrict__ colsum, int64_t *__restrict__ rowrun,
                                                           int64_t *__restrict__ tilesum) {
  const uint32_t J = blockIdx.x, I = blockIdx.y, lane = threadIdx.x;
  const uint32_t c0 = J * kTileC, r0 = I * kTile, c = c0 + 2 * lane;
  int64_t col[2] = {0, 0};
  int64_t run = 0;  // a tile that lies above the diagonal as a whole holds no weight
  if (c0 + kTileC - 1 <= r0 && r0 + kTile <= n) {
    run = tile_sums<VEC, true>(attn, n, ld, r0, c, col);
  } else if (c0 <= r0 + kTile - 1) {
    run = tile_sums<VEC, false>(attn, n, ld, r0, c, col);
  }
  rowrun[(uint64_t)J * n_pad_r + r0 + lane] = run;
  if (lane == kWave - 1) tilesum[(uint64_t)I * gridDim.x + J] = run;
  colsum[(uint64_t)I * n_pad_c + c] = col[0];
  colsum[(uint64_t)I * n_pad_c + c + 1] = col[1];
}

// In place, for three arrays (blockIdx.y picks one): a[k][x] <- sum of a[k'][x] over k' < k   (x < width, k < n_k).
__global__ __launch_bounds__(64) void sat_exclusive_over_tiles_kernel(int64_t *a0, uint32_t n_k0, uint32_t width0,
                                                                      int64_t *a1, uint32_t n_k1, uint32_t width1,
                                                                      int64_t *a2, uint32_t n_k2, uint32_t width2) {
  int64_t *a = blockIdx.y == 0 ? a0 : blockIdx.y == 1 ? a1 : a2;
  const uint32_t n_k = blockIdx.y == 0 ? n_k0 : blockIdx.y == 1 ? n_k1 : n_k2;
  const uint32_t n_pad = blockIdx.y == 0 ? width0 : blockIdx.y == 1 ? width1 : width2;
  const uint32_t x = blockIdx.x * blockDim.x + threadIdx.x;
  if (x >= n_pad) return;
  int64_t run = 0;
  constexpr int kBatch = 32;  // independent loads in flight: the walk down a column is latency, not bandwidth
  for (uint32_t k = 0; k < n_k; k += kBatch) {
    int64_t v[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) v[u] = k + u < n_k ? a[(uint64_t)(k + u) * n_pad + x] : 0;
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      if (k + u < n_k) a[(uint64_t)(k + u) * n_pad + x] = run;
      run += v[u];
    }
  }
}

template <bool VEC_LD, bool VEC_ST, bool INTERIOR>
__device__ __forceinline__ void tile_apply(const float *__restrict__ attn, uint32_t n, uint64_t ld, uint32_t r0,
                                           uint32_t c, const int64_t above_pref[2], int64_t left_row,
                                           int64_t *__restrict__ T) {
  int64_t acc[2] = {0, 0};  // this tile's rows so far, tile's columns up to each of this lane's
  const float *p = attn + (uint64_t)r0 * ld + c;
  int64_t *t = T + (uint64_t)r0 * n + c;
  f32x2 cur[kRowGroup], nxt[kRowGroup];
  load_group<VEC_LD, INTERIOR>(p, ld, n, r0, c, cur);
#pragma unroll 1
  for (uint32_t g = 0; g < kTile / kRowGroup; ++g) {
    if (!INTERIOR && r0 + g * kRowGroup >= n) break;  // same for the whole wave
    p += (uint64_t)kRowGroup * ld;
    if (g + 1 < kTile / kRowGroup) load_group<VEC_LD, INTERIOR>(p, ld, n, r0 + (g + 1) * kRowGroup, c, nxt);
#pragma unroll
    for (int u = 0; u < kRowGroup; ++u) {
      const uint32_t k = g * kRowGroup + u, r = r0 + k;
      int64_t q[2];
      quantise2<INTERIOR>(cur[u], r, c, q);
      q[1] += q[0];
      const int64_t before = wave_inclusive_sum(q[1]) - q[1];
      const int64_t lv = readlane_i64(left_row, k);
      acc[0] += before + q[0], acc[1] += before + q[1];
      const int64_t out0 = acc[0] + above_pref[0] + lv, out1 = acc[1] + above_pref[1] + lv;
      if (INTERIOR || r < n) {  // same for the whole wave
        int64_t *o = t + (uint64_t)u * n;
        if (VEC_ST && (INTERIOR || c + 1 < n)) {  // the wave writes 1 KiB in one piece
          __builtin_nontemporal_store(i64x2{out0, out1}, reinterpret_cast<i64x2 *>(o));
        } else {
          if (c < n) o[0] = out0;
          if (c + 1 < n) o[1] = out1;
        }
      }
    }
    t += (uint64_t)kRowGroup * n;
#pragma unroll
    for (int u = 0; u < kRowGroup; ++u) cur[u] = nxt[u];
  }
}

// With the sensitivity mask known, the table is needed only where a substring search can look: in the
// rows of a coarse segment [a, b], the columns from a - 1 on (and the diagonal, for every row).
// need_from[I] = the smallest such a over the non-sensitive rows of tile row I (kNone: all its rows are
// sensitive).  One workgroup: per tile row its first non-sensitive row and its last sensitive one, a
// running maximum over the latter, and the segment start follows from the two.
constexpr uint32_t kMaxTileRows = 4096;  // 2^18 rows / 64; larger requests get the whole table
__global__ __launch_bounds__(1024) void sat_need_from_kernel(const uint8_t *__restrict__ mask, uint32_t n,
                                                             uint32_t n_i, uint32_t *__restrict__ need_from) {
  __shared__ uint32_t first[kMaxTileRows];  // the first non-sensitive row of tile row I (kNone: none)
  __shared__ uint32_t last[kMaxTileRows];   // 1 + the last sensitive row at or before the end of tile row I (0: none)
  __shared__ uint32_t carry;
  if (threadIdx.x == 0) carry = 0;
  // a wavefront's 64 lanes are the 64 rows of one tile row: two ballots say where it stands
  for (uint32_t r0 = threadIdx.x / kWave * kTile; r0 < n; r0 += blockDim.x) {  // the same for a whole wavefront
    const uint32_t r = r0 + (threadIdx.x & (kWave - 1));
    const unsigned long long sens = __ballot(r < n && mask[r] != 0), open = __ballot(r < n && mask[r] == 0);
    if ((threadIdx.x & (kWave - 1)) == 0) {
      first[r0 / kTile] = open ? r0 + (uint32_t)__ffsll(open) - 1 : kNone;
      last[r0 / kTile] = sens ? r0 + 64 - (uint32_t)__clzll(sens) : 0;
    }
  }
  __syncthreads();
  // inclusive running maximum over last[], a chunk of blockDim.x entries at a time
  for (uint32_t base = 0; base < n_i; base += blockDim.x) {
    const uint32_t I = base + threadIdx.x;
    const uint32_t width = n_i - base < blockDim.x ? n_i - base : blockDim.x;
    for (uint32_t step = 1; step < width; step <<= 1) {
      uint32_t other = 0;
      if (I < n_i && threadIdx.x >= step) other = last[I - step];
      __syncthreads();
      if (I < n_i && other > last[I]) last[I] = other;
      __syncthreads();
    }
    if (I < n_i && carry > last[I]) last[I] = carry;
    __syncthreads();
    if (threadIdx.x == 0) carry = last[base + width - 1];
    __syncthreads();
  }
  for (uint32_t I = threadIdx.x; I < n_i; I += blockDim.x) {
    uint32_t a = first[I];
    // a segment that starts inside the tile row starts at its first non-sensitive row (the rows before it are
    // sensitive); one that reaches in from above starts right after the last sensitive row before the tile row
    if (a != kNone && a == I * kTile) a = I ? last[I - 1] : 0;
    need_from[I] = a;
  }
}

template <bool VEC_LD, bool VEC_ST>
__global__ __launch_bounds__(64) void sat_apply_kernel(const float *__restrict__ attn, uint32_t n, uint64_t ld,
                                                       uint32_t n_pad_c, uint32_t n_pad_r,
                                                       const int64_t *__restrict__ above,
                                                       const int64_t *__restrict__ left,
                                                       const int64_t *__restrict__ tiles_above,
                                                       const uint32_t *__restrict__ need_from /* nullable */,
                                                       int64_t *__restrict__ T) {
  const uint32_t J = blockIdx.x, I = blockIdx.y, lane = threadIdx.x;
  const uint32_t c0 = J * kTileC, r0 = I * kTile, c = c0 + 2 * lane;
  if (c0 > r0 + kTile - 1) return;  // above the diagonal: not written
  if (need_from && c0 + kTileC <= r0) {  // not the tile that holds these rows' diagonal entries
    // the search stages whole 64-column blocks, so it loads columns down to a - 64
    const uint32_t a = need_from[I];
    if (a == kNone || c0 + kTileC + kTile <= a) return;  // left of everything a search looks at in these rows
  }
  // everything above the tile, in the tile's columns up to each of this lane's
  int64_t above_pref[2];
  {
    above_pref[0] = above[(uint64_t)I * n_pad_c + c];
    above_pref[1] = above_pref[0] + above[(uint64_t)I * n_pad_c + c + 1];
    const int64_t before = wave_inclusive_sum(above_pref[1]) - above_pref[1];  // the lanes to the left
    above_pref[0] += before, above_pref[1] += before;
  }
  // everything left of the tile in rows <= r0 + lane: in the tile's own rows, plus the tiles above those
  int64_t left_row = left[(uint64_t)J * n_pad_r + r0 + lane];
  {
    int64_t part = 0;  // tiles_above[I][j]: total of the tiles (I', j), I' < I
    for (uint32_t j = lane; j < J; j += kWave) part += tiles_above[(uint64_t)I * gridDim.x + j];
    left_row += readlane_i64(wave_inclusive_sum(part), kWave - 1);
  }
  if (c0 + kTileC - 1 <= r0 && r0 + kTile <= n)
    tile_apply<VEC_LD, VEC_ST, true>(attn, n, ld, r0, c, above_pref, left_row, T);
  else
    tile_apply<VEC_LD, VEC_ST, false>(attn, n, ld, r0, c, above_pref, left_row, T);
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
                                                            const uint32_t *__restrict__ seg_a,
                                                            int64_t *__restrict__ diag, uint64_t *best_u,
                                                            uint64_t *best_lr, uint32_t *__restrict__ tile_min_a) {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;  // no lane leaves early: the wavefront reduces together
  uint32_t m = kNone;
  if (i < n) {
    diag[i] = T[(uint64_t)i * n + i];
    best_u[i] = 0;        // below every biased score
    best_lr[i] = ~0ull;   // above every packed (l, r)
    m = seg_a[i];
  }
  // a wavefront is one tile of 64 tokens: the earliest segment start among them (kNone if all are sensitive)
#pragma unroll
  for (int s = 1; s < kWave; s <<= 1) {
    const uint32_t o = __shfl_xor(m, s, kWave);
    m = o < m ? o : m;
  }
  if ((threadIdx.x & (kWave - 1)) == 0 && i < n) tile_min_a[i / kTile] = m;
}

// Candidates (l, r) are visited in 64 x 64 blocks: l in [lt*64, +64), r in [rt*64, +64), lt <= rt.
// Lanes run along l, so a row T[r][l0-1 ..] is read as one contiguous piece and nothing needs transposing.
// Workgroup (lt, y) takes the blocks rt = lt + y, lt + y + kSearchSplit, ... of its l tile, up to the
// first r tile all of whose segments start beyond the tile's l (segment starts never decrease with r);
// its four wavefronts take 16 rows of every block each.  It leaves, for every l of the tile, the best
// (score, r) it saw: part_u[y][l] = biased score (0 = no candidate), part_r[y][l] = the smallest r that
// reaches it.
constexpr uint32_t kSearchSplit = 16;
__global__ __launch_bounds__(256) void annotate_search_kernel(const int64_t *__restrict__ T, uint32_t n,
                                                              const int64_t *__restrict__ diag,
                                                              const uint32_t *__restrict__ seg_a,
                                                              const uint32_t *__restrict__ tile_min_a, uint32_t min_len,
                                                              uint64_t *__restrict__ part_u,
                                                              uint32_t *__restrict__ part_r) {
  __shared__ uint64_t group_u[4][kTile];
  __shared__ uint32_t group_r[4][kTile];
  const uint32_t lt = blockIdx.x, n_t = gridDim.x;
  const uint32_t lane = threadIdx.x & (kWave - 1), quarter = threadIdx.x / kWave;
  const uint32_t l = lt * kTile + lane, l_last = lt * kTile + kTile - 1;
  const int64_t d_l = (l >= 1 && l - 1 < n) ? diag[l - 1] : 0;
  const int64_t *col = T + (l ? l - 1 : 0);  // column l - 1 (not read for l = 0)
  bool have = false;
  int64_t best = 0;
  uint32_t best_r = 0;
  for (uint32_t rt = lt + blockIdx.y; rt < n_t; rt += kSearchSplit) {  // ascending r
    const uint32_t min_a = tile_min_a[rt];  // kNone: every token of that tile is sensitive
    if (min_a == kNone || min_a > l_last) break;  // it and every later r belong to segments that start after this tile
    const uint32_t r_first = rt * kTile + quarter * (kTile / 4);
    // everything this block needs is asked for before any of it is used: 16 table entries per lane, and the
    // segment start and diagonal entry of the 16 rows in lanes 0..15 (handed round with readlane below)
    uint32_t a_mine = kNone;
    int64_t d_mine = 0;
    if (r_first + (lane & 15) < n) a_mine = seg_a[r_first + (lane & 15)], d_mine = diag[r_first + (lane & 15)];
    int64_t tv[kTile / 4];
#pragma unroll
    for (uint32_t k = 0; k < kTile / 4; ++k) {
      const uint32_t r = r_first + k;
      tv[k] = (r < n && l >= 1 && l <= r) ? col[(uint64_t)r * n] : 0;  // (entries outside r's segment are not used)
    }
#pragma unroll
    for (uint32_t k = 0; k < kTile / 4; ++k) {
      const uint32_t r = r_first + k;  // the same for the whole wavefront
      const uint32_t a_r = __builtin_amdgcn_readlane(a_mine, k);  // kNone: r is sensitive or past the end
      const int64_t d_r = readlane_i64(d_mine, k);
      if (a_r == kNone || l < a_r || l > r || r - l + 1 < min_len) continue;
      const int64_t score = d_r + d_l - 2 * tv[k];
      if (!have || score > best) {  // r ascending: the smallest r stays on ties
        have = true;
        best = score;
        best_r = r;
      }
    }
  }
  // the four wavefronts looked at different r for the same l: the larger score wins, then the smaller r
  group_u[quarter][lane] = have ? (uint64_t)best ^ kBias : 0;
  group_r[quarter][lane] = best_r;
  __syncthreads();
  if (quarter == 0 && l < n) {
    uint64_t u = group_u[0][lane];
    uint32_t r = group_r[0][lane];
#pragma unroll
    for (int g = 1; g < 4; ++g) {
      const uint64_t ug = group_u[g][lane];
      const uint32_t rg = group_r[g][lane];
      if (ug > u || (ug == u && ug != 0 && rg < r)) u = ug, r = rg;
    }
    part_u[(uint64_t)blockIdx.y * n + l] = u;
    part_r[(uint64_t)blockIdx.y * n + l] = r;
  }
}

// Per l: the best (score, r) over the kSearchSplit parts; the maximum score of l's segment (atomic max).
__global__ __launch_bounds__(256) void annotate_best_score_kernel(uint32_t n, const uint32_t *__restrict__ seg_a,
                                                                  const uint64_t *__restrict__ part_u,
                                                                  const uint32_t *__restrict__ part_r,
                                                                  uint64_t *__restrict__ cand_u,
                                                                  uint32_t *__restrict__ cand_r, uint64_t *best_u) {
  const uint32_t l = blockIdx.x * blockDim.x + threadIdx.x;  // no lane leaves early: the wavefront reduces together
  uint64_t u = 0;
  uint32_t a = kNone;
  if (l < n) {
    u = part_u[l];
    uint32_t r = part_r[l];
#pragma unroll
    for (uint32_t y = 1; y < kSearchSplit; ++y) {
      const uint64_t uy = part_u[(uint64_t)y * n + l];
      const uint32_t ry = part_r[(uint64_t)y * n + l];
      if (uy > u || (uy == u && uy != 0 && ry < r)) u = uy, r = ry;
    }
    cand_u[l] = u;
    cand_r[l] = r;
    a = seg_a[l];
  }
  if (a == kNone) u = 0;  // sensitive or past the end: nothing to report
  // One atomic per wavefront where all lanes that have a segment have the same one (the usual case), else one per lane.
  const unsigned long long with_segment = __ballot(a != kNone);
  if (with_segment == 0) return;  // the same for the whole wavefront
  const uint32_t a_ref = __builtin_amdgcn_readlane(a, __ffsll(with_segment) - 1);
  if (__all(a == kNone || a == a_ref)) {
#pragma unroll
    for (int m = 1; m < kWave; m <<= 1) {
      const uint64_t o = shfl_xor_u64(u, m);
      u = o > u ? o : u;
    }
    if ((threadIdx.x & (kWave - 1)) == 0 && u != 0 && best_u[a_ref] < u)
      atomicMax((unsigned long long *)&best_u[a_ref], (unsigned long long)u);
  } else if (u != 0 && best_u[a] < u) {
    atomicMax((unsigned long long *)&best_u[a], (unsigned long long)u);
  }
}
// Among the l whose best score is their segment's maximum: the smallest (l, r) (atomic min).
__global__ __launch_bounds__(256) void annotate_best_lr_kernel(uint32_t n, const uint32_t *__restrict__ seg_a,
                                                               const uint64_t *__restrict__ cand_u,
                                                               const uint32_t *__restrict__ cand_r,
                                                               const uint64_t *__restrict__ best_u, uint64_t *best_lr) {
  const uint32_t l = blockIdx.x * blockDim.x + threadIdx.x;
  if (l >= n) return;
  const uint32_t a = seg_a[l];
  if (a == kNone || cand_u[l] == 0 || cand_u[l] != best_u[a]) return;
  atomicMin((unsigned long long *)&best_lr[a], (unsigned long long)(((uint64_t)l << 32) | cand_r[l]));
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
    inside = bl <= i && i <= br && score > 0;  // reuse criterion: intra-attention exceeds inter-attention
    if (inside) {
      // inter_i = T[i][bl-1] - T[i-1][bl-1];  intra_i = T[i][i] - T[i-1][i] - inter_i, T[i-1][i] = T[i-1][i-1]
      const int64_t t_i = bl ? T[(uint64_t)i * n + bl - 1] : 0;
      const int64_t t_p = (bl && i) ? T[(uint64_t)(i - 1) * n + bl - 1] : 0;
      const int64_t up = i ? diag[i - 1] : 0;
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
// earlier token first on ties.  Block (x, y): the 64 tokens i of block x against the chunks of tokens j that
// their substrings cover, every kRankSplit-th of them starting with the y-th; the partial counts are
// added up in rank[] (zeroed by the finish kernel).
constexpr uint32_t kRankChunk = 256, kRankSplit = 8;
__global__ __launch_bounds__(256) void annotate_rank_kernel(uint32_t n, const uint32_t *__restrict__ out_l,
                                                            const uint32_t *__restrict__ out_r,
                                                            const uint8_t *__restrict__ reusable,
                                                            const int64_t *__restrict__ d, uint32_t *rank) {
  __shared__ int64_t dj[kRankChunk];
  __shared__ uint32_t lo_all, hi_all;
  // a wavefront's lanes are 64 tokens; the workgroup's four wavefronts take a quarter of every chunk each
  const uint32_t i = blockIdx.x * kWave + (threadIdx.x & (kWave - 1)), quarter = threadIdx.x / kWave;
  const bool mine = i < n && reusable[i];
  const uint32_t bl = mine ? out_l[i] : kNone, br = mine ? out_r[i] : 0u;
  if (threadIdx.x == 0) {
    lo_all = kNone;
    hi_all = 0;
  }
  __syncthreads();
  {  // the span of tokens this workgroup's substrings cover: reduced inside each wavefront, then four atomics
    uint32_t lo = bl, hi = br;
#pragma unroll
    for (int m = 1; m < kWave; m <<= 1) {
      const uint32_t ol = __shfl_xor(lo, m, kWave), oh = __shfl_xor(hi, m, kWave);
      lo = ol < lo ? ol : lo;
      hi = oh > hi ? oh : hi;
    }
    if ((threadIdx.x & (kWave - 1)) == 0 && lo != kNone) {
      atomicMin(&lo_all, lo);
      atomicMax(&hi_all, hi);
    }
  }
  __syncthreads();
  if (lo_all == kNone) return;  // nothing reusable among these tokens
  const int64_t di = mine ? d[i] : 0;
  uint32_t count = 0;
  for (uint32_t chunk = lo_all / kRankChunk + blockIdx.y; chunk <= hi_all / kRankChunk; chunk += kRankSplit) {  // same for all
    const uint32_t j0 = chunk * kRankChunk, j = j0 + threadIdx.x;
    __syncthreads();  // the previous chunk is no longer read
    dj[threadIdx.x] = j < n ? d[j] : 0;
    __syncthreads();
    if (!mine) continue;
    const uint32_t q0 = j0 + quarter * (kRankChunk / 4), q1 = q0 + kRankChunk / 4 - 1;
    const uint32_t from = bl > q0 ? bl : q0, to = br < q1 ? br : q1;  // inclusive
    for (uint32_t jj = from; jj <= to; ++jj) {  // (empty if the substring does not reach into this quarter)
      const int64_t v = dj[jj - j0];
      count += (v > di || (v == di && jj < i)) ? 1u : 0u;
    }
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

}  // namespace
}  // namespace cp

extern "C" size_t cp_sat_scratch_bytes(uint32_t n) {
  using namespace cp;
  const uint64_t n_i = div_up(n, kTile), n_j = div_up(n, kTileC);
  const uint64_t cols = n_i * (n_j * kTileC), rows = n_j * (n_i * kTile);
  // column sums per tile row, running row sums per tile column, tile totals, per-token arrays of cp_annotate
  return (size_t)((cols + rows + n_i * n_j) * 8 + 4 * n_i + 320ull * n + 33 * 256);
}

extern "C" int32_t cp_sat_build(void *stream_, const float *attn, uint32_t n, uint64_t ld, const uint8_t *mask,
                                int64_t *T, void *scratch, size_t scratch_bytes) {
  using namespace cp;
  hipStream_t stream = (hipStream_t)stream_;
  if (n == 0) return CP_OK;
  if (n > (1u << 20)) return CP_ERR_UNSUPPORTED;
  if (!attn || !T || ld < n || !scratch || !aligned(scratch, 256) || !aligned(attn, 4) || !aligned(T, 8))
    return CP_ERR_INVALID_ARG;
  if (scratch_bytes < cp_sat_scratch_bytes(n)) return CP_ERR_SCRATCH;
  const uint32_t n_i = div_up(n, kTile), n_j = div_up(n, kTileC);
  const uint32_t n_pad_c = n_j * kTileC, n_pad_r = n_i * kTile;
  Scratch sc(scratch, scratch_bytes);
  int64_t *colsum = sc.take<int64_t>((size_t)n_i * n_pad_c);
  int64_t *rowsum = sc.take<int64_t>((size_t)n_j * n_pad_r);
  int64_t *tilesum = sc.take<int64_t>((size_t)n_i * n_j);
  if (n_i > kMaxTileRows) mask = nullptr;
  uint32_t *need_from = mask ? sc.take<uint32_t>(n_i) : nullptr;
  if (!colsum || !rowsum || !tilesum || (mask && !need_from)) return CP_ERR_SCRATCH;
  const bool vec_ld = ld % 2 == 0 && aligned(attn, 8);  // every (row, column pair) starts on 8 bytes
  const bool vec_st = n % 2 == 0 && aligned(T, 16);
  const dim3 tiles(n_j, n_i);
  if (mask) sat_need_from_kernel<<<1, 1024, 0, stream>>>(mask, n, n_i, need_from);
  if (vec_ld)
    sat_tile_sums_kernel<true><<<tiles, 64, 0, stream>>>(attn, n, ld, n_pad_c, n_pad_r, colsum, rowsum, tilesum);
  else
    sat_tile_sums_kernel<false><<<tiles, 64, 0, stream>>>(attn, n, ld, n_pad_c, n_pad_r, colsum, rowsum, tilesum);
  // above the tile (column sums over the tile rows before), left of it in its own rows (running row sums
  // over the tile columns before), and the totals of the tiles above each tile
  const uint32_t widest = n_pad_c > n_pad_r ? n_pad_c : n_pad_r;
  sat_exclusive_over_tiles_kernel<<<dim3(div_up(widest, 64), 3), 64, 0, stream>>>(
      colsum, n_i, n_pad_c, rowsum, n_j, n_pad_r, tilesum, n_i, n_j);
  if (vec_ld && vec_st)
    sat_apply_kernel<true, true><<<tiles, 64, 0, stream>>>(attn, n, ld, n_pad_c, n_pad_r, colsum, rowsum, tilesum, need_from, T);
  else if (vec_ld)
    sat_apply_kernel<true, false><<<tiles, 64, 0, stream>>>(attn, n, ld, n_pad_c, n_pad_r, colsum, rowsum, tilesum, need_from, T);
  else if (vec_st)
    sat_apply_kernel<false, true><<<tiles, 64, 0, stream>>>(attn, n, ld, n_pad_c, n_pad_r, colsum, rowsum, tilesum, need_from, T);
  else
    sat_apply_kernel<false, false><<<tiles, 64, 0, stream>>>(attn, n, ld, n_pad_c, n_pad_r, colsum, rowsum, tilesum, need_from, T);
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
  uint32_t *tile_min_a = sc.take<uint32_t>(div_up(n, kTile));
  uint64_t *part_u = sc.take<uint64_t>((size_t)kSearchSplit * n);
  uint32_t *part_l = sc.take<uint32_t>((size_t)kSearchSplit * n);
  uint64_t *cand_u = sc.take<uint64_t>(n);
  uint32_t *cand_l = sc.take<uint32_t>(n);
  if (!agg || !seg_a || !diag || !best_u || !best_lr || !d || !rank || !tile_min_a || !part_u || !part_l || !cand_u ||
      !cand_l)
    return CP_ERR_SCRATCH;
  SegStartOp so{mask, seg_a, n};
  if (int32_t rc = run_scan<SegStartOp>(stream, so, n, agg)) return rc;
  const uint32_t blocks = div_up(n, 256), n_t = div_up(n, kTile);
  annotate_init_kernel<<<blocks, 256, 0, stream>>>(T, n, seg_a, diag, best_u, best_lr, tile_min_a);
  annotate_search_kernel<<<dim3(n_t, kSearchSplit), 256, 0, stream>>>(T, n, diag, seg_a, tile_min_a, min_len, part_u,
                                                                      part_l);
  annotate_best_score_kernel<<<blocks, 256, 0, stream>>>(n, seg_a, part_u, part_l, cand_u, cand_l, best_u);
  annotate_best_lr_kernel<<<blocks, 256, 0, stream>>>(n, seg_a, cand_u, cand_l, best_u, best_lr);
  annotate_finish_kernel<<<blocks, 256, 0, stream>>>(T, n, diag, seg_a, best_u, best_lr, best_l, best_r, best_score,
                                                     reusable, store_mask, d, rank);
  if (rho_percent)
    annotate_rank_kernel<<<dim3(div_up(n, kWave), kRankSplit), 256, 0, stream>>>(n, best_l, best_r, reusable, d, rank);
  annotate_mark_kernel<<<blocks, 256, 0, stream>>>(n, best_l, best_r, reusable, rank, rho_percent, recompute);
  return check_launch();
}

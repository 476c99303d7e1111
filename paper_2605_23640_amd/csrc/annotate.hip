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
#include <type_traits>

#include "cp_device.h"
#include "cp_internal.h"

namespace cp {
namespace {

constexpr uint32_t kTile = 64;    // rows of a table tile; also the block edge of the (l, r) search
constexpr uint32_t kTileC = 128;  // columns of a table tile: two per lane
constexpr uint32_t kNone = 0xFFFFFFFFu;
constexpr uint64_t kBias = 0x8000000000000000ull;  // signed -> unsigned, order preserving

// A weight x counts as round(x * 2^32), ties to even, a 64-bit integer; 0 above the diagonal (read as 0.0f
// by load_x2) and for values that are not finite or beyond 2^18 in magnitude (replaced by 0.0f by the callers).
// A double in [2^20, 2^21) has a unit in the last place of 2^-32, so adding 2^20 + 2^19 to the weight makes
// the hardware addition do the rounding, and the low 52 bits of the result are 2^51 + the wanted integer:
// quantise_biased returns the integer plus kMagicBits.  Sums of these are corrected once, by the number of
// terms times kMagicBits (modulo 2^64), instead of once per weight.
constexpr double kMagic = 1572864.0;                    // 2^20 + 2^19
constexpr uint64_t kMagicBits = 0x4138000000000000ull;  // its bit pattern
__device__ __forceinline__ uint64_t quantise_biased(float x) {
  return (uint64_t)__double_as_longlong((double)x + kMagic);
}
// All weights a lane holds in range?  Compared as integers: a float x >= 0 is in range iff its
// bit pattern, read as a signed integer, is at most that of 2^18; a float with the sign bit set iff its
// pattern, read as unsigned, is at most that of -2^18 (NaN and infinity lie above both bounds).
constexpr int32_t kMaxPosBits = 0x48800000;
constexpr uint32_t kMaxNegBits = 0xC8800000u;

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
// Eight rows from r_first on.  row0 = &attn[r_first][first column of the tile] is the same for the whole
// wavefront and the lane's part of the address is the 32-bit offset c_in_tile, so that the loads take their
// base from scalar registers and no lane computes a 64-bit address.
template <bool VEC, bool INTERIOR>
__device__ __forceinline__ void load_group(const float *__restrict__ row0, uint64_t ld, uint32_t n, uint32_t r_first,
                                           uint32_t c, uint32_t c_in_tile, f32x2 x[kRowGroup]) {
#pragma unroll
  for (int u = 0; u < kRowGroup; ++u)
    x[u] = load_x2<VEC, INTERIOR>(row0 + (uint64_t)u * ld + c_in_tile, n, r_first + u, c);
}
// One group of eight rows: adds this lane's 16 weights to its two column sums and returns, in the lanes
// 8u .. 8u+7, the total of row u over the wavefront's 128 columns.  Every sum carries kMagicBits per weight.
template <bool CHECKED>
__device__ __forceinline__ uint64_t sum_row_group(const f32x2 (&x)[kRowGroup], uint64_t &col0, uint64_t &col1) {
  uint64_t part[kRowGroup];
#pragma unroll
  for (int u = 0; u < kRowGroup; ++u) {
    float a = x[u].x, b = x[u].y;
    if (CHECKED) {
      a = fabsf(a) <= 262144.0f ? a : 0.0f;
      b = fabsf(b) <= 262144.0f ? b : 0.0f;
    }
    const uint64_t q0 = quantise_biased(a), q1 = quantise_biased(b);
    col0 += q0, col1 += q1;
    part[u] = q0 + q1;
  }
  return sum8_over_lanes(part);
}

// A workgroup of four wavefronts sums one tile; wavefront w takes the rows 16w .. 16w + 15 (two groups of eight,
// all requested at once).  Returns this lane's two column sums over the wavefront's rows in col[], and in the lanes
// k < 16 the sum of the wavefront's rows 0 .. k over all columns (lane 15: all its rows; 0 in the other lanes).
// Weights above the diagonal or outside the matrix were read as 0 (load_x2), so only the range of the values is left
// to check, and that is done for a group at once: the per-weight test runs only where a wavefront has met a value
// out of range.
constexpr uint32_t kSumWaves = 4, kSumRows = kTile / kSumWaves;
template <bool VEC, bool INTERIOR>
__device__ __forceinline__ int64_t quarter_tile_sums(const float *__restrict__ attn, uint32_t n, uint64_t ld,
                                                     uint32_t r_first, uint32_t c, uint32_t lane, int64_t col[2]) {
  static_assert(kRowGroup == 8 && kSumRows == 16, "two groups of eight rows; sum8_over_lanes reduces eight rows at a time");
  const uint32_t c_in_tile = 2 * lane;
  const float *p = attn + (uint64_t)r_first * ld + (c - c_in_tile);  // the first weight of these rows: the same in every lane
  uint64_t col0 = 0, col1 = 0, keep = 0;
  auto take = [&](const f32x2 (&x)[kRowGroup], uint32_t g) {
    int32_t hi_pos = (int32_t)0x80000000;
    uint32_t hi_neg = 0;
#pragma unroll
    for (int u = 0; u < kRowGroup; ++u) {
      const uint32_t bx = __float_as_uint(x[u].x), by = __float_as_uint(x[u].y);
      hi_pos = max(hi_pos, max((int32_t)bx, (int32_t)by));
      hi_neg = max(hi_neg, max(bx, by));
    }
    const bool out_of_range = hi_pos > kMaxPosBits || hi_neg > kMaxNegBits;
    const uint64_t rows = __builtin_expect(__ballot(out_of_range) != 0, 0) ? sum_row_group<true>(x, col0, col1)
                                                                           : sum_row_group<false>(x, col0, col1);
    if ((lane & 7) == g) keep = rows;  // lane 8u + g: the total of row 8g + u
  };
  f32x2 xa[kRowGroup], xb[kRowGroup];
  load_group<VEC, INTERIOR>(p, ld, n, r_first, c, c_in_tile, xa);
  load_group<VEC, INTERIOR>(p + (uint64_t)kRowGroup * ld, ld, n, r_first + kRowGroup, c, c_in_tile, xb);
  take(xa, 0);
  take(xb, 1);
  col[0] = (int64_t)(col0 - (uint64_t)kSumRows * kMagicBits), col[1] = (int64_t)(col1 - (uint64_t)kSumRows * kMagicBits);
  // lane k < 16 fetches the total of row k = 8g + u from lane 8u + g, then the running sum down the rows is one wave scan
  const uint32_t from = 8 * (lane & 7) + ((lane >> 3) & 1);
  const uint32_t lo = __shfl((uint32_t)keep, (int)from, kWave), hi = __shfl((uint32_t)(keep >> 32), (int)from, kWave);
  const uint64_t row_total = lane < kSumRows ? (((uint64_t)hi << 32) | lo) - (uint64_t)kTileC * kMagicBits : 0;
  return wave_inclusive_sum((int64_t)row_total);
}

// Tiles that reach the diagonal or lie below it: tile row I holds the tile columns 0 .. I/2, so the rows 2m and
// 2m + 1 hold m + 1 tiles each and m(m + 1) tiles come before row 2m.  Tiles are numbered in that order.
__host__ __device__ inline uint64_t tiles_before_row(uint32_t I) {
  const uint64_t m = I / 2;
  return m * (m + 1) + (I & 1 ? m + 1 : 0);
}
__device__ __forceinline__ void tile_of(uint32_t t, uint32_t &I, uint32_t &J) {
  uint32_t m = (uint32_t)((sqrt(4.0 * (double)t + 1.0) - 1.0) * 0.5);
  while ((uint64_t)m * (m + 1) > t) --m;
  while ((uint64_t)(m + 1) * (m + 2) <= t) ++m;
  const uint32_t rest = t - m * (m + 1);
  // (computed with vector instructions from a value every lane shares: hand the results back to scalar registers)
  I = __builtin_amdgcn_readfirstlane(rest <= m ? 2 * m : 2 * m + 1);
  J = __builtin_amdgcn_readfirstlane(rest <= m ? rest : rest - (m + 1));
}

// colsum[I][c]: sum of column c over the 64 rows of tile row I (width n_pad_c);  rowrun[J][r]: sum of
// the rows r0..r of r's tile row over the 128 columns of tile column J (width n_pad_r);
// tilesum[I][J]: the tile's total (width n_j).  One workgroup per tile on or below the diagonal; the
// entries of the three arrays that belong to tiles above it are neither written nor read.
template <bool VEC>
__global__ __launch_bounds__(kSumWaves *kWave) void sat_tile_sums_kernel(
    const float *__restrict__ attn, uint32_t n, uint64_t ld, uint32_t n_pad_c, uint32_t n_pad_r, uint32_t n_j,
    int64_t *__restrict__ colsum, int64_t *__restrict__ rowrun, int64_t *__restrict__ tilesum) {
  __shared__ int64_t colpart[kSumWaves][kWave][2];
  __shared__ int64_t rows_total[kSumWaves];
  uint32_t I, J;
  tile_of(blockIdx.x, I, J);
  const uint32_t lane = threadIdx.x & (kWave - 1), w = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const uint32_t c0 = J * kTileC, r0 = I * kTile, c = c0 + 2 * lane, r_first = r0 + w * kSumRows;
  int64_t col[2];
  int64_t run;
  if (c0 + kTileC - 1 <= r0 && r0 + kTile <= n)
    run = quarter_tile_sums<VEC, true>(attn, n, ld, r_first, c, lane, col);
  else
    run = quarter_tile_sums<VEC, false>(attn, n, ld, r_first, c, lane, col);
  colpart[w][lane][0] = col[0], colpart[w][lane][1] = col[1];
  if (lane == kSumRows - 1) rows_total[w] = run;
  __syncthreads();
  int64_t rows_before = 0;
  for (uint32_t q = 0; q < w; ++q) rows_before += rows_total[q];
  if (lane < kSumRows) rowrun[(uint64_t)J * n_pad_r + r_first + lane] = rows_before + run;
  if (w == kSumWaves - 1) {
    if (lane == kSumRows - 1) tilesum[(uint64_t)I * n_j + J] = rows_before + run;
  } else if (w == 0) {
    int64_t s0 = 0, s1 = 0;
#pragma unroll
    for (uint32_t q = 0; q < kSumWaves; ++q) s0 += colpart[q][lane][0], s1 += colpart[q][lane][1];
    colsum[(uint64_t)I * n_pad_c + c] = s0;
    colsum[(uint64_t)I * n_pad_c + c + 1] = s1;
  }
}

// With the sensitivity mask known, the table is needed only where a substring search can look: in the
// rows of a coarse segment [a, b], the columns from a - 1 on (and the diagonal, for every row).  The search
// stages whole 64-column blocks, so it reads columns down to a - 64.  For tile row I, with a the smallest
// segment start over its non-sensitive rows, that is the tile columns from (a - 64) / 128 on (none but the one
// that holds the rows' diagonal entries, I / 2, if all its rows are sensitive).  list_tiles (one workgroup)
// finds a per tile row -- its first non-sensitive row and its last sensitive one, a running maximum over the
// latter -- and writes the list of the tiles to build, tile rows ascending: tile_list[t] = pack_tile(I, J) for
// t < *n_listed.  It runs as one workgroup of the carry kernel below.
constexpr uint32_t kMaxTileRows = 4096;  // 2^18 rows / 64; larger requests get the whole table
constexpr uint32_t kListedGrid = 2048;   // workgroups that share out a tile list
__device__ __forceinline__ uint32_t pack_tile(uint32_t I, uint32_t J) { return (I << 12) | J; }  // I < 4096, J <= I / 2
__device__ __forceinline__ void unpack_tile(uint32_t t, uint32_t &I, uint32_t &J) { I = t >> 12, J = t & 0xFFFu; }

// In place over LDS: v[i] <- v[0] (+) ... (+) v[i] for i < count, a chunk of blockDim.x entries at a time.
template <typename Combine>
__device__ __forceinline__ void block_inclusive_scan(uint32_t *v, uint32_t count, uint32_t identity, uint32_t *carry,
                                                     Combine combine) {
  if (threadIdx.x == 0) *carry = identity;
  __syncthreads();
  for (uint32_t base = 0; base < count; base += blockDim.x) {
    const uint32_t i = base + threadIdx.x;
    const uint32_t width = count - base < blockDim.x ? count - base : blockDim.x;
    for (uint32_t step = 1; step < width; step <<= 1) {
      uint32_t other = identity;
      if (i < count && threadIdx.x >= step) other = v[i - step];
      __syncthreads();
      if (i < count) v[i] = combine(other, v[i]);
      __syncthreads();
    }
    if (i < count) v[i] = combine(*carry, v[i]);
    __syncthreads();
    if (threadIdx.x == 0) *carry = v[base + width - 1];
    __syncthreads();
  }
}

constexpr uint32_t kCarryThreads = 1024;  // workgroup of the carry kernel: 16 wavefronts
constexpr uint32_t kCarrySlices = kCarryThreads / kWave;
__device__ __forceinline__ void list_tiles(const uint8_t *__restrict__ mask, uint32_t n, uint32_t n_i,
                                           uint32_t *__restrict__ tile_list, uint32_t *__restrict__ n_listed) {
  __shared__ uint32_t first[kMaxTileRows];  // the first non-sensitive row of tile row I (kNone: none); later: its first tile column
  __shared__ uint32_t last[kMaxTileRows];   // 1 + the last sensitive row at or before the end of tile row I (0: none)
  __shared__ uint32_t upto[kMaxTileRows];   // tiles listed for the tile rows 0 .. I
  __shared__ uint32_t carry;
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
  block_inclusive_scan(last, n_i, 0u, &carry, [](uint32_t x, uint32_t y) { return x > y ? x : y; });
  uint32_t a_mine[kMaxTileRows / kCarryThreads];
#pragma unroll
  for (uint32_t k = 0; k < kMaxTileRows / kCarryThreads; ++k) {
    const uint32_t I = k * kCarryThreads + threadIdx.x;
    uint32_t a = I < n_i ? first[I] : kNone;
    // a segment that starts inside the tile row starts at its first non-sensitive row (the rows before it are
    // sensitive); one that reaches in from above starts right after the last sensitive row before the tile row
    if (a != kNone && a == I * kTile) a = I ? last[I - 1] : 0;
    a_mine[k] = a;
  }
  __syncthreads();  // first[] and last[] have been read
#pragma unroll
  for (uint32_t k = 0; k < kMaxTileRows / kCarryThreads; ++k) {
    const uint32_t I = k * kCarryThreads + threadIdx.x;
    if (I >= n_i) continue;
    const uint32_t a = a_mine[k], j_diag = I / 2;
    uint32_t j_first = j_diag;
    if (a != kNone) {
      const uint32_t j = a >= kTile ? (a - kTile) / kTileC : 0;
      j_first = j < j_diag ? j : j_diag;
    }
    first[I] = j_first;
    upto[I] = j_diag - j_first + 1;
  }
  __syncthreads();
  block_inclusive_scan(upto, n_i, 0u, &carry, [](uint32_t x, uint32_t y) { return x + y; });
  for (uint32_t I = threadIdx.x; I < n_i; I += blockDim.x) {
    uint32_t t = I ? upto[I - 1] : 0;
    for (uint32_t J = first[I]; J <= I / 2; ++J) tile_list[t++] = pack_tile(I, J);
  }
  if (threadIdx.x == 0) *n_listed = upto[n_i - 1];
}

// The carries between tiles, in place, for the three arrays (blockIdx.y = 0, 1, 2):
//   a[k][x] <- sum of a[k'][x] over the k' < k that belong to tiles on or below the diagonal, for the k that do.
//   0: colsum[I][c], tile (I, c / 128): I >= 2 (c / 128)      1: rowrun[J][r], tile (r / 64, J): J <= (r / 64) / 2
//   2: tilesum[I][J]: I >= 2 J
// A workgroup takes 64 neighbouring x; its 16 wavefronts take a sixteenth of the k each (the walk down a column is
// latency, not bandwidth): they add their slice up, exchange the sums, and write the prefixes of their slice --
// from registers when the slice fits one batch of loads, else reading it again.
// blockIdx.y = 3 (one workgroup, only with a mask): the list of the tiles to build, which needs nothing from
// the sums and so costs no launch of its own.
__global__ __launch_bounds__(kCarryThreads) void sat_carry_kernel(int64_t *colsum, uint32_t n_i, uint32_t n_pad_c,
                                                                  int64_t *rowrun, uint32_t n_j, uint32_t n_pad_r,
                                                                  int64_t *tilesum, const uint8_t *__restrict__ mask,
                                                                  uint32_t n, uint32_t *__restrict__ tile_list,
                                                                  uint32_t *__restrict__ n_listed) {
  const uint32_t which = blockIdx.y;
  if (which == 3) {
    if (blockIdx.x == 0) list_tiles(mask, n, n_i, tile_list, n_listed);
    return;
  }
  __shared__ int64_t slice_sum[kCarrySlices][kWave];
  int64_t *a = which == 0 ? colsum : which == 1 ? rowrun : tilesum;
  const uint32_t width = which == 0 ? n_pad_c : which == 1 ? n_pad_r : n_j;
  const uint32_t lane = threadIdx.x & (kWave - 1), slice = threadIdx.x / kWave;
  const uint32_t x = blockIdx.x * kWave + lane;
  if (blockIdx.x * kWave >= width) return;  // the same for the whole workgroup
  uint32_t k_from = 0, k_to = 0;            // [k_from, k_to); empty for x beyond the array
  if (x < width) {
    if (which == 0) k_from = 2 * (x / kTileC), k_to = n_i;
    else if (which == 1) k_from = 0, k_to = (x / kTile) / 2 + 1;
    else k_from = 2 * x, k_to = n_i;
    if (k_from > k_to) k_from = k_to;
  }
  const uint32_t share = (k_to - k_from + kCarrySlices - 1) / kCarrySlices;
  const uint32_t k0 = k_from + slice * share < k_to ? k_from + slice * share : k_to;
  const uint32_t k1 = k0 + share < k_to ? k0 + share : k_to;
  constexpr int kBatch = 16;  // independent loads in flight
  int64_t v[kBatch];
#pragma unroll
  for (int u = 0; u < kBatch; ++u) v[u] = 0;
  int64_t total = 0;
  for (uint32_t k = k0; k < k1; k += kBatch) {
#pragma unroll
    for (int u = 0; u < kBatch; ++u) v[u] = k + u < k1 ? a[(uint64_t)(k + u) * width + x] : 0;
#pragma unroll
    for (int u = 0; u < kBatch; ++u) total += v[u];
  }
  slice_sum[slice][lane] = total;
  __syncthreads();
  int64_t run = 0;
  for (uint32_t q = 0; q < slice; ++q) run += slice_sum[q][lane];
  if (k1 - k0 <= (uint32_t)kBatch) {  // v[] still holds the whole slice
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      if (k0 + u < k1) a[(uint64_t)(k0 + u) * width + x] = run;
      run += v[u];
    }
    return;
  }
  for (uint32_t k = k0; k < k1; k += kBatch) {
#pragma unroll
    for (int u = 0; u < kBatch; ++u) v[u] = k + u < k1 ? a[(uint64_t)(k + u) * width + x] : 0;
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      if (k + u < k1) a[(uint64_t)(k + u) * width + x] = run;
      run += v[u];
    }
  }
}

// A workgroup of four wavefronts builds one tile of the table; wavefront w takes the rows 16w .. 16w + 15, every
// lane two adjacent columns.  All 16 rows of a wavefront are requested at once and stay in registers: first their
// column sums go to the wavefronts below through LDS (what the tile's earlier rows add to every later row), then per
// row: prefix over the lane's two columns, one wave scan across the lanes, running sum down the rows, + what lies
// above the tile in its columns + what lies left of it in rows <= i (left of it in the tile's own rows + the totals
// of the tiles above those).  LISTED: the workgroups share out the tiles of tile_list (the part of the table a search
// can read); otherwise workgroup b takes tile b of the triangle.
constexpr uint32_t kApplyWaves = 4, kApplyRows = kTile / kApplyWaves;
template <bool VEC_LD, bool VEC_ST, bool INTERIOR>
__device__ __forceinline__ void tile_apply(const float *__restrict__ attn, uint32_t n, uint64_t ld, uint32_t r0,
                                           uint32_t c, uint32_t lane, uint32_t w, const int64_t above_pref[2],
                                           int64_t left_row, int64_t (*colpart)[kWave][2], int64_t *__restrict__ T) {
  const uint32_t c_in_tile = 2 * lane, r_first = r0 + w * kApplyRows;
  const float *p = attn + (uint64_t)r_first * ld + (c - c_in_tile);  // the first weight and table entry of the
  int64_t *t = T + (uint64_t)r_first * n + (c - c_in_tile);          // wavefront's rows: the same in every lane
  f32x2 x[kApplyRows];
#pragma unroll
  for (uint32_t u = 0; u < kApplyRows; ++u)
    x[u] = load_x2<VEC_LD, INTERIOR>(p + (uint64_t)u * ld + c_in_tile, n, r_first + u, c);
  // weights above the diagonal or outside the matrix were read as 0; values out of range count as 0 too
  int32_t hi_pos = (int32_t)0x80000000;
  uint32_t hi_neg = 0;
#pragma unroll
  for (uint32_t u = 0; u < kApplyRows; ++u) {
    const uint32_t bx = __float_as_uint(x[u].x), by = __float_as_uint(x[u].y);
    hi_pos = max(hi_pos, max((int32_t)bx, (int32_t)by));
    hi_neg = max(hi_neg, max(bx, by));
  }
  if (__builtin_expect(__ballot(hi_pos > kMaxPosBits || hi_neg > kMaxNegBits) != 0, 0)) {
#pragma unroll
    for (uint32_t u = 0; u < kApplyRows; ++u) {
      x[u].x = fabsf(x[u].x) <= 262144.0f ? x[u].x : 0.0f;
      x[u].y = fabsf(x[u].y) <= 262144.0f ? x[u].y : 0.0f;
    }
  }
  uint64_t s0 = 0, s1 = 0;
#pragma unroll
  for (uint32_t u = 0; u < kApplyRows; ++u) s0 += quantise_biased(x[u].x), s1 += quantise_biased(x[u].y);
  colpart[w][lane][0] = (int64_t)(s0 - (uint64_t)kApplyRows * kMagicBits);
  colpart[w][lane][1] = (int64_t)(s1 - (uint64_t)kApplyRows * kMagicBits);
  __syncthreads();
  int64_t acc[2] = {0, 0};  // the tile's rows before this one, the tile's columns up to each of this lane's
  for (uint32_t q = 0; q < w; ++q) acc[0] += colpart[q][lane][0], acc[1] += colpart[q][lane][1];
  acc[1] += acc[0];
  {
    const int64_t before = wave_inclusive_sum(acc[1]) - acc[1];
    acc[0] += before, acc[1] += before;
  }
#pragma unroll
  for (uint32_t u = 0; u < kApplyRows; ++u) {
    const uint32_t k = w * kApplyRows + u, r = r0 + k;  // the same for the whole wavefront
    int64_t q[2] = {(int64_t)(quantise_biased(x[u].x) - kMagicBits), (int64_t)(quantise_biased(x[u].y) - kMagicBits)};
    q[1] += q[0];
    const int64_t before = wave_inclusive_sum(q[1]) - q[1];
    const int64_t lv = readlane_i64(left_row, k);
    acc[0] += before + q[0], acc[1] += before + q[1];
    const int64_t out0 = acc[0] + above_pref[0] + lv, out1 = acc[1] + above_pref[1] + lv;
    if (INTERIOR || r < n) {
      int64_t *o = t + (uint64_t)u * n + c_in_tile;
      if (VEC_ST && (INTERIOR || c + 1 < n)) {  // the wavefront writes 1 KiB in one piece
        __builtin_nontemporal_store(i64x2{out0, out1}, reinterpret_cast<i64x2 *>(o));
      } else {
        if (c < n) o[0] = out0;
        if (c + 1 < n) o[1] = out1;
      }
    }
  }
}

template <bool VEC_LD, bool VEC_ST, bool LISTED>
__global__ __launch_bounds__(kApplyWaves *kWave) void sat_apply_kernel(
    const float *__restrict__ attn, uint32_t n, uint64_t ld, uint32_t n_pad_c, uint32_t n_pad_r, uint32_t n_j,
    const int64_t *__restrict__ above, const int64_t *__restrict__ left, const int64_t *__restrict__ tiles_above,
    const uint32_t *__restrict__ tile_list, const uint32_t *__restrict__ n_listed, int64_t *__restrict__ T) {
  __shared__ int64_t colpart[2][kApplyWaves][kWave][2];  // two sets: a tile's sums are still read while the next tile's are written
  const uint32_t lane = threadIdx.x & (kWave - 1), w = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const uint32_t n_mine = LISTED ? *n_listed : gridDim.x;
  uint32_t turn = 0;
  for (uint32_t t = blockIdx.x; t < n_mine; t += gridDim.x, turn ^= 1) {  // (one turn unless LISTED)
    uint32_t I, J;
    if (LISTED) {
      unpack_tile(tile_list[t], I, J);
      I = __builtin_amdgcn_readfirstlane(I), J = __builtin_amdgcn_readfirstlane(J);
    } else {
      tile_of(t, I, J);
    }
    const uint32_t c0 = J * kTileC, r0 = I * kTile, c = c0 + 2 * lane;
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
      for (uint32_t j = lane; j < J; j += kWave) part += tiles_above[(uint64_t)I * n_j + j];
      left_row += readlane_i64(wave_inclusive_sum(part), kWave - 1);
    }
    if (c0 + kTileC - 1 <= r0 && r0 + kTile <= n)
      tile_apply<VEC_LD, VEC_ST, true>(attn, n, ld, r0, c, lane, w, above_pref, left_row, colpart[turn], T);
    else
      tile_apply<VEC_LD, VEC_ST, false>(attn, n, ld, r0, c, lane, w, above_pref, left_row, colpart[turn], T);
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
  const uint64_t listed = n_i <= kMaxTileRows ? tiles_before_row((uint32_t)n_i) + 1 : 0;  // tile list and its length
  return (size_t)((cols + rows + n_i * n_j) * 8 + 4 * listed + 320ull * n + 33 * 256);
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
  const uint32_t n_tiles = (uint32_t)tiles_before_row(n_i);  // on or below the diagonal; <= 2^26
  uint32_t *tile_list = mask ? sc.take<uint32_t>(n_tiles) : nullptr;
  uint32_t *n_listed = mask ? sc.take<uint32_t>(1) : nullptr;
  if (!colsum || !rowsum || !tilesum || (mask && (!tile_list || !n_listed))) return CP_ERR_SCRATCH;
  const bool vec_ld = ld % 2 == 0 && aligned(attn, 8);  // every (row, column pair) starts on 8 bytes
  const bool vec_st = n % 2 == 0 && aligned(T, 16);
  if (vec_ld)
    sat_tile_sums_kernel<true><<<n_tiles, kSumWaves * kWave, 0, stream>>>(attn, n, ld, n_pad_c, n_pad_r, n_j, colsum, rowsum, tilesum);
  else
    sat_tile_sums_kernel<false><<<n_tiles, kSumWaves * kWave, 0, stream>>>(attn, n, ld, n_pad_c, n_pad_r, n_j, colsum, rowsum, tilesum);
  // above the tile (column sums over the tile rows before), left of it in its own rows (running row sums
  // over the tile columns before), and the totals of the tiles above each tile
  const uint32_t widest = n_pad_c > n_pad_r ? n_pad_c : n_pad_r;
  sat_carry_kernel<<<dim3(div_up(widest, kWave), mask ? 4 : 3), kCarryThreads, 0, stream>>>(
      colsum, n_i, n_pad_c, rowsum, n_j, n_pad_r, tilesum, mask, n, tile_list, n_listed);
  // with a tile list its length is known on the device only: a fixed number of workgroups shares the tiles out
  const uint32_t grid = mask ? (n_tiles < kListedGrid ? n_tiles : kListedGrid) : n_tiles;
  auto apply = [&](auto vl, auto vs) {
    if (mask)
      sat_apply_kernel<decltype(vl)::value, decltype(vs)::value, true><<<grid, kApplyWaves * kWave, 0, stream>>>(
          attn, n, ld, n_pad_c, n_pad_r, n_j, colsum, rowsum, tilesum, tile_list, n_listed, T);
    else
      sat_apply_kernel<decltype(vl)::value, decltype(vs)::value, false><<<grid, kApplyWaves * kWave, 0, stream>>>(
          attn, n, ld, n_pad_c, n_pad_r, n_j, colsum, rowsum, tilesum, nullptr, nullptr, T);
  };
  if (vec_ld && vec_st) apply(std::true_type{}, std::true_type{});
  else if (vec_ld) apply(std::true_type{}, std::false_type{});
  else if (vec_st) apply(std::false_type{}, std::true_type{});
  else apply(std::false_type{}, std::false_type{});
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

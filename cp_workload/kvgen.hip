// Device side of the synthetic KV value generator: fill and verify kernels.
//
// Input generation and test tooling only.  The definition of a value is stated
// in kvgen.py; this file repeats it for the GPU so that tens of GiB of pool and
// request buffers can be filled and checked in place.  None of the method's
// arithmetic is here and the GPU library does not include this file.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

constexpr uint64_t kC1 = 0x9E3779B97F4A7C15ull;
constexpr uint64_t kC2 = 0xD1B54A32D192ED03ull;
constexpr uint64_t kM = 0xD6E8FEB86659FD93ull;
constexpr uint64_t kUidNone = 0xFFFFFFFFFFFFFFFFull;
constexpr uint32_t kPoison16 = 0xC0DEu;
constexpr uint32_t kScaleBits = 0x3BDDB47Bu;  // float nearest to 1 / 147.8

struct GenLayout {
  uint32_t n_layers, row_elems;
  uint64_t tok_stride, layer_stride, kv_stride;
};

__device__ __forceinline__ uint32_t elem_bits(uint32_t w) {
  int s = (int)((w & 0xFF) + ((w >> 8) & 0xFF) + ((w >> 16) & 0xFF) + (w >> 24));
  float x = (float)(s - 510) * __uint_as_float(kScaleBits);
  uint32_t u = __float_as_uint(x);
  u = u + 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}

// Two bf16 values (elements 2*pair and 2*pair+1) packed low/high in 32 bits.
__device__ __forceinline__ uint32_t pair_bits(uint64_t seed, uint64_t row_id, uint32_t pair) {
  uint64_t z = seed + row_id * kC1 + (uint64_t)pair * kC2;
  z ^= z >> 32;
  z *= kM;
  z ^= z >> 32;
  z *= kM;
  z ^= z >> 32;
  return elem_bits((uint32_t)z) | (elem_bits((uint32_t)(z >> 32)) << 16);
}

// One block per row, rows taken grid-stride.  Thread handles pairs tid, tid+B, ..
__global__ void fill_kernel(uint8_t *base, GenLayout lay, const uint64_t *uid, uint64_t uid_base,
                            uint32_t n_tok, uint64_t seed) {
  const uint64_t n_rows = (uint64_t)n_tok * lay.n_layers * 2;
  const uint32_t n_pairs = lay.row_elems / 2;
  for (uint64_t r = blockIdx.x; r < n_rows; r += gridDim.x) {
    uint32_t kv = (uint32_t)(r & 1);
    uint64_t tl = r >> 1;
    uint32_t l = (uint32_t)(tl % lay.n_layers);
    uint32_t t = (uint32_t)(tl / lay.n_layers);
    uint64_t u = uid ? uid[t] : uid_base + t;
    uint32_t *row = (uint32_t *)(base + t * lay.tok_stride + l * lay.layer_stride + kv * lay.kv_stride);
    uint64_t row_id = (u * lay.n_layers + l) * 2 + kv;
    for (uint32_t p = threadIdx.x; p < n_pairs; p += blockDim.x)
      row[p] = (u == kUidNone) ? (kPoison16 | (kPoison16 << 16)) : pair_bits(seed, row_id, p);
  }
}

__global__ void verify_kernel(const uint8_t *base, GenLayout lay, const uint64_t *uid,
                              const uint8_t *skip_k, uint32_t n_tok, uint64_t seed,
                              unsigned long long *n_bad) {
  const uint64_t n_rows = (uint64_t)n_tok * lay.n_layers * 2;
  const uint32_t n_pairs = lay.row_elems / 2;
  uint32_t bad = 0;
  for (uint64_t r = blockIdx.x; r < n_rows; r += gridDim.x) {
    uint32_t kv = (uint32_t)(r & 1);
    uint64_t tl = r >> 1;
    uint32_t l = (uint32_t)(tl % lay.n_layers);
    uint32_t t = (uint32_t)(tl / lay.n_layers);
    if (kv == 0 && skip_k && skip_k[t]) continue;
    uint64_t u = uid[t];
    const uint32_t *row =
        (const uint32_t *)(base + t * lay.tok_stride + l * lay.layer_stride + kv * lay.kv_stride);
    uint64_t row_id = (u * lay.n_layers + l) * 2 + kv;
    for (uint32_t p = threadIdx.x; p < n_pairs; p += blockDim.x) {
      uint32_t want = (u == kUidNone) ? (kPoison16 | (kPoison16 << 16)) : pair_bits(seed, row_id, p);
      uint32_t got = row[p];
      bad += ((got & 0xFFFFu) != (want & 0xFFFFu)) + ((got >> 16) != (want >> 16));
    }
  }
  if (bad) atomicAdd(n_bad, (unsigned long long)bad);
}

// Plain streaming kernels over a contiguous buffer, 16-byte accesses: what this GPU reaches for a pure
// read, a pure write and a copy.  Benchmarks quote them beside the row mover's rate, and their known
// byte counts calibrate the profiler's HBM counters.  Workgroup w takes the chunks w, w + grid, ...
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int U>
__global__ __launch_bounds__(256) void stream_read_kernel(const uint8_t *__restrict__ a, uint64_t bytes, uint64_t chunk,
                                                          uint32_t *sink) {
  const uint64_t n_chunks = bytes / chunk;
  uint32_t acc = 0;
  for (uint64_t ch = blockIdx.x; ch < n_chunks; ch += gridDim.x) {
    const uint8_t *s = a + ch * chunk;
    for (uint64_t i = (uint64_t)threadIdx.x * 16; i < chunk; i += 256ull * 16 * U) {
      u32x4 v[U];
#pragma unroll
      for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load((const u32x4 *)(s + i + (uint64_t)u * 256 * 16));
#pragma unroll
      for (int u = 0; u < U; ++u) acc += v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
    }
  }
  if (acc == 0x12345678u) sink[0] = acc;  // keeps the loads alive; practically never true
}

// Writing and copying in pieces of 256 * U sixteen-byte vectors (4 KiB for U = 1): workgroup b takes pieces b,
// b + grid, ...; launched with one workgroup per piece, every thread makes one access (per direction) and leaves.
template <int U>
__global__ __launch_bounds__(256) void stream_write_kernel(uint8_t *__restrict__ b, uint64_t n_pieces) {
  const u32x4 v = {0xC0DEC0DEu, 0xC0DEC0DEu, 0xC0DEC0DEu, 0xC0DEC0DEu};
  for (uint64_t p = blockIdx.x; p < n_pieces; p += gridDim.x) {
    uint8_t *d = b + p * (256ull * 16 * U) + (uint64_t)threadIdx.x * 16;
#pragma unroll
    for (int u = 0; u < U; ++u) *(u32x4 *)(d + (uint64_t)u * 256 * 16) = v;
  }
}

template <int U>
__global__ __launch_bounds__(256) void stream_copy_kernel(const uint8_t *__restrict__ a, uint8_t *__restrict__ b,
                                                          uint64_t n_pieces) {
  for (uint64_t p = blockIdx.x; p < n_pieces; p += gridDim.x) {
    const uint64_t at = p * (256ull * 16 * U) + (uint64_t)threadIdx.x * 16;
    u32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = *(const u32x4 *)(a + at + (uint64_t)u * 256 * 16);
#pragma unroll
    for (int u = 0; u < U; ++u) __builtin_nontemporal_store(v[u], (u32x4 *)(b + at + (uint64_t)u * 256 * 16));
  }
}

uint32_t grid_for(uint64_t n_rows) {
  uint64_t g = n_rows < 65536 ? n_rows : 65536;
  return (uint32_t)(g ? g : 1);
}

}  // namespace

extern "C" int kvgen_fill(hipStream_t stream, void *base, GenLayout lay, const uint64_t *uid,
                          uint64_t uid_base, uint32_t n_tok, uint64_t seed) {
  if (n_tok == 0) return 0;
  uint64_t n_rows = (uint64_t)n_tok * lay.n_layers * 2;
  fill_kernel<<<grid_for(n_rows), 256, 0, stream>>>((uint8_t *)base, lay, uid, uid_base, n_tok, seed);
  return (int)hipGetLastError();
}

extern "C" int kvgen_verify(hipStream_t stream, const void *base, GenLayout lay, const uint64_t *uid,
                            const uint8_t *skip_k, uint32_t n_tok, uint64_t seed, uint64_t *n_bad) {
  if (n_tok == 0) return 0;
  uint64_t n_rows = (uint64_t)n_tok * lay.n_layers * 2;
  verify_kernel<<<grid_for(n_rows), 256, 0, stream>>>((const uint8_t *)base, lay, uid, skip_k, n_tok, seed,
                                                      (unsigned long long *)n_bad);
  return (int)hipGetLastError();
}

// mode 0: read `bytes` of a; 1: write `bytes` of b (with the poison pattern); 2: copy a -> b.  bytes must be a
// multiple of 128 KiB; a and b 16-byte aligned, not overlapping.  Shapes chosen from sweeps on MI355X: reading
// is fastest from a thousand workgroups that each walk 128 KiB pieces with 8 loads in flight (7.1 TB/s; one
// 16-byte load per thread reaches 6.8); writing and copying are fastest the other way round, with one workgroup
// per 4 KiB and one 16-byte access per thread, handed out in address order, so that at any moment the chip
// works on one window of a few MiB (6.9 and 6.3 TB/s; with 65,536 workgroups striding over the buffer 5.5 and
// 5.5, and slower the more each workgroup moves).
extern "C" int kvgen_stream(hipStream_t stream, int mode, const void *a, void *b, uint64_t bytes, uint32_t *sink) {
  if (bytes == 0 || bytes % 131072) return (int)hipErrorInvalidValue;
  const uint64_t pieces = bytes / 4096;
  const uint32_t one_each = (uint32_t)(pieces < 0x7FFFFFFFull ? pieces : 0x7FFFFFFFull);  // (more pieces: the kernels loop)
  if (mode == 0) stream_read_kernel<8><<<1024, 256, 0, stream>>>((const uint8_t *)a, bytes, 131072, sink);
  else if (mode == 1) stream_write_kernel<1><<<one_each, 256, 0, stream>>>((uint8_t *)b, pieces);
  else if (mode == 2) stream_copy_kernel<1><<<one_each, 256, 0, stream>>>((const uint8_t *)a, (uint8_t *)b, pieces);
  else return (int)hipErrorInvalidValue;
  return (int)hipGetLastError();
}

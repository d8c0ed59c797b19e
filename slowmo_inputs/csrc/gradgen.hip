// Device side of the seeded input generator (test and benchmark inputs; not
// part of the optimizer library).  Evaluates the same counter-based function
// as generator.py:
//   key = mix64(mix64(seed + G*(worker+1)) ^ (S*(step+1)))
//   w_l = mix64(key + G*(3*index + l + 1)),  l = 0..2
//   n   = (sum of the twelve 16-bit fields of w_0..w_2 - 393210) / 65536
//   out = scale * n     (one fp32 product; bf16: round to nearest even)
// Integer arithmetic only up to the final exact conversion, so host and
// device produce identical bits.
#include <hip/hip_runtime.h>

#include <cstdint>

namespace {

constexpr uint64_t kG = 0x9E3779B97F4A7C15ull;
constexpr uint64_t kS = 0xD1342543DE82EF95ull;

__host__ __device__ inline uint64_t mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

__device__ inline uint32_t fields16(uint64_t w) {
  return static_cast<uint32_t>(w & 0xFFFF) + static_cast<uint32_t>((w >> 16) & 0xFFFF) +
         static_cast<uint32_t>((w >> 32) & 0xFFFF) + static_cast<uint32_t>(w >> 48);
}

__device__ inline float unit_normal(uint64_t key, uint64_t index) {
  uint64_t c = 3 * index;
  uint32_t s = fields16(mix64(key + kG * (c + 1))) + fields16(mix64(key + kG * (c + 2))) +
               fields16(mix64(key + kG * (c + 3)));
  return static_cast<float>(static_cast<int32_t>(s) - 393210) * (1.0f / 65536.0f);
}

__device__ inline uint16_t bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  return static_cast<uint16_t>((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

template <bool BF16>
__global__ __launch_bounds__(256) void k_fill(void *out, int64_t n, int64_t first_index,
                                              uint64_t seed, int32_t worker0,
                                              int64_t worker_stride, int64_t step, float scale) {
  const int32_t w = blockIdx.y;
  const uint64_t key =
      mix64(mix64(seed + kG * static_cast<uint64_t>(worker0 + w + 1)) ^
            (kS * static_cast<uint64_t>(step + 1)));
  const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
  for (int64_t j = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; j < n; j += stride) {
    float v = scale * unit_normal(key, static_cast<uint64_t>(first_index + j));
    if (BF16) {
      static_cast<uint16_t *>(out)[w * worker_stride + j] = bf16_rne(v);
    } else {
      static_cast<float *>(out)[w * worker_stride + j] = v;
    }
  }
}

// Plain copy of n 16-byte vectors: a kernel of known traffic (16 n bytes
// read, 16 n bytes written) against which hardware counters are scaled.
__global__ __launch_bounds__(256) void k_calib_copy(const float4 *__restrict__ src,
                                                    float4 *__restrict__ dst, int64_t n) {
  int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src[i];
}

}  // namespace

// Copies `bytes` (a multiple of 16, both pointers 16-byte aligned) from src to
// dst on the device with k_calib_copy.  Returns 0 or a hipError_t value.
extern "C" int slowmo_inputs_calib_copy(const void *src, void *dst, int64_t bytes, void *stream) {
  if (bytes <= 0) return 0;
  if (!src || !dst || bytes % 16) return static_cast<int>(hipErrorInvalidValue);
  const int64_t n = bytes / 16;
  hipLaunchKernelGGL(k_calib_copy, dim3(static_cast<unsigned>((n + 255) / 256)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), static_cast<const float4 *>(src),
                     static_cast<float4 *>(dst), n);
  return static_cast<int>(hipGetLastError());
}

// out[w * worker_stride + j] = scale * n(seed, worker0 + w, step, first_index + j)
// for w in [0, n_workers), j in [0, n).  `out` is a device pointer of fp32
// (bf16 = 0) or bf16 (bf16 = 1) elements.  Returns 0, or a hipError_t value.
extern "C" int slowmo_inputs_fill(void *out, int64_t n, int64_t first_index, uint64_t seed,
                                  int32_t worker0, int32_t n_workers, int64_t worker_stride,
                                  int64_t step, float scale, int32_t bf16, void *stream) {
  if (n <= 0 || n_workers <= 0) return 0;
  if (!out || n_workers > 65535) return static_cast<int>(hipErrorInvalidValue);
  int64_t want = (n + 255) / 256;
  dim3 grid(static_cast<unsigned>(want < 65536 ? want : 65536), static_cast<unsigned>(n_workers));
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (bf16) {
    hipLaunchKernelGGL(k_fill<true>, grid, dim3(256), 0, s, out, n, first_index, seed, worker0,
                       worker_stride, step, scale);
  } else {
    hipLaunchKernelGGL(k_fill<false>, grid, dim3(256), 0, s, out, n, first_index, seed, worker0,
                       worker_stride, step, scale);
  }
  return static_cast<int>(hipGetLastError());
}

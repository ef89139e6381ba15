// Device twin of the counter-based input generator (gfx950).
//
// Seeded INPUT generator only: it fills a device buffer with the synthetic
// vector that stands in for a learner's gradient (or the initial weights).
// None of the parameter server's arithmetic lives here.  The integer recipe is
// the one documented in synth/gradgen.py; every step is exact integer work
// followed by one exact int->float conversion and ONE binary32 multiply, so the
// bits equal the numpy implementation's.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

constexpr uint64_t kGolden = 0x9E3779B97F4A7C15ull;
constexpr uint64_t kSecond = 0xD1B54A32D192ED03ull;
constexpr uint64_t kTail = 0x8CB92BA72F3D8DD7ull;
constexpr int kIhMean = 4 * 65535;

__device__ __forceinline__ uint64_t mix(uint64_t x) {
  x ^= x >> 30;
  x *= 0xBF58476D1CE4E5B9ull;
  x ^= x >> 27;
  x *= 0x94D049BB133111EBull;
  x ^= x >> 31;
  return x;
}

__device__ __forceinline__ uint32_t lanes(uint64_t h) {
  return (uint32_t)(h & 0xFFFF) + (uint32_t)((h >> 16) & 0xFFFF) + (uint32_t)((h >> 32) & 0xFFFF) +
         (uint32_t)(h >> 48);
}

__device__ __forceinline__ float value_at(uint64_t key, uint64_t k, float scale, float scale_tail,
                                          uint32_t tail_per) {
  const uint64_t u = key + k * kGolden;
  const int s = (int)(lanes(mix(u)) + lanes(mix(u ^ kSecond))) - kIhMean;
  float sc = scale;
  if (tail_per) {
    const uint64_t t = mix(u + kTail);
    if ((((t >> 32) * (uint64_t)tail_per) >> 32) == 0) sc = scale_tail;
  }
  return __fmul_rn((float)s, sc);
}

__global__ __launch_bounds__(256) void synth_fill_kernel(float* __restrict__ dst, uint64_t n, uint64_t key,
                                                         float scale, float scale_tail, uint32_t tail_per) {
  const uint64_t i4 = ((uint64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
  if (i4 + 4 <= n) {
    float4 v;
    v.x = value_at(key, i4 + 0, scale, scale_tail, tail_per);
    v.y = value_at(key, i4 + 1, scale, scale_tail, tail_per);
    v.z = value_at(key, i4 + 2, scale, scale_tail, tail_per);
    v.w = value_at(key, i4 + 3, scale, scale_tail, tail_per);
    *reinterpret_cast<float4*>(dst + i4) = v;
  } else {
    for (uint64_t k = i4; k < n; ++k) dst[k] = value_at(key, k, scale, scale_tail, tail_per);
  }
}

}  // namespace

// dst: device pointer to n floats, 16-byte aligned; stream: hipStream_t (borrowed).
// Returns 0 or the hipError_t of the launch.
extern "C" int synth_fill(float* dst, uint64_t n, uint64_t key, float scale, float scale_tail, uint32_t tail_per,
                          void* stream) {
  if (n == 0) return 0;
  if (!dst || (reinterpret_cast<uintptr_t>(dst) & 15u)) return (int)hipErrorInvalidValue;
  const uint64_t n4 = (n + 3) / 4;
  const uint64_t blocks = (n4 + 255) / 256;
  if (blocks > 0x7FFFFFFFull) return (int)hipErrorInvalidValue;
  hipLaunchKernelGGL(synth_fill_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, dst, n, key, scale,
                     scale_tail, tail_per);
  return (int)hipGetLastError();
}

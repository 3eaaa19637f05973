// Shared device/host helpers for the gfx950 kernels of the speculative-round library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fard {

typedef __bf16 bf16;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int WAVE = 64;

// activation selectors shared by the GEMM epilogues
enum Act { ACT_NONE = 0, ACT_GELU = 1, ACT_SILU = 2 };

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16 x) { return (float)x; }
template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float x) { return (bf16)x; }

// erf by the rational-times-Gaussian approximation of Abramowitz & Stegun 7.1.26 (|error| < 1.5e-7):
// branch-free, unlike the library erff, so epilogues that apply it to 48 accumulators stay straight-line.
__device__ __forceinline__ float erf_as(float x) {
  const float ax = fabsf(x);
  const float t = 1.0f / (1.0f + 0.3275911f * ax);
  const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
  const float y = 1.0f - poly * __expf(-ax * ax);
  return copysignf(y, x);
}
__device__ __forceinline__ float gelu_erf(float x) { return 0.5f * x * (1.0f + erf_as(x * 0.70710678118654752f)); }
__device__ __forceinline__ float silu(float x) { return x / (1.0f + __expf(-x)); }
__device__ __forceinline__ float apply_act(float x, int act) {
  return act == ACT_GELU ? gelu_erf(x) : (act == ACT_SILU ? silu(x) : x);
}

// butterfly reductions over the 64 lanes of a wavefront
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
  return v;
}

// effective row count: host upper bound clipped by an optional device-side count
__device__ __forceinline__ int eff_rows(int m_host, const int* m_dev) {
  if (m_dev == nullptr) return m_host;
  int m = *m_dev;
  return m < m_host ? m : m_host;
}

}  // namespace fard

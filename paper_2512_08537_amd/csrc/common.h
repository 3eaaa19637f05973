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

// Reductions over the 64 lanes of a wavefront without a trip through the LDS crossbar: four data-parallel-primitive
// steps make every row of 16 lanes uniform (neighbour, neighbouring pair, mirrored half row, mirrored row), then the
// four row values are read as scalars.  All 64 lanes must be active.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
constexpr int DPP_SWAP1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int DPP_SWAP2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int DPP_HALF_MIRROR = 0x141; // lane i of a group of 8 reads lane 7 - i
constexpr int DPP_MIRROR = 0x140;      // lane i of a row of 16 reads lane 15 - i
__device__ __forceinline__ float lane_value(float v, int lane) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp_move<DPP_SWAP1>(v);
  v += dpp_move<DPP_SWAP2>(v);
  v += dpp_move<DPP_HALF_MIRROR>(v);
  v += dpp_move<DPP_MIRROR>(v);
  return v;
}
__device__ __forceinline__ float row16_max(float v) {
  v = fmaxf(v, dpp_move<DPP_SWAP1>(v));
  v = fmaxf(v, dpp_move<DPP_SWAP2>(v));
  v = fmaxf(v, dpp_move<DPP_HALF_MIRROR>(v));
  v = fmaxf(v, dpp_move<DPP_MIRROR>(v));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
  v = row16_sum(v);
  return (lane_value(v, 0) + lane_value(v, 16)) + (lane_value(v, 32) + lane_value(v, 48));
}
__device__ __forceinline__ float wave_max(float v) {
  v = row16_max(v);
  return fmaxf(fmaxf(lane_value(v, 0), lane_value(v, 16)), fmaxf(lane_value(v, 32), lane_value(v, 48)));
}
// The same over each half of the wave (lanes 0-31, lanes 32-63): every lane gets its own half's result.
__device__ __forceinline__ float half_sum(float v) {
  v = row16_sum(v);
  const float lo = lane_value(v, 0) + lane_value(v, 16), hi = lane_value(v, 32) + lane_value(v, 48);
  return (threadIdx.x & 32) ? hi : lo;
}
__device__ __forceinline__ float half_max(float v) {
  v = row16_max(v);
  const float lo = fmaxf(lane_value(v, 0), lane_value(v, 16)), hi = fmaxf(lane_value(v, 32), lane_value(v, 48));
  return (threadIdx.x & 32) ? hi : lo;
}
// Exchanges between the halves of the wave (lanes l and l ^ 32) and between neighbouring rows of 16 (l and l ^ 16)
// by one register swap each: after swapping a value with itself, one result holds the lower partner's value in
// both places and the other the upper partner's.
__device__ __forceinline__ float other_half(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_int(v), __float_as_int(v), false, false);
  return __int_as_float((threadIdx.x & 32) ? r[0] : r[1]);
}
__device__ __forceinline__ float xor32_sum(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_int(v), __float_as_int(v), false, false);
  return __int_as_float(r[0]) + __int_as_float(r[1]);
}
__device__ __forceinline__ float xor32_max(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_int(v), __float_as_int(v), false, false);
  return fmaxf(__int_as_float(r[0]), __int_as_float(r[1]));
}
__device__ __forceinline__ float xor16_sum(float v) {
  const auto r = __builtin_amdgcn_permlane16_swap(__float_as_int(v), __float_as_int(v), false, false);
  return __int_as_float(r[0]) + __int_as_float(r[1]);
}

// Tile order of a bf16 activation matrix [rows, K] (K % 32 == 0) that a narrow-tile GEMM reads as its A operand: the
// 16-byte pieces a lane of the 16 x 16 x 32 MFMA takes (8 consecutive k of one row), rows innermost inside a block of
// 16 rows x 32 k, so that a wave's operand load reads 1 KiB of consecutive memory (GemmArgs::a_tiled).  Offset in
// elements of (r, k); 4 or 8 consecutive k starting at a multiple of 4 or 8 stay contiguous.
__device__ __host__ __forceinline__ size_t tile_offset(int r, int k, int K) {
  return ((((size_t)(r >> 4) * (size_t)(K >> 5) + (size_t)(k >> 5)) * 4 + (size_t)((k >> 3) & 3)) * 16 + (size_t)(r & 15)) * 8 + (size_t)(k & 7);
}

// effective row count: host upper bound clipped by an optional device-side count
__device__ __forceinline__ int eff_rows(int m_host, const int* m_dev) {
  if (m_dev == nullptr) return m_host;
  int m = *m_dev;
  return m < m_host ? m : m_host;
}

}  // namespace fard

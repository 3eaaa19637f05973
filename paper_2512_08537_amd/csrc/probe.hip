// Peak probes: what this GPU sustains on the two resources the round's kernels are priced against.
//   - a streaming read of a caller's buffer (16 B per lane per load, grid-stride, nothing written but one word per workgroup)
//   - a register-only loop of bf16 32x32x16 MFMAs (four independent accumulators per wave, no memory traffic)
// Neither is part of the decoding round; the benchmark reports its roofline fractions against these beside the published peaks.
#include <hip/hip_runtime.h>

#include "kernels.h"

namespace fard {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

constexpr int PROBE_THREADS = 256;

__global__ __launch_bounds__(PROBE_THREADS) void probe_read_kernel(const u32x4* __restrict__ buf, long n16, unsigned* __restrict__ sink) {
  const long stride = (long)gridDim.x * PROBE_THREADS;
  long i = (long)blockIdx.x * PROBE_THREADS + threadIdx.x;
  unsigned acc = 0;
  // four loads in flight per lane
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const u32x4 a = __builtin_nontemporal_load(buf + i);
    const u32x4 b = __builtin_nontemporal_load(buf + i + stride);
    const u32x4 c = __builtin_nontemporal_load(buf + i + 2 * stride);
    const u32x4 d = __builtin_nontemporal_load(buf + i + 3 * stride);
    acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
  }
  for (; i < n16; i += stride) {
    const u32x4 a = __builtin_nontemporal_load(buf + i);
    acc ^= a.x ^ a.y ^ a.z ^ a.w;
  }
  // one word per workgroup keeps the loads alive
  for (int off = 32; off > 0; off >>= 1) acc ^= __shfl_xor(acc, off);
  __shared__ unsigned red[PROBE_THREADS / 64];
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) sink[blockIdx.x] = red[0] ^ red[1] ^ red[2] ^ red[3];
}

__global__ __launch_bounds__(PROBE_THREADS) void probe_mfma_kernel(int iters, float* __restrict__ sink) {
  // operands made from the lane id so that the compiler cannot fold the loop
  bf16x8 a, b;
  for (int e = 0; e < 8; ++e) {
    a[e] = (__bf16)(float)((threadIdx.x + e) & 3);
    b[e] = (__bf16)(float)((threadIdx.x * 3 + e) & 1);
  }
  f32x16 c0 = {}, c1 = {}, c2 = {}, c3 = {};
  for (int it = 0; it < iters; ++it) {
    c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
    c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
    c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
    c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
  }
  float s = 0.f;
  for (int e = 0; e < 16; ++e) s += c0[e] + c1[e] + c2[e] + c3[e];
  sink[(long)blockIdx.x * PROBE_THREADS + threadIdx.x] = s;
}

}  // namespace

size_t probe_sink_bytes(int kind, int blocks) {
  return kind == 0 ? (size_t)blocks * sizeof(unsigned) : (size_t)blocks * PROBE_THREADS * sizeof(float);
}

hipError_t launch_probe_read(hipStream_t s, const void* buf, long bytes, int blocks, void* sink) {
  probe_read_kernel<<<blocks, PROBE_THREADS, 0, s>>>((const u32x4*)buf, bytes / 16, (unsigned*)sink);
  return hipGetLastError();
}

hipError_t launch_probe_mfma(hipStream_t s, int iters, int blocks, void* sink) {
  probe_mfma_kernel<<<blocks, PROBE_THREADS, 0, s>>>(iters, (float*)sink);
  return hipGetLastError();
}

}  // namespace fard

// GEMM kernels: out = epilogue(A[M,K] * W[K,N]).
//
// bf16 path (gfx950 MFMA): weights are pre-laid in v_mfma_f32_32x32x16_bf16 B-fragment order so
// that every wave streams them from HBM straight into registers with fully contiguous 1 KiB
// loads (no LDS round trip for the operand that dominates the bytes when M is a few hundred
// rows).  The small activation tile goes through LDS, double-buffered, and is shared by the
// waves of a workgroup, each of which owns its own 32*WN output columns.  Workgroups are
// numbered so that all M-tiles of one weight panel land on the same XCD (ids are dealt to the
// 8 XCDs round-robin) and the panel is fetched from HBM once per L2.
//
// fp32 path: a plain LDS-tiled FMA kernel, used by the small all-fp32 configuration.
#include "gemm.h"

namespace fard {

namespace {

constexpr int BK = 64;                 // k per pipeline step (4 MFMA k-blocks of 16)
constexpr int LDS_STRIDE = BK + 8;     // bf16 per LDS row: 144 B keeps 16-byte reads conflict-poor

template <int WM, int WN, int NW>
__global__ __launch_bounds__(64 * NW) void gemm_bf16_kernel(GemmArgs a, int n_tiles, int m_tiles,
                                                            int splits, int steps_per_split) {
  constexpr int BM = 32 * WM;
  constexpr int THREADS = 64 * NW;
  constexpr int CHUNKS = BM * (BK / 8);                    // 16-byte chunks in one A tile
  constexpr int CPT = (CHUNKS + THREADS - 1) / THREADS;    // chunks per thread
  __shared__ __attribute__((aligned(16))) bf16 lds[2][BM * LDS_STRIDE];

  // blockIdx -> (weight panel, m tile): panels are dealt to XCDs, the m tiles of a panel are
  // consecutive slots of that XCD.
  const int id = blockIdx.x;
  const int xcd = id & 7, slot = id >> 3;
  const int pq = slot / m_tiles, mt = slot - pq * m_tiles;
  const int panel = pq * 8 + xcd;
  if (panel >= n_tiles * splits) return;
  const int nt = panel % n_tiles, sp = panel / n_tiles;

  const int M = eff_rows(a.M, a.m_dev);
  const int m0 = mt * BM;
  if (m0 >= M) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nblocks = a.N >> 5;
  const int kb16 = a.K >> 4;
  const int nb0 = (nt * NW + wave) * WN;
  const int total_steps = a.K / BK;
  const int t_begin = sp * steps_per_split;
  int T = total_steps - t_begin;
  if (T > steps_per_split) T = steps_per_split;

  const bf16* __restrict__ A = (const bf16*)a.A;
  const bf16x8* __restrict__ Wp = (const bf16x8*)a.W;

  f32x16 acc[WM][WN];
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  bf16x8 areg[CPT];
  bf16x8 breg[2][4][WN];

  auto load_a = [&](int t) {
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
      const int c = tid + i * THREADS;
      bf16x8 v;
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = (bf16)0.f;
      if (c < CHUNKS) {
        const int row = c >> 3, kc = c & 7;
        const int gr = m0 + row;
        if (gr < M) v = *(const bf16x8*)(A + (size_t)gr * a.lda + (size_t)(t_begin + t) * BK + kc * 8);
      }
      areg[i] = v;
    }
  };
  auto store_a = [&](int buf) {
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
      const int c = tid + i * THREADS;
      if (c < CHUNKS) {
        const int row = c >> 3, kc = c & 7;
        *(bf16x8*)(&lds[buf][row * LDS_STRIDE + kc * 8]) = areg[i];
      }
    }
  };
  auto load_b = [&](int t, bf16x8 (&b)[4][WN]) {
#pragma unroll
    for (int j = 0; j < WN; ++j) {
      if (nb0 + j < nblocks) {
        const bf16x8* p = Wp + ((size_t)(nb0 + j) * kb16 + (size_t)(t_begin + t) * 4) * 64 + lane;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) b[ks][j] = p[ks * 64];
      }
    }
  };
  auto compute = [&](int buf, const bf16x8 (&b)[4][WN]) {
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      bf16x8 af[WM];
#pragma unroll
      for (int i = 0; i < WM; ++i)
        af[i] = *(const bf16x8*)(&lds[buf][(32 * i + (lane & 31)) * LDS_STRIDE + ks * 16 + (lane >> 5) * 8]);
#pragma unroll
      for (int j = 0; j < WN; ++j) {
        if (nb0 + j < nblocks) {
#pragma unroll
          for (int i = 0; i < WM; ++i)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], b[ks][j], acc[i][j], 0, 0, 0);
        }
      }
    }
  };

  load_a(0);
  load_b(0, breg[0]);
  store_a(0);
  __syncthreads();
  for (int t = 0; t < T; t += 2) {
    if (t + 1 < T) { load_a(t + 1); load_b(t + 1, breg[1]); }
    compute(0, breg[0]);
    if (t + 1 < T) store_a(1);
    __syncthreads();
    if (t + 1 < T) {
      if (t + 2 < T) { load_a(t + 2); load_b(t + 2, breg[0]); }
      compute(1, breg[1]);
      if (t + 2 < T) store_a(0);
      __syncthreads();
    }
  }

  // epilogue: register e of a 32x32 accumulator holds row 8*(e/4) + 4*(lane/32) + e%4, column lane%32
  const int cl = lane & 31, rhalf = (lane >> 5) * 4;
  if (a.epi == EPI_SWIGLU) {
    if constexpr (WN == 2) {
      if (nb0 + 1 < nblocks) {
        const int col = (nb0 >> 1) * 32 + cl;
        bf16* out = (bf16*)a.out;
#pragma unroll
        for (int i = 0; i < WM; ++i)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int row = m0 + 32 * i + 8 * (e >> 2) + rhalf + (e & 3);
            if (row < M) out[(size_t)row * a.ldo + col] = (bf16)(silu(acc[i][0][e]) * acc[i][1][e]);
          }
      }
    }
    return;
  }
#pragma unroll
  for (int j = 0; j < WN; ++j) {
    if (nb0 + j >= nblocks) continue;
    const int col = (nb0 + j) * 32 + cl;
    const float bv = (a.bias != nullptr && sp == 0) ? a.bias[col] : 0.f;
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int row = m0 + 32 * i + 8 * (e >> 2) + rhalf + (e & 3);
        if (row >= M) continue;
        float v = acc[i][j][e] + bv;
        const size_t o = (size_t)row * a.ldo + col;
        if (a.epi == EPI_STORE) {
          ((bf16*)a.out)[o] = (bf16)apply_act(v, a.act);
        } else if (a.epi == EPI_STORE_F32) {
          ((float*)a.out)[o] = apply_act(v, a.act);
        } else {
          if (a.epi == EPI_GATE_RESID) v *= a.gate[(size_t)row * a.ldg + col];
          float* dst = (float*)a.out + o;
          if (splits > 1) atomicAdd(dst, v);     // partial sums of a split K range meet in memory
          else *dst += v;
        }
      }
  }
}

template <int WM, int WN, int NW>
hipError_t launch_cfg(hipStream_t s, const GemmArgs& a, int splits) {
  const int BN = 32 * WN * NW, BM = 32 * WM;
  const int n_tiles = (a.N + BN - 1) / BN;
  const int m_tiles = (a.M + BM - 1) / BM;
  const int total_steps = a.K / BK;
  if (splits > total_steps) splits = total_steps;
  if (splits < 1) splits = 1;
  const int sps = (total_steps + splits - 1) / splits;
  splits = (total_steps + sps - 1) / sps;
  const int panels = n_tiles * splits;
  const int grid = ((panels + 7) / 8) * 8 * m_tiles;
  gemm_bf16_kernel<WM, WN, NW><<<grid, 64 * NW, 0, s>>>(a, n_tiles, m_tiles, splits, sps);
  return hipGetLastError();
}

template <int WM>
hipError_t launch_wm(hipStream_t s, const GemmArgs& a) {
  const int m_tiles = (a.M + 32 * WM - 1) / (32 * WM);
  const bool resid = (a.epi == EPI_RESID || a.epi == EPI_GATE_RESID);
  // wide wave tiles only when that still leaves enough workgroups to cover the chip
  const int tiles_wn2 = ((a.N + 255) / 256) * m_tiles;
  const bool wn2 = (a.epi == EPI_SWIGLU) || tiles_wn2 >= 512;
  const int BN = wn2 ? 256 : 128;
  const int tiles = ((a.N + BN - 1) / BN) * m_tiles;
  int splits = 1;
  if (resid && tiles < 256) {
    splits = (256 + tiles - 1) / tiles;
    const int max_splits = a.K / (2 * BK) > 0 ? a.K / (2 * BK) : 1;   // keep >= 2 pipeline steps per split
    if (splits > max_splits) splits = max_splits;
    if (splits > 16) splits = 16;
  }
  return wn2 ? launch_cfg<WM, 2, 4>(s, a, splits) : launch_cfg<WM, 1, 4>(s, a, splits);
}

// ---------------------------------------------------------------------------------- fp32 path
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmArgs a) {
  __shared__ float As[16][17];
  __shared__ float Bs[16][17];
  __shared__ float Bu[16][17];
  const int M = eff_rows(a.M, a.m_dev);
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int row = blockIdx.y * 16 + ty, col = blockIdx.x * 16 + tx;
  const bool swiglu = a.epi == EPI_SWIGLU;
  const int ncols = swiglu ? a.N / 2 : a.N;
  if ((int)blockIdx.y * 16 >= M) return;
  const float* A = (const float*)a.A;
  const float* W = (const float*)a.W;
  float acc = 0.f, accu = 0.f;
  for (int k0 = 0; k0 < a.K; k0 += 16) {
    As[ty][tx] = (row < M && k0 + tx < a.K) ? A[(size_t)row * a.lda + k0 + tx] : 0.f;
    const bool ok = (k0 + ty < a.K) && (col < ncols);
    Bs[ty][tx] = ok ? W[(size_t)(k0 + ty) * a.N + col] : 0.f;
    if (swiglu) Bu[ty][tx] = ok ? W[(size_t)(k0 + ty) * a.N + ncols + col] : 0.f;
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      acc += As[ty][k] * Bs[k][tx];
      if (swiglu) accu += As[ty][k] * Bu[k][tx];
    }
    __syncthreads();
  }
  if (row >= M || col >= ncols) return;
  const size_t o = (size_t)row * a.ldo + col;
  if (swiglu) { ((float*)a.out)[o] = silu(acc) * accu; return; }
  float v = acc + (a.bias ? a.bias[col] : 0.f);
  if (a.epi == EPI_STORE || a.epi == EPI_STORE_F32) {
    ((float*)a.out)[o] = apply_act(v, a.act);
  } else {
    if (a.epi == EPI_GATE_RESID) v *= a.gate[(size_t)row * a.ldg + col];
    ((float*)a.out)[o] += v;
  }
}

template <typename TS>
__global__ void pack_weight_kernel(const TS* __restrict__ src, int ld, int K, int N, bf16x8* __restrict__ dst,
                                   int nb_offset, int nb_stride) {
  const int kb16 = K >> 4, nblocks = N >> 5;
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;   // (nb, kb, lane)
  const size_t total = (size_t)nblocks * kb16 * 64;
  if (idx >= total) return;
  const int lane = (int)(idx & 63);
  const size_t r = idx >> 6;
  const int kb = (int)(r % kb16), nb = (int)(r / kb16);
  const int n = nb * 32 + (lane & 31);
  const int k0 = kb * 16 + (lane >> 5) * 8;
  bf16x8 v;
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = (bf16)to_f32(src[(size_t)(k0 + i) * ld + n]);
  const size_t dnb = (size_t)nb_offset + (size_t)nb * nb_stride;
  dst[(dnb * kb16 + kb) * 64 + lane] = v;
}

}  // namespace

hipError_t launch_gemm_bf16(hipStream_t s, const GemmArgs& a) {
  if (a.M <= 0) return hipSuccess;
  if (a.K % BK != 0 || a.N % 32 != 0 || a.lda % 8 != 0) return hipErrorInvalidValue;
  if (a.epi == EPI_SWIGLU && a.N % 64 != 0) return hipErrorInvalidValue;
  if (a.M <= 32) return launch_wm<1>(s, a);
  if (a.M <= 64) return launch_wm<2>(s, a);
  return launch_wm<3>(s, a);
}

hipError_t launch_gemm_f32(hipStream_t s, const GemmArgs& a) {
  if (a.M <= 0) return hipSuccess;
  const int ncols = a.epi == EPI_SWIGLU ? a.N / 2 : a.N;
  dim3 grid((ncols + 15) / 16, (a.M + 15) / 16);
  gemm_f32_kernel<<<grid, 256, 0, s>>>(a);
  return hipGetLastError();
}

hipError_t launch_pack_weight(hipStream_t s, const void* src, int src_is_bf16, int ld, int K, int N,
                              void* dst, int nb_offset, int nb_stride) {
  if (K % 16 != 0 || N % 32 != 0) return hipErrorInvalidValue;
  const size_t total = (size_t)(N / 32) * (K / 16) * 64;
  const int threads = 256;
  const unsigned blocks = (unsigned)((total + threads - 1) / threads);
  if (src_is_bf16)
    pack_weight_kernel<bf16><<<blocks, threads, 0, s>>>((const bf16*)src, ld, K, N, (bf16x8*)dst, nb_offset, nb_stride);
  else
    pack_weight_kernel<float><<<blocks, threads, 0, s>>>((const float*)src, ld, K, N, (bf16x8*)dst, nb_offset, nb_stride);
  return hipGetLastError();
}

}  // namespace fard

// Narrow-tile GEMM for the small-batch GEMMs of a round.
//
// The draft steps and their diffusion-head decodes multiply a few dozen rows by 2-8 MB weight matrices,
// hundreds of times per round, in one dependent chain: a launch costs one memory round trip whatever it
// computes, so the kernel is built to need exactly one.  No K split, so any epilogue works without
// atomics and the result is deterministic.  One workgroup per 16 weight columns
// (v_mfma_f32_16x16x32_bf16: lane l holds row / column l % 16 and k = 8 (l / 16) .. + 8 of a 32-k step;
// accumulator register e is row 4 (l / 16) + e); the 4 waves interleave the 32-k steps.  Weight and
// activation fragments go straight from memory into MFMA operand registers -- the 16-column B fragment is
// two 256-byte halves of the packed 32-column fragments -- so a wave's first NS steps are one memory
// round trip with no LDS staging and no barrier before the MFMAs.  A workgroup owns MT x NT tiles of 16 x 16
// (NT > 1 when many row slabs would otherwise re-read the activations too often); blockIdx.y walks the
// row slabs.
//
// A norm that precedes the GEMM can be applied in the epilogue instead of by a launch of its own (LNF): the
// operand is the raw rows as bf16, the weights carry the norm's gain, every wave sums its rows' statistics from the
// activation fragments it feeds to the MFMAs, and the epilogue applies rstd, mean and the weights' column sums.
//
// Measured alternatives that lost and are not kept: 32-column tiles with K split over workgroups and fp32
// atomics (the atomics cost 1-2 us per launch and grow with the split count); normalising the operand while it
// is loaded (fp32 rows read in MFMA fragment order touch 4x the cache lines of the bf16 operand, and a separate
// pass over the rows for their statistics in every workgroup hot-spots the L2 lines of those rows).
#include "gemm.h"

namespace fard {

namespace {

// Epilogue of the narrow-tile kernels over the [16 MT, 16 NT] tile of a workgroup: a thread keeps one group of
// 4 columns and walks the rows.  The operands that do not depend on the product (gate, old value of a
// read-modify-write target, bias) are requested by prefetch() at kernel start; finish() adds the 4 waves'
// partial tiles through LDS and writes 8-16 bytes per thread.
// ADA: the kernel instance carries the operands of the modulated-norm fold (GemmArgs::ada_*, copy_scale, mom_out);
// the other instances keep their register budget.
template <int MT, int NT, bool ADA>
struct NarrowEpi {
  static constexpr int CG = 4 * NT;                        // 4-column groups per row
  static constexpr int RPP = 256 / CG;                     // rows per pass
  static constexpr int EP = (16 * MT + RPP - 1) / RPP;     // passes
  static constexpr int LDT = 16 * NT + 4;                  // floats per row of a partial tile in LDS
  static constexpr int ROWS = 16 * MT;                     // rows of the tile
  static constexpr int TPR = 256 / ROWS;                   // threads that share a row's tile moments (16 or 8 consecutive lanes)
  static constexpr int MOMT = 128 / TPR;                   // tile moments per thread: K <= 2048
  f32x4 gate[EP], old[EP], bias4, cs4;
  f32x4 c1[ADA ? EP : 1], c0[ADA ? EP : 1], vs[ADA ? EP : 1];   // modulated-norm fold (ada_*); scale of the bf16 copy
  float mom_m[ADA ? MOMT : 1], mom_q[ADA ? MOMT : 1], mom_pivot;   // this thread's share of its row's tile moments
  int er, ec;
  __device__ __forceinline__ void prefetch(const GemmArgs& a, int M, int m0, int n0) {
    er = threadIdx.x / CG;
    ec = (threadIdx.x % CG) * 4;
    bias4 = f32x4{0.f, 0.f, 0.f, 0.f};
    const bool rmw = (a.epi == EPI_RESID || a.epi == EPI_GATE_RESID);
#pragma unroll
    for (int i = 0; i < EP; ++i) {
      int r = m0 + er + RPP * i;
      r = r < M ? r : M - 1;
      gate[i] = f32x4{1.f, 1.f, 1.f, 1.f};
      old[i] = f32x4{0.f, 0.f, 0.f, 0.f};
      if (a.epi == EPI_GATE_RESID) gate[i] = *(const f32x4*)(a.gate + (size_t)r * a.ldg + n0 + ec);
      if (rmw) old[i] = *(const f32x4*)((const float*)a.out + (size_t)r * a.ldo + n0 + ec);
    }
    if (a.bias != nullptr && blockIdx.z == 0) bias4 = *(const f32x4*)(a.bias + n0 + ec);
    cs4 = f32x4{0.f, 0.f, 0.f, 0.f};
    if (a.ln_cs != nullptr) cs4 = *(const f32x4*)(a.ln_cs + n0 + ec);
    if constexpr (ADA) {
    if (a.ada_mom != nullptr || a.copy_scale != nullptr) {
#pragma unroll
      for (int i = 0; i < EP; ++i) {
        int r = m0 + er + RPP * i;
        r = r < M ? r : M - 1;
        if (a.ada_mom != nullptr) {
          c1[i] = *(const f32x4*)(a.ada_c1 + (size_t)r * a.ada_ld + n0 + ec);
          c0[i] = *(const f32x4*)(a.ada_c0 + (size_t)r * a.ada_ld + n0 + ec);
        }
        if (a.copy_scale != nullptr) vs[i] = *(const f32x4*)(a.copy_scale + (size_t)r * a.copy_ld + n0 + ec);
      }
    }
    if (a.ada_mom != nullptr) {
      // (mean, centred sum of squares) of every 16-column tile of the rows, left by the GEMM that wrote them:
      // thread t of the TPR that share row tid / TPR takes tiles t, t + TPR, ...
      int r = m0 + (int)threadIdx.x / TPR;
      r = r < M ? r : M - 1;
      const int n_tiles = a.K >> 4, t0 = threadIdx.x % TPR;
      typedef float f32x2 __attribute__((ext_vector_type(2)));
      const f32x2* mp = (const f32x2*)a.ada_mom + (size_t)r * a.ada_mom_ld;   // the row's tiles are consecutive pairs
      mom_pivot = mp[0][0];
#pragma unroll
      for (int i = 0; i < MOMT; ++i) {
        const int tile = t0 + TPR * i;
        const f32x2 q = mp[tile < n_tiles ? tile : 0];
        mom_m[i] = q[0];
        mom_q[i] = q[1];
      }
    }
    }
  }
  // mean and 1 / std of the tile's rows from the tile moments (pairwise update of Chan et al. for equal counts, about
  // the first tile's mean as pivot), into rowstat[row] = {mean, rstd}; all threads, before the epilogue's barrier
  __device__ __forceinline__ void row_stats(const GemmArgs& a, float* rowstat) {
    const int n_tiles = a.K >> 4, t0 = threadIdx.x % TPR;
    float sd = 0.f, sd2 = 0.f, sq = 0.f;
#pragma unroll
    for (int i = 0; i < MOMT; ++i) {
      if (t0 + TPR * i < n_tiles) {
        const float d = mom_m[i] - mom_pivot;
        sd += d;
        sd2 = fmaf(d, d, sd2);
        sq += mom_q[i];
      }
    }
    auto red = [](float v) {
      v += dpp_move<DPP_SWAP1>(v);
      v += dpp_move<DPP_SWAP2>(v);
      v += dpp_move<DPP_HALF_MIRROR>(v);
      if (TPR == 16) v += dpp_move<DPP_MIRROR>(v);
      return v;
    };
    sd = red(sd); sd2 = red(sd2); sq = red(sq);
    if (t0 == 0) {
      const float inv_t = 1.0f / (float)n_tiles;
      const float mean = mom_pivot + sd * inv_t;
      const float m2 = sq + 16.0f * fmaxf(sd2 - sd * sd * inv_t, 0.f);
      const int row = threadIdx.x / TPR;
      rowstat[row * 2] = mean;
      rowstat[row * 2 + 1] = 1.0f / sqrtf(m2 / (float)a.K + a.ada_eps);
    }
  }
  // LNF: stat holds the 4 waves' (sum x, sum x^2) of every row of the tile, over their shares of K
  template <bool LNF>
  __device__ __forceinline__ void finish(const GemmArgs& a, const f32x4 (&acc)[MT][NT], float* red, const float* stat,
                                         float* rowstat, int M, int m0, int n0) {
    const int lane = threadIdx.x & 63, kw = threadIdx.x >> 6;
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
      for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e)
          red[(kw * 16 * MT + 16 * i + 4 * (lane >> 4) + e) * LDT + 16 * j + (lane & 15)] = acc[i][j][e];
    if constexpr (ADA) { if (a.ada_mom != nullptr) row_stats(a, rowstat); }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < EP; ++i) {
      const int row = er + RPP * i;
      if (m0 + row >= M || row >= 16 * MT) continue;
      f32x4 v = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int k = 0; k < 4; ++k) v += *(const f32x4*)(red + (k * 16 * MT + row) * LDT + ec);
      if constexpr (LNF) {
        float s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          s1 += stat[(k * 16 * MT + row) * 2];
          s2 += stat[(k * 16 * MT + row) * 2 + 1];
        }
        const float inv_k = 1.0f / (float)a.K;
        const float mean = a.ln_rms ? 0.f : s1 * inv_k;
        const float var = fmaxf(s2 * inv_k - mean * mean, 0.f);
        const float rstd = rsqrtf(var + a.ln_eps);
        v = (v - cs4 * mean) * rstd;
      }
      if constexpr (ADA) { if (a.ada_mom != nullptr) v = (v - c1[i] * rowstat[row * 2]) * rowstat[row * 2 + 1] + c0[i]; }
      v += bias4;
      const size_t o = (size_t)(m0 + row) * a.ldo + n0 + ec;
      // the same 4 columns in tile order (GemmArgs::out_tiled): half a 16-byte piece
      const int gr = m0 + row, gc = n0 + ec;
      const size_t ot = ((((size_t)(gr >> 4) * (a.N >> 5) + (gc >> 5)) * 4 + ((gc >> 3) & 3)) * 16 + (gr & 15)) * 8 + (gc & 7);
      if (a.epi == EPI_STORE) {
        bf16x4 t;
#pragma unroll
        for (int e = 0; e < 4; ++e) t[e] = (bf16)apply_act(v[e], a.act);
        *(bf16x4*)((bf16*)a.out + (a.out_tiled ? ot : o)) = t;
      } else if (a.epi == EPI_STORE_F32) {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = apply_act(v[e], a.act);
        *(f32x4*)((float*)a.out + o) = v;
      } else if (a.epi == EPI_PARTIAL) {
        *(f32x4*)((float*)a.out + (size_t)blockIdx.z * a.part_stride + o) = v;
      } else {
        const f32x4 nv = old[i] + gate[i] * v;
        *(f32x4*)((float*)a.out + o) = nv;
        if (a.copy_bf16 != nullptr) {
          bf16x4 t;
          if (ADA && a.copy_scale != nullptr) {
#pragma unroll
            for (int e = 0; e < 4; ++e) t[e] = (bf16)(nv[e] * (1.0f + vs[ADA ? i : 0][e]));
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) t[e] = (bf16)nv[e];
          }
          *(bf16x4*)((bf16*)a.copy_bf16 + (a.out_tiled ? ot : o)) = t;
        }
        if (ADA && a.mom_out != nullptr) {
          // moments of the updated row over this 16-column tile: its 4 threads are one quad of lanes (the quad
          // shares the row, so it is whole or skipped as one)
          float sm = (nv[0] + nv[1]) + (nv[2] + nv[3]);
          sm += dpp_move<DPP_SWAP1>(sm);
          sm += dpp_move<DPP_SWAP2>(sm);
          const float mean = sm * (1.0f / 16.0f);
          float q = 0.f;
#pragma unroll
          for (int e = 0; e < 4; ++e) { const float d = nv[e] - mean; q = fmaf(d, d, q); }
          q += dpp_move<DPP_SWAP1>(q);
          q += dpp_move<DPP_SWAP2>(q);
          if ((threadIdx.x & 3) == 0) {
            typedef float f32x2 __attribute__((ext_vector_type(2)));
            *((f32x2*)a.mom_out + (size_t)(m0 + row) * a.mom_ld + ((n0 + ec) >> 4)) = f32x2{mean, q};
          }
        }
      }
    }
  }
};

// MT x NT: 16x16 output tiles of the workgroup (rows x columns).  NS: k-steps per operand a wave keeps in
// flight (its whole K range when ONESHOT).
// LNF: the norm of the rows is applied in the epilogue (GemmArgs::ln_cs); the row statistics are summed from the
// activation fragments on their way into the MFMAs.
template <int MT, int NT, int NS, bool ONESHOT, bool LNF, bool ADA>
__global__ __launch_bounds__(256, (LNF && NS == 8 && !ADA) ? 2 : 1) void gemm_narrow_kernel(GemmArgs a) {   // (the statistics must
  // not cost the 32 x 64 tile its second workgroup per compute unit: 16 registers over the limit otherwise)
  using Epi = NarrowEpi<MT, NT, ADA>;
  extern __shared__ __attribute__((aligned(16))) float red[];   // 4 * 16 * MT * Epi::LDT floats (+ 4 * 16 * MT * 2 if LNF) + 16 * MT * 2
  // The operand loads are clamped by the host's row bound; the device-side row count, a dependent read, is only waited
  // for when the loads are in flight (a launch would otherwise spend one more memory round trip before its first load).
  const int Mh = a.M;
  const int m0 = blockIdx.y * 16 * MT;                     // row slab of this workgroup
  if (m0 >= Mh) return;
  const int tid = threadIdx.x, lane = tid & 63, kw = tid >> 6;
  const int kb16 = a.K >> 4;
  // K slice of this workgroup (blockIdx.z; the whole K unless EPI_PARTIAL): 32-k steps [s0, s0 + kb32)
  const int sps = ((a.K >> 5) + (int)gridDim.z - 1) / (int)gridDim.z;
  const int s0 = blockIdx.z * sps;
  const int kb32 = min(sps, (a.K >> 5) - s0);
  const int my_steps = (kb32 - kw + 3) >> 2;               // steps s0 + kw, s0 + kw + 4, ... (may be 0)
  const int n0 = blockIdx.x * 16 * NT;

  // packed B: fragment (nb, kb16 index) holds lane L = 32 * (k / 8 % 2) + n % 32
  const int kg = lane >> 4;                                // k group of this lane inside a 32-k step
  const bf16x8* __restrict__ bbase[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    const int c16 = blockIdx.x * NT + j;
    bbase[j] = (const bf16x8*)a.W + (size_t)(c16 >> 1) * kb16 * 64 + (kg >> 1) * 64 + (kg & 1) * 32 + (c16 & 1) * 16 +
               (lane & 15);
  }
  const bf16* __restrict__ abase[MT];
  const int a_step = a.a_tiled ? 512 : 32;                 // elements between a lane's pieces of consecutive 32-k steps
#pragma unroll
  for (int i = 0; i < MT; ++i) {
    int r = m0 + 16 * i + (lane & 15);
    r = r < Mh ? r : Mh - 1;                               // (a workgroup's last row tiles may lie past the matrix)
    if (a.a_tiled) {                                       // tile order (GemmArgs::a_tiled)
      abase[i] = (const bf16*)a.A + (((size_t)(r >> 4) * (a.K >> 5) * 4 + kg) * 16 + (r & 15)) * 8;
    } else {
      abase[i] = (const bf16*)a.A + (size_t)r * a.lda + kg * 8;
    }
  }
  bf16x8 breg[NS][NT], areg[NS][MT];
  auto load_ab = [&](int t, int p) {
    int s = kw + 4 * t;
    s = s0 + (s < kb32 ? s : kb32 - 1);                    // past the end: a re-read, zeroed at use
#pragma unroll
    for (int j = 0; j < NT; ++j) breg[p][j] = bbase[j][(size_t)s * 128];
#pragma unroll
    for (int i = 0; i < MT; ++i) areg[p][i] = *(const bf16x8*)(abase[i] + (size_t)s * a_step);
  };
#pragma unroll
  for (int p = 0; p < NS; ++p) load_ab(p, p);

  Epi epi;
  epi.prefetch(a, Mh, m0, n0);
  const int M = eff_rows(a.M, a.m_dev);
  if (m0 >= M) return;                                     // (uniform over the workgroup)
  __builtin_amdgcn_sched_barrier(0);

  f32x4 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  bf16x8 zero8;
#pragma unroll
  for (int e = 0; e < 8; ++e) zero8[e] = (bf16)0.f;
  float s1[MT], s2[MT];
#pragma unroll
  for (int i = 0; i < MT; ++i) s1[i] = s2[i] = 0.f;
  auto step = [&](int g, bool live) {
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      const bf16x8 af = live ? areg[g][i] : zero8;
      if constexpr (LNF) {
        // sum x and sum x^2 of the fragment's 8 values, two per instruction (v_dot2c_f32_bf16: fp32 accumulate)
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        bf16x2 ones;
        ones[0] = (bf16)1.0f;
        ones[1] = (bf16)1.0f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          bf16x2 pr;
          pr[0] = af[2 * e];
          pr[1] = af[2 * e + 1];
          s1[i] = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, s1[i], false);
          s2[i] = __builtin_amdgcn_fdot2_f32_bf16(pr, pr, s2[i], false);
        }
      }
#pragma unroll
      for (int j = 0; j < NT; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af, breg[g][j], acc[i][j], 0, 0, 0);
    }
  };
  if constexpr (ONESHOT) {
#pragma unroll
    for (int g = 0; g < NS; ++g) step(g, g < my_steps);
  } else {
    for (int t0 = 0; t0 < my_steps; t0 += NS) {
#pragma unroll
      for (int g = 0; g < NS; ++g) {
        step(g, t0 + g < my_steps);
        load_ab(t0 + g + NS, g);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }

  float* stat = red + 4 * 16 * MT * Epi::LDT;
  float* rowstat = stat + (LNF ? 4 * 16 * MT * 2 : 0);
  if constexpr (LNF) {
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      s1[i] = xor32_sum(xor16_sum(s1[i]));
      s2[i] = xor32_sum(xor16_sum(s2[i]));
      if (lane < 16) {
        stat[(kw * 16 * MT + 16 * i + lane) * 2] = s1[i];
        stat[(kw * 16 * MT + 16 * i + lane) * 2 + 1] = s2[i];
      }
    }
  }
  epi.template finish<LNF>(a, acc, red, stat, rowstat, M, m0, n0);
}

}  // namespace

bool narrow_supported(const GemmArgs& a) {
  if (a.epi == EPI_PARTIAL && (a.k_slices < 1 || a.k_slices > 64 || (a.k_slices > 1 && a.part_stride < (size_t)a.M * a.ldo))) return false;
  if (a.ln_cs != nullptr && (a.epi == EPI_PARTIAL || a.k_slices > 1)) return false;
  if (a.copy_bf16 != nullptr && a.epi != EPI_RESID && a.epi != EPI_GATE_RESID) return false;
  if (a.copy_scale != nullptr && a.copy_bf16 == nullptr) return false;
  if (a.out_tiled && !(a.epi == EPI_STORE || a.copy_bf16 != nullptr)) return false;
  if (a.out_tiled && a.k_slices > 1) return false;
  if ((a.a_tiled && a.K % 32 != 0) || (a.out_tiled && a.N % 32 != 0)) return false;
  if (a.mom_out != nullptr && a.epi != EPI_RESID && a.epi != EPI_GATE_RESID) return false;
  if (a.ada_mom != nullptr && ((a.epi != EPI_STORE && a.epi != EPI_STORE_F32) || a.ln_cs != nullptr || a.K > 2048 ||
                               a.ada_c1 == nullptr || a.ada_c0 == nullptr))
    return false;
  return a.M >= 1 && a.N % 32 == 0 && a.K % 64 == 0 && a.epi != EPI_SWIGLU;
}

hipError_t launch_gemm_narrow(hipStream_t s, const GemmArgs& a) {
  if (!narrow_supported(a)) return hipErrorInvalidValue;
  const int kz = (a.epi == EPI_PARTIAL && a.k_slices > 1) ? a.k_slices : 1;
  const int steps = ((a.K / 32 + kz - 1) / kz + 3) / 4;      // 32-k steps of the busiest wave
  // rows beyond one workgroup's tile go to further workgroups (blockIdx.y) that re-read the weight columns
  // out of L2: ids of one column tile differ by a multiple of 8, so they share an XCD when N % 128 == 0
#define FARD_NR_L(MTV, NTV, NSV, ONE, LNFV, ADAV)                                                          \
  do {                                                                                                     \
    constexpr size_t lds = ((size_t)4 * 16 * MTV * (16 * NTV + 4 + (LNFV ? 2 : 0)) + 16 * MTV * 2) * sizeof(float); \
    if constexpr (lds > 64 * 1024) {                                                                       \
      static bool attr_set = false;                                                                        \
      if (!attr_set) {                                                                                     \
        hipError_t e = hipFuncSetAttribute((const void*)gemm_narrow_kernel<MTV, NTV, NSV, ONE, LNFV, ADAV>, \
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);          \
        if (e != hipSuccess) return e;                                                                     \
        attr_set = true;                                                                                   \
      }                                                                                                    \
    }                                                                                                      \
    gemm_narrow_kernel<MTV, NTV, NSV, ONE, LNFV, ADAV><<<dim3(a.N / (16 * NTV), (a.M + 16 * MTV - 1) / (16 * MTV), kz), 256, lds, s>>>(a); \
  } while (0)
  // the modulated-norm fold: the tile shapes the head's GEMMs take (K = N <= 1536)
  if (a.ada_mom != nullptr || a.mom_out != nullptr || a.copy_scale != nullptr) {
    if (a.ln_cs != nullptr || steps > 12) return hipErrorInvalidValue;
    if (a.M <= 64) { if (steps <= 8) FARD_NR_L(1, 1, 8, true, false, true); else FARD_NR_L(1, 1, 12, true, false, true); }
    else if (steps <= 8 && a.N % 64 == 0) FARD_NR_L(2, 4, 8, true, false, true);
    else if (steps <= 8) FARD_NR_L(2, 2, 8, true, false, true);
    else FARD_NR_L(2, 2, 12, true, false, true);
    return hipGetLastError();
  }
#define FARD_NR(MTV, NTV, NSV, ONE)                      \
  do {                                                   \
    if (a.ln_cs != nullptr) FARD_NR_L(MTV, NTV, NSV, ONE, true, false); \
    else FARD_NR_L(MTV, NTV, NSV, ONE, false, false);    \
  } while (0)
  if (a.M <= 64) {
    // a few dozen rows: 16-row workgroups (more of them, half the activation bytes each) measured ahead of
    // 32-row ones; two column tiles per workgroup once the matrix is wide
    const bool wide = a.N >= 2048;
    if (steps <= 8) { if (wide) FARD_NR(1, 2, 8, true); else FARD_NR(1, 1, 8, true); }
    else if (steps <= 12) { if (wide) FARD_NR(1, 2, 12, true); else FARD_NR(1, 1, 12, true); }
    else if (steps <= 16) { if (wide) FARD_NR(1, 2, 16, true); else FARD_NR(1, 1, 16, true); }
    else FARD_NR(1, 1, 8, false);
  } else if (steps <= 8 && a.N % 64 == 0) {
    // several row slabs: 64 columns per workgroup quarter the re-reads of the activations (measured best at
    // 288 rows for N = 1024 .. 4096; slabs of 48, 64 or 96 rows re-read the weights less often but lengthen every
    // workgroup's chain of load, MFMAs and epilogue: a round is 9-17 % slower with them)
    FARD_NR(2, 4, 8, true);
  } else if (steps <= 12) {
    if (steps <= 8) FARD_NR(2, 2, 8, true);
    else FARD_NR(2, 2, 12, true);
  } else {
    if (steps <= 16) FARD_NR(2, 1, 16, true);
    else FARD_NR(2, 1, 8, false);
  }
#undef FARD_NR
#undef FARD_NR_L
  return hipGetLastError();
}

}  // namespace fard

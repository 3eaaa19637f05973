// Skinny GEMM (M <= 64 rows) with fused activation-side work.
//
// The draft steps and their diffusion-head decodes multiply at most a few dozen rows by 2-40 MB weight
// matrices, hundreds of times per round, in one dependent chain: every launch costs one memory round
// trip whatever it computes, so the chain is shortened by doing the row-wise work that sits between two
// GEMMs inside the GEMMs themselves:
//  * SK_A_NORM: the activation operand is norm(h) (layer / RMS norm, optional gain and bias, optional
//    per-row AdaLN scale and shift); every workgroup recomputes the statistics of its <= 64 rows from the
//    fp32 stream (a few hundred KB out of L2) and normalises only its own K slice;
//  * SK_A_ACT: the operand is act(acc + bias): the previous GEMM left raw fp32 partial sums (split-K
//    atomics into a zeroed buffer), and its bias and activation are applied here on load;
//  * a workgroup can also clear a slice of an unrelated buffer (the next accumulation target).
// Layout of a launch: one workgroup per (32 weight columns, K slice); its 4 waves interleave the k-steps
// of the slice; all weight fragments of a wave (or the first 8) and the gate values of the epilogue are
// requested before anything else; the activation slice goes through LDS once; partial tiles of the 4
// waves meet in LDS and leave as 16-byte row-contiguous accesses (fp32 atomics when K is split).
#include "gemm.h"

namespace fard {

namespace {

constexpr int SK_P = 8;                 // weight fragments a wave keeps in flight
constexpr int SK_LDT = 36;              // floats per row of a partial tile in LDS (32 + 4: conflict-free float4 reads)
constexpr int SK_NV = 8;                // a normalised row is at most 8 * 256 elements

__device__ __forceinline__ bf16x4 pack4(float a, float b, float c, float d) {
  bf16x4 o;
  o[0] = (bf16)a; o[1] = (bf16)b; o[2] = (bf16)c; o[3] = (bf16)d;
  return o;
}

template <int WM, int AMODE>
__global__ __launch_bounds__(256) void gemm_skinny_kernel(SkinnyArgs x, int n_tiles, int splits, int sps,
                                                          int lds_stride) {
  constexpr int BM = 32 * WM;
  extern __shared__ __attribute__((aligned(16))) char lds_raw[];
  bf16* lds_a = (bf16*)lds_raw;
  const GemmArgs& a = x.g;
  const int id = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, kw = tid >> 6;

  // side job: clear this workgroup's share of an unrelated buffer
  if (x.zero_ptr != nullptr) {
    const int per = (((x.zero_n + (int)gridDim.x - 1) / (int)gridDim.x) + 3) & ~3;
    const int lo = id * per;
    int hi = lo + per;
    if (hi > x.zero_n) hi = x.zero_n;
    for (int i = lo + tid * 4; i < hi; i += 1024) *(f32x4*)(x.zero_ptr + i) = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  const int M = eff_rows(a.M, a.m_dev);
  if (M <= 0) return;
  const int sp = id % splits, nt = id / splits;            // splits of one column tile are neighbours
  const int kb16 = a.K >> 4;
  const int s_begin = sp * sps;
  int n_steps = kb16 - s_begin;
  if (n_steps > sps) n_steps = sps;
  const int my_steps = (n_steps - kw + 3) >> 2;            // this wave: steps kw, kw + 4, ...
  const int k0 = s_begin * 16, ks = n_steps * 16;
  const int n0 = nt * 32;

  // ---- weight ring: slot p holds the wave's step t with t % SK_P == p
  const bf16x8* __restrict__ bbase = (const bf16x8*)a.W + ((size_t)nt * kb16 + s_begin) * 64 + lane;
  bf16x8 breg[SK_P];
  auto load_b = [&](int t, int p) {
    int s = kw + 4 * t;
    s = s < n_steps ? s : n_steps - 1;                     // past the end: a re-read, zeroed at use
    breg[p] = bbase[(size_t)s * 64];
  };
#pragma unroll
  for (int p = 0; p < SK_P; ++p) load_b(p, p);

  // ---- epilogue operands that do not depend on the product
  const int er = tid >> 3, ec = (tid & 7) * 4;             // thread -> (row, 4 columns) of the output tile
  f32x4 gate[WM], bias4 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int i = 0; i < WM; ++i) {
    gate[i] = f32x4{1.f, 1.f, 1.f, 1.f};
    if (a.epi == EPI_GATE_RESID) {
      int r = er + 32 * i;
      r = r < M ? r : M - 1;
      gate[i] = *(const f32x4*)(a.gate + (size_t)r * a.ldg + n0 + ec);
    }
  }
  if (a.bias != nullptr && sp == 0) bias4 = *(const f32x4*)(a.bias + n0 + ec);
  __builtin_amdgcn_sched_barrier(0);

  // ---- activation slice [BM rows, ks] -> LDS as bf16 (rows past M repeat row M - 1; never stored)
  const int ppr = n_steps * 2;                             // 8-element pieces per row
  const int pieces = BM * ppr;
  if constexpr (AMODE == SK_A_BF16) {
    const bf16* __restrict__ A = (const bf16*)a.A;
    for (int p0 = 0; p0 < pieces; p0 += 8 * 256) {
      bf16x8 v[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        int p = p0 + i * 256 + tid;
        p = p < pieces ? p : pieces - 1;
        int row = p / ppr;
        const int kc = p - row * ppr;
        row = row < M ? row : M - 1;
        v[i] = *(const bf16x8*)(A + (size_t)row * a.lda + k0 + kc * 8);
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int p = p0 + i * 256 + tid;
        if (p < pieces) {
          const int row = p / ppr, kc = p - row * ppr;
          *(bf16x8*)(lds_a + row * lds_stride + kc * 8) = v[i];
        }
      }
    }
  } else if constexpr (AMODE == SK_A_ACT) {
    const float* __restrict__ A = (const float*)a.A;
    for (int p0 = 0; p0 < pieces; p0 += 4 * 256) {
      f32x4 v[4][2], bb[4][2];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        int p = p0 + i * 256 + tid;
        p = p < pieces ? p : pieces - 1;
        int row = p / ppr;
        const int kc = p - row * ppr;
        row = row < M ? row : M - 1;
        const float* src = A + (size_t)row * a.lda + k0 + kc * 8;
        v[i][0] = *(const f32x4*)src;
        v[i][1] = *(const f32x4*)(src + 4);
        if (x.a_bias != nullptr) {
          bb[i][0] = *(const f32x4*)(x.a_bias + k0 + kc * 8);
          bb[i][1] = *(const f32x4*)(x.a_bias + k0 + kc * 8 + 4);
        } else {
          bb[i][0] = bb[i][1] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int p = p0 + i * 256 + tid;
        if (p < pieces) {
          const int row = p / ppr, kc = p - row * ppr;
          bf16x8 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            o[e] = (bf16)apply_act(v[i][0][e] + bb[i][0][e], x.a_act);
            o[4 + e] = (bf16)apply_act(v[i][1][e] + bb[i][1][e], x.a_act);
          }
          *(bf16x8*)(lds_a + row * lds_stride + kc * 8) = o;
        }
      }
    }
  } else {
    // SK_A_NORM.  Two prefetched pieces per thread cover a [32, 128] slice; the rest is fetched after the statistics.
    const float* __restrict__ H = (const float*)a.A;
    float* stats = (float*)(lds_raw + (size_t)BM * lds_stride * 2);      // [BM][2]: mean, 1/std
    constexpr int PF = 2;
    f32x4 hv[PF][2], scv[PF][2], shv[PF][2];
    auto fetch_piece = [&](int p, f32x4 (&h2)[2], f32x4 (&sc2)[2], f32x4 (&sh2)[2]) {
      p = p < pieces ? p : pieces - 1;
      int row = p / ppr;
      const int kc = p - row * ppr;
      row = row < M ? row : M - 1;
      const int col = k0 + kc * 8;
      const float* src = H + (size_t)row * a.lda + col;
      h2[0] = *(const f32x4*)src;
      h2[1] = *(const f32x4*)(src + 4);
      if (x.ln_scale != nullptr) {
        const float* s1 = x.ln_scale + (size_t)row * x.ld_mod + col;
        const float* s2 = x.ln_shift + (size_t)row * x.ld_mod + col;
        sc2[0] = *(const f32x4*)s1; sc2[1] = *(const f32x4*)(s1 + 4);
        sh2[0] = *(const f32x4*)s2; sh2[1] = *(const f32x4*)(s2 + 4);
      }
    };
    auto finish_piece = [&](int p, const f32x4 (&h2)[2], const f32x4 (&sc2)[2], const f32x4 (&sh2)[2]) {
      if (p >= pieces) return;
      const int row = p / ppr, kc = p - row * ppr;
      const int col = k0 + kc * 8;
      const float mean = stats[2 * row], rstd = stats[2 * row + 1];
      bf16x8 o;
#pragma unroll
      for (int hlf = 0; hlf < 2; ++hlf) {
        f32x4 y;
#pragma unroll
        for (int e = 0; e < 4; ++e) y[e] = (h2[hlf][e] - mean) * rstd;
        if (x.ln_gain != nullptr) y *= *(const f32x4*)(x.ln_gain + col + 4 * hlf);
        if (x.ln_beta != nullptr) y += *(const f32x4*)(x.ln_beta + col + 4 * hlf);
        if (x.ln_scale != nullptr) y = y * (1.0f + sc2[hlf]) + sh2[hlf];
#pragma unroll
        for (int e = 0; e < 4; ++e) o[4 * hlf + e] = (bf16)y[e];
      }
      *(bf16x8*)(lds_a + row * lds_stride + kc * 8) = o;
    };
#pragma unroll
    for (int i = 0; i < PF; ++i) fetch_piece(i * 256 + tid, hv[i], scv[i], shv[i]);
    __builtin_amdgcn_sched_barrier(0);
    // statistics: wave kw owns rows kw, kw + 4, ...; two rows at a time, each row whole in registers
    const int nv = a.K >> 8;                               // K % 256 == 0, K <= 256 * SK_NV (host check)
    const float inv_k = 1.0f / (float)a.K;
    for (int r0 = kw; r0 < BM; r0 += 8) {
      f32x4 v[2][SK_NV];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        int row = r0 + 4 * u;
        row = row < M ? row : M - 1;
        const f32x4* src = (const f32x4*)(H + (size_t)row * a.lda);
#pragma unroll
        for (int i = 0; i < SK_NV; ++i)
          if (i < nv) v[u][i] = src[lane + 64 * i];
      }
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < SK_NV; ++i)
          if (i < nv) s += v[u][i][0] + v[u][i][1] + v[u][i][2] + v[u][i][3];
        const float mean = (x.norm_kind == 0) ? wave_sum(s) * inv_k : 0.f;
        float q = 0.f;
#pragma unroll
        for (int i = 0; i < SK_NV; ++i)
          if (i < nv) {
#pragma unroll
            for (int e = 0; e < 4; ++e) { const float t = v[u][i][e] - mean; q += t * t; }
          }
        const float var = wave_sum(q) * inv_k;
        if (lane == 0 && r0 + 4 * u < BM) {
          stats[2 * (r0 + 4 * u)] = mean;
          stats[2 * (r0 + 4 * u) + 1] = 1.0f / sqrtf(var + x.ln_eps);
        }
      }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < PF; ++i) finish_piece(i * 256 + tid, hv[i], scv[i], shv[i]);
    for (int p0 = PF * 256; p0 < pieces; p0 += 2 * 256) {
      f32x4 h2[2][2], sc2[2][2], sh2[2][2];
#pragma unroll
      for (int i = 0; i < 2; ++i) fetch_piece(p0 + i * 256 + tid, h2[i], sc2[i], sh2[i]);
#pragma unroll
      for (int i = 0; i < 2; ++i) finish_piece(p0 + i * 256 + tid, h2[i], sc2[i], sh2[i]);
    }
  }
  __syncthreads();

  // ---- MFMA loop: A fragments from LDS one step ahead, weights from the ring
  f32x16 acc[WM];
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
  bf16x8 zero8;
#pragma unroll
  for (int e = 0; e < 8; ++e) zero8[e] = (bf16)0.f;
  const int foff = (lane & 31) * lds_stride + (lane >> 5) * 8;
  auto frag = [&](int t, bf16x8 (&f)[WM]) {
    int s = kw + 4 * t;
    s = s < n_steps ? s : n_steps - 1;
#pragma unroll
    for (int i = 0; i < WM; ++i) f[i] = *(const bf16x8*)(lds_a + 32 * i * lds_stride + foff + s * 16);
  };
  bf16x8 af[2][WM];
  frag(0, af[0]);
  for (int t0 = 0; t0 < my_steps; t0 += SK_P) {
#pragma unroll
    for (int g = 0; g < SK_P; ++g) {
      const int t = t0 + g;
      frag(t + 1, af[(g + 1) & 1]);
      const bool live = t < my_steps;
#pragma unroll
      for (int i = 0; i < WM; ++i)
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(live ? af[g & 1][i] : zero8, breg[g], acc[i], 0, 0, 0);
      load_b(t + SK_P, g);
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  // ---- partial tiles of the 4 waves meet in LDS
  float* red = (float*)lds_raw;
  __syncthreads();                                         // the activation slice is no longer read
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int row = 32 * i + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
      red[(kw * BM + row) * SK_LDT + (lane & 31)] = acc[i][e];
    }
  __syncthreads();
  const bool atomic = splits > 1;
#pragma unroll
  for (int i = 0; i < WM; ++i) {
    const int row = er + 32 * i;
    if (row >= M) continue;
    f32x4 v = bias4;
#pragma unroll
    for (int k = 0; k < 4; ++k) v += *(const f32x4*)(red + (k * BM + row) * SK_LDT + ec);
    const size_t o = (size_t)row * a.ldo + n0 + ec;
    if (a.epi == EPI_STORE) {
      *(bf16x4*)((bf16*)a.out + o) = pack4(apply_act(v[0], a.act), apply_act(v[1], a.act), apply_act(v[2], a.act),
                                            apply_act(v[3], a.act));
    } else if (a.epi == EPI_STORE_F32) {
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = apply_act(v[e], a.act);
      *(f32x4*)((float*)a.out + o) = v;
    } else {
      v *= gate[i];
      float* dst = (float*)a.out + o;
      if (atomic) {
#pragma unroll
        for (int e = 0; e < 4; ++e) atomicAdd(dst + e, v[e]);
      } else {
        *(f32x4*)dst = *(const f32x4*)dst + v;
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------------
// Narrow-tile variant: no K split, so any epilogue works without atomics and the result is
// deterministic.  One workgroup per 16 weight columns (v_mfma_f32_16x16x32_bf16: lane l holds row /
// column l % 16 and k = 8 (l / 16) .. + 8 of a 32-k step; accumulator register e is row 4 (l / 16) + e);
// the 4 waves interleave the 32-k steps.  Weight and activation fragments go straight from memory into
// MFMA operand registers -- the 16-column B fragment is two 256-byte halves of the packed 32-column
// fragments -- so a wave's first SK_P steps are one memory round trip with no LDS staging and no
// barrier before the MFMAs.  MT: 16-row tiles per workgroup; blockIdx.y walks the row slabs.
constexpr int NR_LDT = 20;              // floats per row of a partial tile in LDS

template <int MT, bool ONESHOT>
__global__ __launch_bounds__(256) void gemm_narrow_kernel(GemmArgs a) {
  __shared__ __attribute__((aligned(16))) float red[4 * 16 * MT * NR_LDT];
  const int M = eff_rows(a.M, a.m_dev);
  const int m0 = blockIdx.y * 16 * MT;                     // row slab of this workgroup
  if (m0 >= M) return;
  const int c16 = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, kw = tid >> 6;
  const int kb16 = a.K >> 4, kb32 = a.K >> 5;
  const int my_steps = (kb32 - kw + 3) >> 2;               // steps kw, kw + 4, ... (may be 0)
  const int n0 = c16 * 16;

  // packed B: fragment (nb, kb16 index) holds lane L = 32 * (k / 8 % 2) + n % 32
  const int kg = lane >> 4;                                // k group of this lane inside a 32-k step
  const bf16x8* __restrict__ bbase = (const bf16x8*)a.W + (size_t)(c16 >> 1) * kb16 * 64 + (kg >> 1) * 64 +
                                     (kg & 1) * 32 + (c16 & 1) * 16 + (lane & 15);
  const bf16* __restrict__ abase[MT];
#pragma unroll
  for (int i = 0; i < MT; ++i) {
    int r = m0 + 16 * i + (lane & 15);
    r = r < M ? r : M - 1;
    abase[i] = (const bf16*)a.A + (size_t)r * a.lda + kg * 8;
  }
  bf16x8 breg[SK_P], areg[SK_P][MT];
  auto load_ab = [&](int t, int p) {
    int s = kw + 4 * t;
    s = s < kb32 ? s : kb32 - 1;                           // past the end: a re-read, zeroed at use
    breg[p] = bbase[(size_t)s * 128];
#pragma unroll
    for (int i = 0; i < MT; ++i) areg[p][i] = *(const bf16x8*)(abase[i] + (size_t)s * 32);
  };
#pragma unroll
  for (int p = 0; p < SK_P; ++p) load_ab(p, p);

  // epilogue operands that do not depend on the product: thread -> (row, 2 columns)
  const int er = tid >> 3, ec = (tid & 7) * 2;
  constexpr int EP = (16 * MT + 31) / 32;                  // passes of 32 rows
  float2 gate[EP], old[EP], bias2 = {0.f, 0.f};
  const bool rmw = (a.epi == EPI_RESID || a.epi == EPI_GATE_RESID);
#pragma unroll
  for (int i = 0; i < EP; ++i) {
    int r = m0 + er + 32 * i;
    r = r < M ? r : M - 1;
    gate[i] = float2{1.f, 1.f};
    old[i] = float2{0.f, 0.f};
    if (a.epi == EPI_GATE_RESID) gate[i] = *(const float2*)(a.gate + (size_t)r * a.ldg + n0 + ec);
    if (rmw) old[i] = *(const float2*)((const float*)a.out + (size_t)r * a.ldo + n0 + ec);
  }
  if (a.bias != nullptr) bias2 = *(const float2*)(a.bias + n0 + ec);
  __builtin_amdgcn_sched_barrier(0);

  f32x4 acc[MT];
#pragma unroll
  for (int i = 0; i < MT; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  bf16x8 zero8;
#pragma unroll
  for (int e = 0; e < 8; ++e) zero8[e] = (bf16)0.f;
  if constexpr (ONESHOT) {
#pragma unroll
    for (int g = 0; g < SK_P; ++g) {
      const bf16x8 b = (g < my_steps) ? breg[g] : zero8;
#pragma unroll
      for (int i = 0; i < MT; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(areg[g][i], b, acc[i], 0, 0, 0);
    }
  } else {
    for (int t0 = 0; t0 < my_steps; t0 += SK_P) {
#pragma unroll
      for (int g = 0; g < SK_P; ++g) {
        const bf16x8 b = (t0 + g < my_steps) ? breg[g] : zero8;
#pragma unroll
        for (int i = 0; i < MT; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(areg[g][i], b, acc[i], 0, 0, 0);
        load_ab(t0 + g + SK_P, g);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }

  // partial tiles of the 4 waves meet in LDS
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int e = 0; e < 4; ++e)
      red[(kw * 16 * MT + 16 * i + 4 * (lane >> 4) + e) * NR_LDT + (lane & 15)] = acc[i][e];
  __syncthreads();
#pragma unroll
  for (int i = 0; i < EP; ++i) {
    const int row = er + 32 * i;
    if (m0 + row >= M || row >= 16 * MT) continue;
    float2 v = bias2;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float2 pv = *(const float2*)(red + (k * 16 * MT + row) * NR_LDT + ec);
      v.x += pv.x;
      v.y += pv.y;
    }
    const size_t o = (size_t)(m0 + row) * a.ldo + n0 + ec;
    if (a.epi == EPI_STORE) {
      bf16* dst = (bf16*)a.out + o;
      typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
      bf16x2 t;
      t[0] = (bf16)apply_act(v.x, a.act);
      t[1] = (bf16)apply_act(v.y, a.act);
      *(bf16x2*)dst = t;
    } else if (a.epi == EPI_STORE_F32) {
      *(float2*)((float*)a.out + o) = float2{apply_act(v.x, a.act), apply_act(v.y, a.act)};
    } else {
      *(float2*)((float*)a.out + o) = float2{old[i].x + gate[i].x * v.x, old[i].y + gate[i].y * v.y};
    }
  }
}

template <int WM, int AMODE>
hipError_t launch_skinny_t(hipStream_t s, const SkinnyArgs& x, int n_tiles, int splits, int sps) {
  const int BM = 32 * WM;
  const int lds_stride = sps * 16 + 8;
  size_t lds = (size_t)BM * lds_stride * 2 + (size_t)BM * 8;
  const size_t red = (size_t)4 * BM * SK_LDT * 4;
  if (lds < red) lds = red;
  static bool attr_set = false;                            // per template instance
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)gemm_skinny_kernel<WM, AMODE>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, SK_LDS_MAX);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  gemm_skinny_kernel<WM, AMODE><<<n_tiles * splits, 256, lds, s>>>(x, n_tiles, splits, sps, lds_stride);
  return hipGetLastError();
}

}  // namespace

bool skinny_supported(const SkinnyArgs& x) {
  const GemmArgs& a = x.g;
  if (a.M < 1 || a.M > 64 || a.N % 32 != 0 || a.K % 64 != 0) return false;
  if (a.epi == EPI_SWIGLU) return false;
  if (x.a_mode == SK_A_NORM && (a.K % 256 != 0 || a.K > 256 * SK_NV)) return false;
  if (x.zero_ptr != nullptr && x.zero_n % 4 != 0) return false;
  return true;
}

hipError_t launch_gemm_skinny(hipStream_t s, const SkinnyArgs& x) {
  const GemmArgs& a = x.g;
  if (!skinny_supported(x)) return hipErrorInvalidValue;
  const int WM = a.M <= 32 ? 1 : 2;
  const int BM = 32 * WM;
  const int n_tiles = a.N / 32;
  const int kb16 = a.K / 16;
  const bool can_split = (a.epi == EPI_RESID || a.epi == EPI_GATE_RESID);
  // K splits until the grid covers the chip; a split is at least 4 k-steps (one per wave)
  int splits = 1;
  if (x.force_splits > 0) splits = x.force_splits;
  else if (can_split && n_tiles < 256) splits = (256 + n_tiles - 1) / n_tiles;
  if (!can_split) splits = 1;
  // the activation slice of a workgroup must fit in LDS
  const int sps_cap = ((SK_LDS_MAX - BM * 8) / (BM * 2) - 8) / 16 / 4 * 4;
  int sps = (kb16 + splits - 1) / splits;
  sps = (sps + 3) & ~3;
  if (sps > sps_cap) {
    if (!can_split) return hipErrorInvalidValue;           // callers check skinny_fits() first
    sps = sps_cap;
  }
  splits = (kb16 + sps - 1) / sps;
#define FARD_SK(WMV)                                                                          \
  switch (x.a_mode) {                                                                         \
    case SK_A_BF16: return launch_skinny_t<WMV, SK_A_BF16>(s, x, n_tiles, splits, sps);       \
    case SK_A_ACT: return launch_skinny_t<WMV, SK_A_ACT>(s, x, n_tiles, splits, sps);         \
    case SK_A_NORM: return launch_skinny_t<WMV, SK_A_NORM>(s, x, n_tiles, splits, sps);       \
    default: return hipErrorInvalidValue;                                                     \
  }
  if (WM == 1) { FARD_SK(1) }
  FARD_SK(2)
#undef FARD_SK
}

bool narrow_supported(const GemmArgs& a) {
  return a.M >= 1 && a.N % 32 == 0 && a.K % 64 == 0 && a.epi != EPI_SWIGLU;
}

hipError_t launch_gemm_narrow(hipStream_t s, const GemmArgs& a) {
  if (!narrow_supported(a)) return hipErrorInvalidValue;
  const bool oneshot = (a.K / 32 + 3) / 4 <= SK_P;
  // rows beyond one workgroup's tile go to further workgroups (blockIdx.y) that re-read the weight columns
  // out of L2: ids of one column tile differ by a multiple of 8, so they share an XCD when N % 128 == 0
#define FARD_NR(MTV)                                                                  \
  do {                                                                                \
    const dim3 grid(a.N / 16, (a.M + 16 * MTV - 1) / (16 * MTV));                     \
    if (oneshot) gemm_narrow_kernel<MTV, true><<<grid, 256, 0, s>>>(a);               \
    else gemm_narrow_kernel<MTV, false><<<grid, 256, 0, s>>>(a);                      \
  } while (0)
  if (a.M <= 16) FARD_NR(1);
  else if (a.M <= 32 || a.M > 64) FARD_NR(2);
  else FARD_NR(4);
#undef FARD_NR
  return hipGetLastError();
}

bool skinny_fits(const SkinnyArgs& x) {
  if (!skinny_supported(x)) return false;
  const GemmArgs& a = x.g;
  const bool can_split = (a.epi == EPI_RESID || a.epi == EPI_GATE_RESID);
  if (can_split) return true;
  const int BM = a.M <= 32 ? 32 : 64;
  const int sps_cap = ((SK_LDS_MAX - BM * 8) / (BM * 2) - 8) / 16 / 4 * 4;
  return ((a.K / 16 + 3) & ~3) <= sps_cap;
}

}  // namespace fard

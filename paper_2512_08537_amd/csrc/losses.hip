// Training-side losses of the draft model: the attention-entropy loss L_entropy (Sec. 3; S2.1) with its gradients
// with respect to the queries and keys of the layer it is taken on, and the Smooth-L1 feature regression loss.
//
// L_entropy = -(1 / (B N R)) sum_{b,h,r} H_{b,h,r},  H_r = -sum_c Omega_{r,c} ln Omega_{r,c},
// Omega_r = softmax over the causal row r of s_{r,c} = q_r . k_c / sqrt(d_head) (c <= r).
// dL/ds_{r,c} = Omega_{r,c} (ln Omega_{r,c} + H_r) / (B N R); dq_r = sum_c dL/ds k_c / sqrt(d); dk_c = sum_r dL/ds q_r / sqrt(d).
//
// Three passes over 32 x 32 score tiles, none of which writes a score to memory (v_mfma_f32_32x32x16_bf16):
//  1. row statistics: a wave owns 32 queries of one head and walks the key blocks up to the diagonal with a running
//     (max, sum e^t, sum e^t t); it leaves ln sum exp and H per row;
//  2. dq: the same walk; the tile of dL/ds is rebuilt from the statistics and multiplied with the keys;
//  3. dk: a wave owns 32 keys of one kv head and walks the query blocks from the diagonal on, over every query head
//     of its group; dL/ds is rebuilt with queries and keys in swapped roles and multiplied with the queries.
// No atomics: every output element has one owner.
//
// Layouts.  The score tile comes out of the MFMA with one operand's 32 rows spread over (register, lane half): register
// e of lane half hh holds MFMA row 8 (e / 4) + 4 hh + e % 4.  The rows of that operand are loaded in a permuted
// order (bits 2 and 3 of the row index swapped), so that register e of half hh holds logical index
// 16 (e / 8) + 8 hh + e % 8: registers 8 t .. 8 t + 7 are then, as they stand, the operand fragment of k-step t of
// the second product (lane -> row lane % 32, eight consecutive contraction indices starting at 16 t + 8 hh).  The
// other operand of the second product needs eight consecutive keys (queries) for one feature index: it is read from
// transposed copies [d_head][R] of k and q, which a small kernel writes first.
#include "kernels.h"

namespace fard {

namespace {

__device__ __forceinline__ int perm32(int i) { return (i & ~12) | ((i & 4) << 1) | ((i & 8) >> 1); }

// running (m, l, a): l = sum e^{s - m}, a = sum e^{s - m} (s - m)
struct Stat {
  float m, l, a;
};
__device__ __forceinline__ void stat_raise(Stat& s, float m_new) {
  if (m_new > s.m) {
    if (s.l > 0.f) {
      const float d = m_new - s.m, f = __expf(-d);
      s.a = (s.a - d * s.l) * f;
      s.l *= f;
    }
    s.m = m_new;
  }
}
__device__ __forceinline__ void stat_merge(Stat& s, const Stat& o) {
  if (o.l <= 0.f) return;
  Stat t = o;
  const float m = fmaxf(s.m, t.m);
  stat_raise(s, m);
  stat_raise(t, m);
  s.l += t.l;
  s.a += t.a;
}

// in [n][R][dh] -> out [n][dh][Rp], zero beyond R.  32 x 32 tiles through LDS.
__global__ __launch_bounds__(256) void transpose_kernel(const bf16* __restrict__ in, bf16* __restrict__ out, int R, int Rp, int dh) {
  __shared__ bf16 tile[32][33];
  const int n = blockIdx.z, r0 = blockIdx.x * 32, d0 = blockIdx.y * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  for (int i = ty; i < 32; i += 8) {
    const int r = r0 + i;
    tile[i][tx] = (r < R) ? in[((size_t)n * R + r) * dh + d0 + tx] : (bf16)0.f;
  }
  __syncthreads();
  for (int i = ty; i < 32; i += 8) out[((size_t)n * dh + d0 + i) * Rp + r0 + tx] = tile[tx][i];
}

template <int DH>
struct Frag {
  bf16x8 f[DH / 16];
};

// rows of a [R][DH] matrix as MFMA operand: lane -> row `row` (clamped), k-slots 16 s + 8 hh
template <int DH>
__device__ __forceinline__ void load_rows(Frag<DH>& fr, const bf16* __restrict__ base, int row, int R, int hh) {
  const int rr = row < R ? row : R - 1;
  const bf16* p = base + (size_t)rr * DH + 8 * hh;
#pragma unroll
  for (int s = 0; s < DH / 16; ++s) fr.f[s] = *(const bf16x8*)(p + 16 * s);
}

template <int DH>
__device__ __forceinline__ f32x16 score_tile(const Frag<DH>& rows, const Frag<DH>& cols) {
  f32x16 acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
#pragma unroll
  for (int s = 0; s < DH / 16; ++s) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rows.f[s], cols.f[s], acc, 0, 0, 0);
  return acc;
}

// ---- pass 1: row statistics.  One wave per (b, h, 32 queries); queries are the MFMA columns.
template <int DH>
__global__ __launch_bounds__(256) void ent_stats_kernel(const bf16* __restrict__ q, const bf16* __restrict__ k, int H, int Hkv, int R,
                                                        int Rp, int n_waves, float scale, float* __restrict__ lse,
                                                        float* __restrict__ hrow) {
  const int wid = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (wid >= n_waves) return;
  const int lane = threadIdx.x & 63, c = lane & 31, hh = lane >> 5;
  const int nqb = Rp >> 5, qb = wid % nqb, bh = wid / nqb;
  const int b = bh / H, h = bh - b * H, bkv = b * Hkv + h / (H / Hkv);
  const int query = qb * 32 + c;
  Frag<DH> qf, kf;
  load_rows<DH>(qf, q + (size_t)bh * R * DH, query, R, hh);
  Stat st{-INFINITY, 0.f, 0.f};
  const bf16* kb_base = k + (size_t)bkv * R * DH;
  for (int kb = 0; kb <= qb; ++kb) {
    load_rows<DH>(kf, kb_base, kb * 32 + perm32(c), R, hh);
    const f32x16 acc = score_tile<DH>(kf, qf);
    float sv[16], mx = -INFINITY;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int key = kb * 32 + 16 * (e >> 3) + 8 * hh + (e & 7);
      sv[e] = (key <= query && key < R) ? acc[e] * scale : -INFINITY;
      mx = fmaxf(mx, sv[e]);
    }
    if (mx > -INFINITY) {
      stat_raise(st, mx);
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        if (sv[e] > -INFINITY) {
          const float t = sv[e] - st.m, ex = __expf(t);
          st.l += ex;
          st.a = fmaf(ex, t, st.a);
        }
      }
    }
  }
  Stat o;
  o.m = other_half(st.m);
  o.l = other_half(st.l);
  o.a = other_half(st.a);
  stat_merge(st, o);
  if (hh == 0) {
    const float ll = __logf(st.l);
    lse[(size_t)bh * Rp + query] = st.m + ll;
    hrow[(size_t)bh * Rp + query] = (query < R) ? ll - st.a / st.l : 0.f;
  }
}

// dL/ds of one tile from its scores: reg e <-> (row-operand index idx_e, column-operand index of the lane).
// QUERY_IN_REGS: the registers run over queries (pass 3), else over keys (pass 2).
template <bool QUERY_IN_REGS>
__device__ __forceinline__ void grad_tile(const f32x16& acc, int reg_base, int lane_idx, int hh, int R, float scale, float cc,
                                          const float* __restrict__ lse, const float* __restrict__ hrow, bf16x8 (&g)[2]) {
  float lq[16], hq[16];
  if constexpr (QUERY_IN_REGS) {
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int q0 = reg_base + 16 * t + 8 * hh;
      const f32x4 l0 = *(const f32x4*)(lse + q0), l1 = *(const f32x4*)(lse + q0 + 4);
      const f32x4 h0 = *(const f32x4*)(hrow + q0), h1 = *(const f32x4*)(hrow + q0 + 4);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        lq[8 * t + j] = l0[j]; lq[8 * t + 4 + j] = l1[j];
        hq[8 * t + j] = h0[j]; hq[8 * t + 4 + j] = h1[j];
      }
    }
  } else {
    const float l = lse[lane_idx], hv = hrow[lane_idx];
#pragma unroll
    for (int e = 0; e < 16; ++e) { lq[e] = l; hq[e] = hv; }
  }
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    const int ridx = reg_base + 16 * (e >> 3) + 8 * hh + (e & 7);
    const int key = QUERY_IN_REGS ? lane_idx : ridx, query = QUERY_IN_REGS ? ridx : lane_idx;
    float gv = 0.f;
    if (key <= query && query < R) {
      const float lnp = acc[e] * scale - lq[e];
      gv = cc * __expf(lnp) * (lnp + hq[e]);
    }
    g[e >> 3][e & 7] = (bf16)gv;
  }
}

// ---- pass 2: dq.  One wave per (b, h, 32 queries).
template <int DH>
__global__ __launch_bounds__(256) void ent_dq_kernel(const bf16* __restrict__ q, const bf16* __restrict__ k, const bf16* __restrict__ kT,
                                                     int H, int Hkv, int R, int Rp, int n_waves, float scale, float cc,
                                                     const float* __restrict__ lse, const float* __restrict__ hrow,
                                                     float* __restrict__ dq) {
  const int wid = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (wid >= n_waves) return;
  const int lane = threadIdx.x & 63, c = lane & 31, hh = lane >> 5;
  const int nqb = Rp >> 5, qb = wid % nqb, bh = wid / nqb;
  const int b = bh / H, h = bh - b * H, bkv = b * Hkv + h / (H / Hkv);
  const int query = qb * 32 + c;
  Frag<DH> qf, kf;
  load_rows<DH>(qf, q + (size_t)bh * R * DH, query, R, hh);
  f32x16 out[DH / 32];
#pragma unroll
  for (int d = 0; d < DH / 32; ++d)
#pragma unroll
    for (int e = 0; e < 16; ++e) out[d][e] = 0.f;
  const bf16* kb_base = k + (size_t)bkv * R * DH;
  const bf16* kT_base = kT + (size_t)bkv * DH * Rp;
  const float* lse_b = lse + (size_t)bh * Rp;
  const float* h_b = hrow + (size_t)bh * Rp;
  for (int kb = 0; kb <= qb; ++kb) {
    load_rows<DH>(kf, kb_base, kb * 32 + perm32(c), R, hh);
    const f32x16 acc = score_tile<DH>(kf, qf);
    bf16x8 g[2];
    grad_tile<false>(acc, kb * 32, query, hh, R, scale, cc, lse_b, h_b, g);
    // dq[query, d] += sum_key g[key, query] k[key, d]: rows = queries (the lanes), contraction = keys (the registers)
#pragma unroll
    for (int d = 0; d < DH / 32; ++d)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const bf16x8 kt = *(const bf16x8*)(kT_base + (size_t)(32 * d + c) * Rp + kb * 32 + 16 * t + 8 * hh);
        out[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(g[t], kt, out[d], 0, 0, 0);
      }
  }
  float* dq_b = dq + (size_t)bh * R * DH;
#pragma unroll
  for (int d = 0; d < DH / 32; ++d)
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int row = qb * 32 + 8 * (e >> 2) + 4 * hh + (e & 3);
      if (row < R) dq_b[(size_t)row * DH + 32 * d + c] = out[d][e];
    }
}

// ---- pass 3: dk.  One wave per (b, kv head, 32 keys); keys are the MFMA columns of the score tile.
template <int DH>
__global__ __launch_bounds__(256) void ent_dk_kernel(const bf16* __restrict__ q, const bf16* __restrict__ k, const bf16* __restrict__ qT,
                                                     int H, int Hkv, int R, int Rp, int n_waves, float scale, float cc,
                                                     const float* __restrict__ lse, const float* __restrict__ hrow,
                                                     float* __restrict__ dk) {
  const int wid = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (wid >= n_waves) return;
  const int lane = threadIdx.x & 63, c = lane & 31, hh = lane >> 5;
  const int nkb = Rp >> 5, kb = wid % nkb, bkv = wid / nkb;
  const int b = bkv / Hkv, hkv = bkv - b * Hkv, G = H / Hkv;
  const int key = kb * 32 + c;
  Frag<DH> qf, kf;
  load_rows<DH>(kf, k + (size_t)bkv * R * DH, key, R, hh);
  f32x16 out[DH / 32];
#pragma unroll
  for (int d = 0; d < DH / 32; ++d)
#pragma unroll
    for (int e = 0; e < 16; ++e) out[d][e] = 0.f;
  for (int gi = 0; gi < G; ++gi) {
    const int bh = b * H + hkv * G + gi;
    const bf16* q_b = q + (size_t)bh * R * DH;
    const bf16* qT_b = qT + (size_t)bh * DH * Rp;
    const float* lse_b = lse + (size_t)bh * Rp;
    const float* h_b = hrow + (size_t)bh * Rp;
    for (int qb = kb; qb < nkb; ++qb) {
      load_rows<DH>(qf, q_b, qb * 32 + perm32(c), R, hh);
      const f32x16 acc = score_tile<DH>(qf, kf);
      bf16x8 g[2];
      grad_tile<true>(acc, qb * 32, key, hh, R, scale, cc, lse_b, h_b, g);
      // dk[key, d] += sum_query g[query, key] q[query, d]: rows = keys (the lanes), contraction = queries
#pragma unroll
      for (int d = 0; d < DH / 32; ++d)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const bf16x8 qt = *(const bf16x8*)(qT_b + (size_t)(32 * d + c) * Rp + qb * 32 + 16 * t + 8 * hh);
          out[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(g[t], qt, out[d], 0, 0, 0);
        }
    }
  }
  float* dk_b = dk + (size_t)bkv * R * DH;
#pragma unroll
  for (int d = 0; d < DH / 32; ++d)
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int row = kb * 32 + 8 * (e >> 2) + 4 * hh + (e & 3);
      if (row < R) dk_b[(size_t)row * DH + 32 * d + c] = out[d][e];
    }
}

// partial[blk] = sum of hrow over this workgroup's share of the valid rows (fixed order); optionally copies the valid
// rows to h_out [BH, R].  sum_partials_kernel turns the partial sums into the loss.
__global__ __launch_bounds__(256) void ent_loss_kernel(const float* __restrict__ hrow, int BH, int R, int Rp,
                                                       float* __restrict__ partial, float* __restrict__ h_out) {
  __shared__ float part[4];
  float s = 0.f;
  const long n = (long)BH * R;
  for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long)gridDim.x * 256) {
    const long bh = i / R, r = i - bh * R;
    const float v = hrow[bh * Rp + r];
    if (h_out) h_out[i] = v;
    s += v;
  }
  s = wave_sum(s);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) partial[blockIdx.x] = part[0] + part[1] + part[2] + part[3];
}

// Smooth-L1: per-workgroup partial sums (fixed order), gradient per element.
template <typename T>
__global__ __launch_bounds__(256) void smooth_l1_kernel(const T* __restrict__ pred, const T* __restrict__ target, long n, float beta,
                                                        float* __restrict__ partial, float* __restrict__ dpred) {
  __shared__ float part[4];
  float s = 0.f;
  const float inv_n = 1.0f / (float)n;
  for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long)gridDim.x * 256) {
    const float d = to_f32(pred[i]) - to_f32(target[i]), a = fabsf(d);
    const bool quad = a < beta;
    s += quad ? 0.5f * d * d / beta : a - 0.5f * beta;
    if (dpred) dpred[i] = (quad ? d / beta : copysignf(1.0f, d)) * inv_n;
  }
  s = wave_sum(s);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) partial[blockIdx.x] = part[0] + part[1] + part[2] + part[3];
}
__global__ __launch_bounds__(64) void sum_partials_kernel(const float* __restrict__ partial, int n_part, float inv_n, float* __restrict__ loss) {
  float s = 0.f;
  for (int i = threadIdx.x; i < n_part; i += 64) s += partial[i];
  s = wave_sum(s);
  if (threadIdx.x == 0) *loss = s * inv_n;
}

template <int DH>
hipError_t entropy_loss_t(hipStream_t s, const bf16* q, const bf16* k, int B, int H, int Hkv, int R, void* scratch, float* loss,
                          float* h_rows, float* dq, float* dk) {
  const int Rp = (R + 31) & ~31, nb = Rp >> 5;
  const EntLossScratch lay = entropy_loss_scratch(B, H, Hkv, R, DH);
  char* base = (char*)scratch;
  bf16* qT = (bf16*)(base + lay.qT);
  bf16* kT = (bf16*)(base + lay.kT);
  float* lse = (float*)(base + lay.lse);
  float* hrow = (float*)(base + lay.hrow);
  const float scale = 1.0f / sqrtf((float)DH);
  const float cc = scale / ((float)B * (float)H * (float)R);
  const int wq = B * H * nb, wk = B * Hkv * nb;
  ent_stats_kernel<DH><<<(wq + 3) / 4, 256, 0, s>>>(q, k, H, Hkv, R, Rp, wq, scale, lse, hrow);
  float* partial = (float*)(base + lay.partial);
  const long n_rows = (long)B * H * R;
  const int n_part = (int)((n_rows + 1023) / 1024 < ENT_LOSS_PARTS ? (n_rows + 1023) / 1024 : ENT_LOSS_PARTS);
  ent_loss_kernel<<<n_part, 256, 0, s>>>(hrow, B * H, R, Rp, partial, h_rows);
  sum_partials_kernel<<<1, 64, 0, s>>>(partial, n_part, -1.0f / (float)n_rows, loss);
  if (dq) {
    transpose_kernel<<<dim3(nb, DH / 32, B * Hkv), 256, 0, s>>>(k, kT, R, Rp, DH);
    ent_dq_kernel<DH><<<(wq + 3) / 4, 256, 0, s>>>(q, k, kT, H, Hkv, R, Rp, wq, scale, cc, lse, hrow, dq);
  }
  if (dk) {
    transpose_kernel<<<dim3(nb, DH / 32, B * H), 256, 0, s>>>(q, qT, R, Rp, DH);
    ent_dk_kernel<DH><<<(wk + 3) / 4, 256, 0, s>>>(q, k, qT, H, Hkv, R, Rp, wk, scale, cc, lse, hrow, dk);
  }
  return hipGetLastError();
}

}  // namespace

EntLossScratch entropy_loss_scratch(int B, int H, int Hkv, int R, int dh) {
  const size_t Rp = (size_t)((R + 31) & ~31);
  EntLossScratch l;
  l.qT = 0;
  l.kT = l.qT + (size_t)B * H * dh * Rp * 2;
  l.lse = l.kT + (size_t)B * Hkv * dh * Rp * 2;
  l.hrow = l.lse + (size_t)B * H * Rp * 4;
  l.partial = l.hrow + (size_t)B * H * Rp * 4;
  l.bytes = l.partial + (size_t)ENT_LOSS_PARTS * 4;
  return l;
}

hipError_t launch_entropy_loss(hipStream_t s, const void* q, const void* k, int B, int H, int Hkv, int R, int dh, void* scratch,
                               float* loss, float* h_rows, float* dq, float* dk) {
  if (B < 1 || H < 1 || Hkv < 1 || H % Hkv != 0 || R < 1) return hipErrorInvalidValue;
  if (dh == 32) return entropy_loss_t<32>(s, (const bf16*)q, (const bf16*)k, B, H, Hkv, R, scratch, loss, h_rows, dq, dk);
  if (dh == 64) return entropy_loss_t<64>(s, (const bf16*)q, (const bf16*)k, B, H, Hkv, R, scratch, loss, h_rows, dq, dk);
  if (dh == 128) return entropy_loss_t<128>(s, (const bf16*)q, (const bf16*)k, B, H, Hkv, R, scratch, loss, h_rows, dq, dk);
  return hipErrorInvalidValue;
}

hipError_t launch_smooth_l1(hipStream_t s, int is_bf16, const void* pred, const void* target, long n, float beta, float* partial,
                            int n_part, float* loss, float* dpred) {
  if (n < 1 || n_part < 1 || !(beta > 0.f)) return hipErrorInvalidValue;
  if (is_bf16) smooth_l1_kernel<bf16><<<n_part, 256, 0, s>>>((const bf16*)pred, (const bf16*)target, n, beta, partial, dpred);
  else smooth_l1_kernel<float><<<n_part, 256, 0, s>>>((const float*)pred, (const float*)target, n, beta, partial, dpred);
  sum_partials_kernel<<<1, 64, 0, s>>>(partial, n_part, 1.0f / (float)n, loss);
  return hipGetLastError();
}

}  // namespace fard

// KV-cached causal attention for the few query rows of a speculative block.
//
// bf16 path.  One workgroup of 4 waves per (sample, kv head); the waves take the 32-position
// blocks of the cache round-robin and merge their partial results through LDS at the end.
// The products are computed transposed so that nothing but Q passes through a layout change:
//   S^T = K Q^T    A operand = one K block (keys as rows) read as contiguous 1 KiB fragments,
//                  B operand = Q^T held in registers for the whole kernel;
//   O^T = V^T P^T  A operand = one V block (dims as rows, keys along k), B operand = P^T taken
//                  directly from the S^T accumulators (the cache stores V with its keys permuted
//                  to the accumulator order, see rowops.hip), so probabilities never leave registers.
// Every output column of both products is one query row, i.e. one lane pair (lane, lane+32):
// the running softmax triple (m, l, a) with a = sum e^{s-m}(s-m) lives in those lanes; the row
// entropy ln l - a/l of the attention distribution (Eq. 1 / S2.1 indicator) falls out for free.
// With grouped KV heads the G query heads of a KV head are packed into the columns (G*n_q <= 64).
//
// With learned positions (no RoPE) the kernel also appends the new rows' K and V to the cache, so a layer
// needs no separate append launch.
//
// fp32 path: one wave per (row, head), scores staged in LDS; for the small fp32 configuration.
#include "kernels.h"

#include <algorithm>

namespace fard {

namespace {

#ifndef ATTN_OCC
#define ATTN_OCC 4
#endif
#define ATTN_MIN_WG(DH, NQB) (((DH) == 64 && (NQB) == 1) ? ATTN_OCC : 1)

template <int DH, int NQB>
__global__ __launch_bounds__(256, ATTN_MIN_WG(DH, NQB)) void attn_bf16_kernel(const bf16* __restrict__ qkv, int ld, int n_heads, KvGeom kv,
                                                        const int* __restrict__ cache_len,
                                                        const int* __restrict__ row_start, const int* __restrict__ row_cnt,
                                                        bf16* __restrict__ out, int ldo, float* __restrict__ ent_heads,
                                                        int append, int pass_stride, AttnSplit sp, int out_tiled) {
  constexpr int DC = DH / 16;      // k16 chunks of the head dim (QK^T)
  constexpr int DB = DH / 32;      // 32-dim row blocks of O^T
  constexpr int NCOL = 32 * NQB;
  // merge area: one slab of partial O^T per wave (4 DH (NCOL + 1) floats of dynamic LDS: 17-133 KB), so that the
  // four waves meet behind one barrier; with one shared accumulator and a read-modify-write round per wave the merge was
  // 5.3 us of a 15.8 us launch at DH = 128 with 64 columns
  constexpr int OLD = NCOL + 1;                            // padded row: conflict-free column-major reads
  __shared__ float s_m[4][NCOL], s_l[4][NCOL], s_a[4][NCOL];
  extern __shared__ __attribute__((aligned(16))) float s_o[];

  const int Hk = kv.n_kv_heads;
  const int G = n_heads / Hk;
  const int b = blockIdx.x / Hk, hk = blockIdx.x - b * Hk;
  // several passes in one launch (blockIdx.y; the longest, i.e. last, pass is dispatched first): the per-sample
  // arrays of pass p start p * pass_stride entries in
  const int pass_off = ((int)gridDim.y - 1 - (int)blockIdx.y) * pass_stride;
  cache_len += pass_off;
  row_start += pass_off;
  if (row_cnt) row_cnt += pass_off;
  const int r0 = row_start[b];
  const int nq = row_cnt ? row_cnt[b] : row_start[b + 1] - r0;     // (row_cnt: a pass over part of the sample's rows)
  if (nq <= 0) return;
  const int p0 = cache_len[b];
  const int ncols = nq * G;                       // column c <-> (query head hk*G + c / nq, row c % nq)
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int cl = lane & 31, g = lane >> 5;
  const float scale = rsqrtf((float)DH);

  // Q^T fragments: lane supplies column cl (+32*qb), dims 16*dc + 8*g .. +7
  bf16x8 qf[DC][NQB];
  int jrow[NQB];
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    const int c = cl + 32 * qb;
    const bool ok = c < ncols;
    const int gq = ok ? c / nq : 0;
    const int j = ok ? c - gq * nq : 0;
    jrow[qb] = ok ? j : -1;
    const bf16* qp = qkv + (size_t)(r0 + j) * ld + (size_t)(hk * G + gq) * DH + 8 * g;
#pragma unroll
    for (int dc = 0; dc < DC; ++dc) {
      bf16x8 v;
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = (bf16)0.f;
      if (ok) v = *(const bf16x8*)(qp + 16 * dc);
      qf[dc][qb] = v;
    }
  }

  const size_t head_elems = (size_t)kv.ctx_pad * DH;
  bf16* Kb = (bf16*)kv.k + ((size_t)b * Hk + hk) * head_elems;
  bf16* Vb = (bf16*)kv.v + ((size_t)b * Hk + hk) * head_elems;

  float m_run[NQB], l_run[NQB], a_run[NQB];
  f32x16 o[DB][NQB];
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    m_run[qb] = -INFINITY;
    l_run[qb] = 0.f;
    a_run[qb] = 0.f;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int e = 0; e < 16; ++e) o[db][qb][e] = 0.f;
  }

  const int n_keys = p0 + nq;
  const int n_blocks = (n_keys + 31) >> 5;
  // Blocks that hold only cached positions come first; with `append` the workgroup then stores the new rows'
  // K and V into the cache (it owns this sample's kv head) and reads the blocks that contain them afterwards.
  const int tail0 = append ? (p0 >> 5) : n_blocks;
  for (int phase = 0; phase < 2; ++phase) {
    if (phase == 1) {
      if (!append) break;
      const bf16* ksrc = qkv + (size_t)r0 * ld + (size_t)(n_heads + hk) * DH;
      const bf16* vsrc = ksrc + (size_t)Hk * DH;
      constexpr int D8 = DH / 8;
      for (int idx = tid; idx < nq * D8; idx += 256) {       // K: 8 dims of a key are contiguous in the cache
        const int j = idx / D8, d8 = idx - j * D8;
        *(bf16x8*)(Kb + k_offset_bf16(p0 + j, d8 * 8, DH)) = *(const bf16x8*)(ksrc + (size_t)j * ld + d8 * 8);
      }
      for (int idx = tid; idx < nq * DH; idx += 256) {       // V: keys are contiguous, dims are not
        const int j = idx / DH, d = idx - j * DH;
        Vb[v_offset_bf16(p0 + j, d, DH)] = vsrc[(size_t)j * ld + d];
      }
      __threadfence_block();
      __syncthreads();
    }
      int kb_lo = (phase == 0) ? 0 : tail0, kb_hi = (phase == 0) ? tail0 : n_blocks;
    if (sp.n > 1) {                                        // this workgroup's share of the key blocks (append == 0)
      kb_lo = (int)(((long)n_blocks * blockIdx.z) / sp.n);
      kb_hi = (int)(((long)n_blocks * (blockIdx.z + 1)) / sp.n);
    }
  for (int kb = kb_lo + wave; kb < kb_hi; kb += 4) {
    const bf16x8* kblk = (const bf16x8*)(Kb + (size_t)kb * 32 * DH);
    const bf16x8* vblk = (const bf16x8*)(Vb + (size_t)kb * 32 * DH);
    bf16x8 kf[DC];
#pragma unroll
    for (int dc = 0; dc < DC; ++dc) kf[dc] = kblk[dc * 64 + lane];
    bf16x8 vf[DB][2];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) vf[db][hf] = vblk[(db * 2 + hf) * 64 + lane];

#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      f32x16 s;
#pragma unroll
      for (int e = 0; e < 16; ++e) s[e] = 0.f;
#pragma unroll
      for (int dc = 0; dc < DC; ++dc) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[dc], qf[dc][qb], s, 0, 0, 0);
      // register e holds key 32*kb + 8*(e/4) + 4*g + e%4 for query column cl
      const int lim = (jrow[qb] >= 0) ? p0 + jrow[qb] : -1;     // last visible position
      float bmax = -INFINITY;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int key = kb * 32 + 8 * (e >> 2) + 4 * g + (e & 3);
        s[e] = (key <= lim) ? s[e] * scale : -INFINITY;
        bmax = fmaxf(bmax, s[e]);
      }
      bmax = xor32_max(bmax);
      const float m_new = fmaxf(m_run[qb], bmax);
      float psum = 0.f, asum = 0.f;
      bf16x8 pf[2];
      if (m_new == -INFINITY) {
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
          for (int i = 0; i < 8; ++i) pf[hf][i] = (bf16)0.f;
      } else {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const float t = s[e] - m_new;                       // -inf for masked keys
          const float p = (s[e] == -INFINITY) ? 0.f : __expf(t);
          psum += p;
          asum += (s[e] == -INFINITY) ? 0.f : p * t;
          pf[e >> 3][e & 7] = (bf16)p;
        }
        psum = xor32_sum(psum);
        asum = xor32_sum(asum);
        float corr = 1.f;
        if (m_run[qb] != -INFINITY) {
          const float dl = m_run[qb] - m_new;
          corr = __expf(dl);
          a_run[qb] = corr * (a_run[qb] + dl * l_run[qb]);
          l_run[qb] = corr * l_run[qb];
        }
        a_run[qb] += asum;
        l_run[qb] += psum;
        m_run[qb] = m_new;
        if (corr != 1.f) {
#pragma unroll
          for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[db][qb][e] *= corr;
        }
      }
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
          o[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[db][hf], pf[hf], o[db][qb], 0, 0, 0);
    }
  }
  }

  // ---- merge the four waves
  if (g == 0) {
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      s_m[wave][cl + 32 * qb] = m_run[qb];
      s_l[wave][cl + 32 * qb] = l_run[qb];
      s_a[wave][cl + 32 * qb] = a_run[qb];
    }
  }
  __syncthreads();
  float f_me[NQB];
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    const int c = cl + 32 * qb;
    float mstar = -INFINITY;
    for (int w = 0; w < 4; ++w) mstar = fmaxf(mstar, s_m[w][c]);
    f_me[qb] = (m_run[qb] == -INFINITY) ? 0.f : __expf(m_run[qb] - mstar);
  }
  // every wave lays its rescaled partial O^T down in its own slab: one barrier, no read-modify-write rounds
  float* slab = s_o + (size_t)wave * DH * OLD;
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int dim = 32 * db + 8 * (e >> 2) + 4 * g + (e & 3);   // O^T row
        slab[dim * OLD + cl + 32 * qb] = o[db][qb][e] * f_me[qb];
      }
  __syncthreads();
  // ---- normalise and write: thread -> (column, 8 consecutive dims)
  constexpr int D8 = DH / 8;
  for (int idx = tid; idx < NCOL * D8; idx += 256) {
    const int c = idx / D8, d8 = idx - c * D8;
    if (c >= ncols) continue;
    float mstar = -INFINITY;
    for (int w = 0; w < 4; ++w) mstar = fmaxf(mstar, s_m[w][c]);
    float lstar = 0.f, astar = 0.f;
    for (int w = 0; w < 4; ++w) {
      const float mw = s_m[w][c];
      if (mw == -INFINITY) continue;
      const float dl = mw - mstar, f = __expf(dl);
      lstar += f * s_l[w][c];
      astar += f * (s_a[w][c] + dl * s_l[w][c]);
    }
    const int gq = c / nq, j = c - gq * nq;
    const int head = hk * G + gq;
    if (sp.n > 1) {
      // keys split over workgroups: this one's running triple and unnormalised O row (relative to its own maximum)
      // go to the planes that attn_merge_kernel folds
      const size_t slot = ((size_t)blockIdx.z * sp.rows + (r0 + j)) * n_heads + head;
      f32x4 lo, hi;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        float acc = s_o[(d8 * 8 + i) * OLD + c];
#pragma unroll
        for (int w = 1; w < 4; ++w) acc += s_o[((size_t)w * DH + d8 * 8 + i) * OLD + c];
        if (i < 4) lo[i] = acc; else hi[i - 4] = acc;
      }
      *(f32x4*)(sp.o + slot * DH + d8 * 8) = lo;
      *(f32x4*)(sp.o + slot * DH + d8 * 8 + 4) = hi;
      if (d8 == 0) *(f32x4*)(sp.mla + slot * 4) = f32x4{mstar, lstar, astar, 0.f};
      continue;
    }
    const float inv = 1.0f / lstar;
    bf16x8 v;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float acc = s_o[(d8 * 8 + i) * OLD + c];
#pragma unroll
      for (int w = 1; w < 4; ++w) acc += s_o[((size_t)w * DH + d8 * 8 + i) * OLD + c];
      v[i] = (bf16)(acc * inv);
    }
    // (out_tiled: the rows in the tile order the output projection's narrow-tile GEMM reads; 8 dims are one piece)
    *(bf16x8*)(out + (out_tiled ? tile_offset(r0 + j, head * DH + d8 * 8, ldo) : (size_t)(r0 + j) * ldo + (size_t)head * DH + d8 * 8)) = v;
    if (ent_heads != nullptr && d8 == 0) ent_heads[(size_t)(r0 + j) * n_heads + head] = logf(lstar) - astar * inv;
  }
}

// Folds the per-split results of attn_bf16_kernel: thread -> (row, head, 8 dims).
__global__ __launch_bounds__(256) void attn_merge_kernel(AttnSplit sp, int n_heads, int dh, int M, const int* __restrict__ m_dev,
                                                         bf16* __restrict__ out, int ldo, float* __restrict__ ent_heads,
                                                         int out_tiled) {
  const int Me = eff_rows(M, m_dev);
  const int d8n = dh >> 3;
  const long total = (long)Me * n_heads * d8n;
  for (long idx = (long)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (long)gridDim.x * 256) {
    const int d8 = (int)(idx % d8n);
    const long rh = idx / d8n;                             // row * n_heads + head
    // every split's triple and output piece are requested before the first is used (split by split the kernel waited
    // for memory once per split)
    constexpr int NS = 8;                                  // sp.n <= 8 (checked at launch)
    f32x4 t[NS], lo[NS], hi[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const size_t slot = (size_t)(s < sp.n ? s : 0) * sp.rows * n_heads + rh;
      t[s] = *(const f32x4*)(sp.mla + slot * 4);
      lo[s] = *(const f32x4*)(sp.o + slot * dh + d8 * 8);
      hi[s] = *(const f32x4*)(sp.o + slot * dh + d8 * 8 + 4);
    }
    float mstar = -INFINITY;
#pragma unroll
    for (int s = 0; s < NS; ++s)
      if (s < sp.n) mstar = fmaxf(mstar, t[s][0]);
    float lstar = 0.f, astar = 0.f;
    float acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.f;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      if (s >= sp.n || t[s][0] == -INFINITY) continue;     // (a split that saw no visible key)
      const float dl = t[s][0] - mstar, f = __expf(dl);
      lstar += f * t[s][1];
      astar += f * (t[s][2] + dl * t[s][1]);
#pragma unroll
      for (int i = 0; i < 4; ++i) { acc[i] += f * lo[s][i]; acc[4 + i] += f * hi[s][i]; }
    }
    const float inv = 1.0f / lstar;
    const int row = (int)(rh / n_heads), head = (int)(rh - (long)row * n_heads);
    bf16x8 v;
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = (bf16)(acc[i] * inv);
    *(bf16x8*)(out + (out_tiled ? tile_offset(row, head * dh + d8 * 8, ldo) : (size_t)row * ldo + (size_t)head * dh + d8 * 8)) = v;
    if (ent_heads != nullptr && d8 == 0) ent_heads[rh] = logf(lstar) - astar * inv;
  }
}

// fp32 path: one wave per (row, head).
__global__ __launch_bounds__(64) void attn_f32_kernel(const float* __restrict__ qkv, int ld, int n_heads, KvGeom kv,
                                                      const int* __restrict__ cache_len,
                                                      const int* __restrict__ row_start, const int* __restrict__ row_cnt,
                                                      int B, float* __restrict__ out,
                                                      int ldo, float* __restrict__ ent_heads, int max_keys, int pass_stride) {
  extern __shared__ float s_p[];                 // [max_keys] scores / probabilities
  const int head = blockIdx.x, b = blockIdx.z % B, j = blockIdx.y;
  const int pass_off = ((int)blockIdx.z / B) * pass_stride;       // passes of one launch: blockIdx.z = pass * B + b
  cache_len += pass_off;
  row_start += pass_off;
  if (row_cnt) row_cnt += pass_off;
  const int r0 = row_start[b];
  const int nq = row_cnt ? row_cnt[b] : row_start[b + 1] - r0;
  if (j >= nq) return;
  const int Hk = kv.n_kv_heads, dh = kv.d_head;
  const int hk = (head * Hk) / n_heads;
  const int lane = threadIdx.x;
  const int vis = cache_len[b] + j + 1;
  const float* q = qkv + (size_t)(r0 + j) * ld + (size_t)head * dh;
  const float* Kc = (const float*)kv.k + ((size_t)b * Hk + hk) * (size_t)kv.ctx_pad * dh;
  const float* Vc = (const float*)kv.v + ((size_t)b * Hk + hk) * (size_t)kv.ctx_pad * dh;
  const float scale = 1.0f / sqrtf((float)dh);
  float mx = -INFINITY;
  for (int c = lane; c < vis; c += WAVE) {
    float s = 0.f;
    for (int d = 0; d < dh; ++d) s += q[d] * Kc[(size_t)c * dh + d];
    s *= scale;
    s_p[c] = s;
    mx = fmaxf(mx, s);
  }
  mx = wave_max(mx);
  float l = 0.f, a = 0.f;
  for (int c = lane; c < vis; c += WAVE) {
    const float t = s_p[c] - mx, e = expf(t);
    s_p[c] = e;
    l += e;
    a += e * t;
  }
  l = wave_sum(l);
  a = wave_sum(a);
  __syncthreads();
  const float inv = 1.0f / l;
  for (int d = lane; d < dh; d += WAVE) {
    float acc = 0.f;
    for (int c = 0; c < vis; ++c) acc += s_p[c] * Vc[(size_t)c * dh + d];
    out[(size_t)(r0 + j) * ldo + (size_t)head * dh + d] = acc * inv;
  }
  if (ent_heads != nullptr && lane == 0) ent_heads[(size_t)(r0 + j) * n_heads + head] = logf(l) - a * inv;
}

}  // namespace

hipError_t launch_attention(hipStream_t s, const void* qkv, int ld, int n_heads, KvGeom kv, const int* cache_len,
                            const int* row_start, int B, int nq_max, void* out, int ldo, float* ent_heads, int append,
                            const int* row_cnt, int n_pass, const AttnSplit* split, int M, const int* m_dev, int out_tiled) {
  if (B <= 0 || nq_max <= 0 || n_pass <= 0) return hipSuccess;
  // several passes at once read rows that an earlier pass of the same launch would have had to store
  if (n_pass > 1 && (append || row_cnt == nullptr || n_pass > 65535 || (long)B * n_pass > 65535)) return hipErrorInvalidValue;
  if (out_tiled && (!kv.is_bf16 || ldo % 32 != 0)) return hipErrorInvalidValue;
  if (!kv.is_bf16) {
    if (append) return hipErrorInvalidValue;
    dim3 grid(n_heads, nq_max, B * n_pass);
    const size_t smem = (size_t)kv.ctx_pad * sizeof(float);
    if (smem > 64 * 1024) return hipErrorInvalidValue;
    attn_f32_kernel<<<grid, 64, smem, s>>>((const float*)qkv, ld, n_heads, kv, cache_len, row_start, row_cnt, B, (float*)out,
                                           ldo, ent_heads, kv.ctx_pad, B);
    return hipGetLastError();
  }
  const int G = n_heads / kv.n_kv_heads;
  const int cols = G * nq_max;
  if (cols > 64 || n_heads % kv.n_kv_heads != 0) return hipErrorInvalidValue;
  AttnSplit sp{};
  sp.n = 1;
  if (split != nullptr && split->n > 1) {
    if (append || n_pass != 1 || split->o == nullptr || split->mla == nullptr || M > split->rows || M < 1 || split->n > 8)
      return hipErrorInvalidValue;                          // (the merge kernel holds at most 8 splits in registers)
    sp = *split;
  }
  const dim3 grid(B * kv.n_kv_heads, n_pass, sp.n);
  const int ps = B;
  const bf16* q = (const bf16*)qkv;
  bf16* o = (bf16*)out;
  float* eh = sp.n > 1 ? nullptr : ent_heads;              // with split keys the merge writes the entropies
#define FARD_ATT(DHV, NQBV)                                                                                          \
  do {                                                                                                               \
    constexpr int lds = 4 * DHV * (32 * NQBV + 1) * 4;     /* the four waves' slabs of partial O^T */                 \
    if constexpr (lds > 64 * 1024) {                                                                                 \
      static bool attr_set = false;                                                                                  \
      if (!attr_set) {                                                                                               \
        hipError_t e = hipFuncSetAttribute((const void*)attn_bf16_kernel<DHV, NQBV>,                                 \
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds);                         \
        if (e != hipSuccess) return e;                                                                               \
        attr_set = true;                                                                                             \
      }                                                                                                              \
    }                                                                                                                \
    attn_bf16_kernel<DHV, NQBV><<<grid, 256, lds, s>>>(q, ld, n_heads, kv, cache_len, row_start, row_cnt, o, ldo, eh, \
                                                       append, ps, sp, out_tiled);                                   \
  } while (0)
  if (kv.d_head == 64) {
    if (cols <= 32) FARD_ATT(64, 1); else FARD_ATT(64, 2);
  } else if (kv.d_head == 128) {
    if (cols <= 32) FARD_ATT(128, 1); else FARD_ATT(128, 2);
  } else if (kv.d_head == 32) {
    if (cols <= 32) FARD_ATT(32, 1); else FARD_ATT(32, 2);
  } else {
    return hipErrorInvalidValue;
  }
#undef FARD_ATT
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || sp.n <= 1) return e;
  const long total = (long)M * n_heads * (kv.d_head / 8);
  const unsigned blocks = (unsigned)std::min<long>((total + 255) / 256, 2048);
  attn_merge_kernel<<<blocks, 256, 0, s>>>(sp, n_heads, kv.d_head, M, m_dev, o, ldo, ent_heads, out_tiled);
  return hipGetLastError();
}

}  // namespace fard

// Row-wise kernels around the GEMMs: row maps, embedding, norms, RoPE + KV append, entropy
// pre-filter, head sampler pieces, accept test.  Memory-bound or tiny; one wave or one
// workgroup per row, fp32 arithmetic, vector loads where rows are long.
#include "kernels.h"
#include <type_traits>

namespace fard {

namespace {

// ================================================================== row maps
__global__ __launch_bounds__(256) void build_rows_kernel(const int* n_base, int add, int B, int K, int D,
                                                         const int* cache_len, RowMaps maps,
                                                         const float* x_first, const float* x_rest,
                                                         float* x_out, int* aux_row, int m_max, int nq_cap) {
  __shared__ int s_scan[256];
  __shared__ int s_len[256];
  __shared__ int s_carry;
  const int tid = threadIdx.x;
  if (tid == 0) s_carry = 0;
  __syncthreads();
  for (int base = 0; base < B; base += 256) {
    const int b = base + tid;
    int nq = 0;
    if (b < B) {
      nq = (n_base ? n_base[b] : 0) + add;
      if (nq < 0) nq = 0;
      if (nq > nq_cap) nq = nq_cap;
    }
    s_scan[tid] = nq;
    __syncthreads();
    for (int o = 1; o < 256; o <<= 1) {          // inclusive Hillis-Steele scan
      int v = (tid >= o) ? s_scan[tid - o] : 0;
      __syncthreads();
      s_scan[tid] += v;
      __syncthreads();
    }
    const int carry = s_carry;
    const int start = carry + s_scan[tid] - nq;
    if (b < B) {
      maps.row_start[b] = start < m_max ? start : m_max;
      s_len[tid] = cache_len[b];
    }
    __syncthreads();
    // the rows of these 256 samples, dealt to the threads: row -> sample by bisection of the inclusive scan
    const int block_total = s_scan[255];
    auto sample_of = [&](int rl, int& jj) {
      int lo = 0, hi = 255;                        // smallest i with s_scan[i] > rl
      while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (s_scan[mid] > rl) hi = mid; else lo = mid + 1;
      }
      jj = rl - (lo ? s_scan[lo - 1] : 0);
      return lo;
    };
    for (int rl = tid; rl < block_total; rl += 256) {
      const int r = carry + rl;
      if (r >= m_max) break;
      int jj;
      const int i = sample_of(rl, jj);
      maps.row_sample[r] = base + i;
      maps.row_j[r] = jj;
      maps.row_pos[r] = s_len[i] + jj;
      if (aux_row) aux_row[r] = (base + i) * (K + 1) + jj;
    }
    if (x_out) {
      const bool vec4 = (D & 3) == 0 && ((((uintptr_t)x_first) | ((uintptr_t)x_rest) | ((uintptr_t)x_out)) & 15) == 0;
      if (vec4) {
        // 16-byte pieces, four of a thread's loads in flight at once (the rows are a few dozen bytes each)
        const int D4 = D >> 2, n4 = block_total * D4;
        for (int e0 = tid; e0 < n4; e0 += 4 * 256) {
          f32x4 v[4];
          size_t dst[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int e = e0 + u * 256;
            dst[u] = (size_t)-1;
            if (e < n4) {
              const int rl = e / D4, cc = e - rl * D4;
              const int r = carry + rl;
              if (r < m_max) {
                int jj;
                const int i = sample_of(rl, jj);
                const float* src = (jj == 0) ? x_first + (size_t)(base + i) * D : x_rest + ((size_t)(base + i) * K + (jj - 1)) * D;
                v[u] = *(const f32x4*)(src + 4 * cc);
                dst[u] = (size_t)r * D + 4 * cc;
              }
            }
          }
#pragma unroll
          for (int u = 0; u < 4; ++u)
            if (dst[u] != (size_t)-1) *(f32x4*)(x_out + dst[u]) = v[u];
        }
      } else {
        for (int e = tid; e < block_total * D; e += 256) {
          const int rl = e / D, cc = e - rl * D;
          const int r = carry + rl;
          if (r >= m_max) break;
          int jj;
          const int i = sample_of(rl, jj);
          const float* src = (jj == 0) ? x_first + (size_t)(base + i) * D : x_rest + ((size_t)(base + i) * K + (jj - 1)) * D;
          x_out[(size_t)r * D + cc] = src[cc];
        }
      }
    }
    __syncthreads();
    if (tid == 255) s_carry = carry + s_scan[255];
    __syncthreads();
  }
  if (tid == 0) {
    int total = s_carry;
    if (total > m_max) total = m_max;
    maps.row_start[B] = total;
    *maps.m_total = total;
  }
}

// ================================================================== embedding
// v + sum_k xv[k] * W[k, c] for a projection from D latent components (W [D, ld] row-major).  For D <= 16 every
// weight and input load is issued before the first use: the sum is one memory round trip, not D.
template <typename T, typename XP>
__device__ __forceinline__ float in_proj(float v, XP xv, float xscale, int D, const T* __restrict__ W, int ld, int c) {
  if (D <= 16) {
    float wv[16], xr[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      const int kk = k < D ? k : 0;
      wv[k] = to_f32(W[(size_t)kk * ld + c]);
      xr[k] = xv[kk];
    }
#pragma unroll
    for (int k = 0; k < 16; ++k) v += (k < D) ? (xr[k] * xscale) * wv[k] : 0.f;
    return v;
  }
  for (int k = 0; k < D; ++k) v += (xv[k] * xscale) * to_f32(W[(size_t)k * ld + c]);
  return v;
}

template <typename T>
__global__ __launch_bounds__(256) void embed_kernel(const float* __restrict__ x, int ldx, int D, const T* __restrict__ w_in,
                                                    const float* __restrict__ b_in, const T* __restrict__ pos_table,
                                                    const int* __restrict__ row_pos, const T* __restrict__ cond_table,
                                                    const int* __restrict__ cond_id, float* __restrict__ h, int d,
                                                    int M, const int* m_dev) {
  const int Me = eff_rows(M, m_dev);
  const int r = blockIdx.y;
  if (r >= Me) return;
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= d) return;
  float v;
  const int id = cond_id ? cond_id[r] : -1;
  if (id >= 0) {
    v = to_f32(cond_table[(size_t)id * d + c]);
  } else {
    const float pv = pos_table ? to_f32(pos_table[(size_t)row_pos[r] * d + c]) : 0.f;
    v = in_proj<T>(b_in ? b_in[c] : 0.f, x + (size_t)r * ldx, 1.0f, D, w_in, d, c) + pv;
  }
  h[(size_t)r * d + c] = v;
}

// ================================================================== norms
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) red[wave] = v;
  __syncthreads();
  float t = 0.f;
  const int nw = blockDim.x >> 6;
  for (int i = 0; i < nw; ++i) t += red[i];
  return t;
}

// both sums of a 256-thread workgroup in one round (two barriers)
__device__ __forceinline__ void block_sum2(float& a, float& b, float* red) {
  a = wave_sum(a);
  b = wave_sum(b);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) { red[wave] = a; red[4 + wave] = b; }
  __syncthreads();
  a = red[0] + red[1] + red[2] + red[3];
  b = red[4] + red[5] + red[6] + red[7];
}

// One workgroup per row.  The row is read once with 16-byte loads and stays in registers for the
// statistics and the output pass (d <= 256 * 4 * NORM_VPT); everything a thread needs is requested
// before the first reduction so that the loads overlap.
constexpr int NORM_VPT = 8;         // largest instance; the launcher picks the smallest VPT that covers d
template <typename T>
__device__ __forceinline__ void store4(T* p, float a, float b, float c, float d);
template <>
__device__ __forceinline__ void store4<float>(float* p, float a, float b, float c, float d) {
  *(f32x4*)p = f32x4{a, b, c, d};
}
template <>
__device__ __forceinline__ void store4<bf16>(bf16* p, float a, float b, float c, float d) {
  bf16x4 v;
  v[0] = (bf16)a; v[1] = (bf16)b; v[2] = (bf16)c; v[3] = (bf16)d;
  *(bf16x4*)p = v;
}

template <typename T, int VPT>
__global__ __launch_bounds__(256) void norm_kernel(const float* __restrict__ h, int d, int M, const int* m_dev,
                                                   int norm_type, float eps, const float* __restrict__ g,
                                                   const float* __restrict__ b, const float* __restrict__ shift,
                                                   const float* __restrict__ scale, int ldm,
                                                   const int* __restrict__ in_map, T* __restrict__ out,
                                                   const float* __restrict__ parts, int n_parts, size_t part_stride,
                                                   float* __restrict__ h_wb, int out_tiled) {
  __shared__ float red[8];
  const int Me = eff_rows(M, m_dev);
  const int r = blockIdx.x;
  if (r >= Me) return;
  const float* row = h + (size_t)(in_map ? in_map[r] : r) * d;
  const int n4 = d >> 2;                                   // d % 4 == 0 (checked on the host)
  f32x4 x[VPT];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < VPT; ++i) {
    const int c4 = threadIdx.x + i * 256;
    x[i] = (c4 < n4) ? ((const f32x4*)row)[c4] : f32x4{0.f, 0.f, 0.f, 0.f};
  }
  // the row's modulation (AdaLN) is requested with the row itself: one memory round trip instead of a second one after
  // the reduction
  f32x4 scv[VPT], shv[VPT];
  if (scale) {
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
      const int c4 = threadIdx.x + i * 256;
      const int cc = c4 < n4 ? c4 : 0;
      scv[i] = *(const f32x4*)(scale + (size_t)r * ldm + cc * 4);
      shv[i] = *(const f32x4*)(shift + (size_t)r * ldm + cc * 4);
    }
  }
  if (n_parts > 0) {
    // deferred residual update: the preceding GEMM left K-slice partial sums; fold them in (and write the row back).
    // Four planes at a time, all their loads requested before the first is added: plane by plane the kernel waited for
    // memory once per plane (10-14 us for a 5120-wide row with 5 planes).
    const size_t ro = (size_t)(in_map ? in_map[r] : r) * d;
    for (int p0 = 0; p0 < n_parts; p0 += 4) {
      f32x4 t[4][VPT];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int p = p0 + q < n_parts ? p0 + q : n_parts - 1;
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
          const int c4 = threadIdx.x + i * 256;
          t[q][i] = *(const f32x4*)(parts + (size_t)p * part_stride + ro + (c4 < n4 ? c4 : 0) * 4);
        }
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (p0 + q < n_parts) {
#pragma unroll
          for (int i = 0; i < VPT; ++i) x[i] += t[q][i];
        }
      }
    }
  }
  // one reduction round for both moments, taken about a pivot (the row's first element) so that
  // E[(x-p)^2] - E[x-p]^2 does not cancel for rows with a large mean
  const float pivot = row[0];
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < VPT; ++i) {
    const int c4 = threadIdx.x + i * 256;
    if (c4 < n4) {
#pragma unroll
      for (int e = 0; e < 4; ++e) { const float t = x[i][e] - pivot; s += t; q = fmaf(t, t, q); }
    }
  }
  block_sum2(s, q, red);
  if (n_parts > 0 && h_wb != nullptr) {
    // the completed row goes back only now: every thread has read the pivot (element 0 of the old row) before the
    // barriers of the reduction
    const size_t ro = (size_t)(in_map ? in_map[r] : r) * d;
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
      const int c4 = threadIdx.x + i * 256;
      if (c4 < n4) *(f32x4*)(h_wb + ro + c4 * 4) = x[i];
    }
  }
  const float m1 = s / (float)d, m2 = q / (float)d;
  const float mean = (norm_type == 0) ? pivot + m1 : 0.f;
  // RMS norm: E[x^2] = E[(x-p)^2] + 2 p E[x-p] + p^2
  const float var = (norm_type == 0) ? fmaxf(m2 - m1 * m1, 0.f) : fmaxf(m2 + 2.f * pivot * m1 + pivot * pivot, 0.f);
  const float rstd = 1.0f / sqrtf(var + eps);
#pragma unroll
  for (int i = 0; i < VPT; ++i) {
    const int c4 = threadIdx.x + i * 256;
    if (c4 >= n4) continue;
    f32x4 y;
#pragma unroll
    for (int e = 0; e < 4; ++e) y[e] = (x[i][e] - mean) * rstd;
    if (g) { const f32x4 v = ((const f32x4*)g)[c4]; y *= v; }
    if (b) { const f32x4 v = ((const f32x4*)b)[c4]; y += v; }
    if (scale) y = y * (1.0f + scv[i]) + shv[i];
    store4<T>(out + (out_tiled ? tile_offset(r, c4 * 4, d) : (size_t)r * d + c4 * 4), y[0], y[1], y[2], y[3]);
  }
}

// ================================================================== RoPE + KV append
template <typename T>
__global__ __launch_bounds__(256) void rope_append_kernel(T* __restrict__ qkv, int ld, int n_heads, KvGeom kv,
                                                          int rope, float theta, const int* __restrict__ row_sample,
                                                          const int* __restrict__ row_pos, int M, const int* m_dev) {
  const int Me = eff_rows(M, m_dev);
  const int r = blockIdx.x;
  if (r >= Me) return;
  const int dh = kv.d_head, Hk = kv.n_kv_heads, half = dh >> 1;
  const int b = row_sample[r], pos = row_pos[r];
  T* row = qkv + (size_t)r * ld;
  const int n_rot_heads = n_heads + Hk;         // q heads then k heads are rotated
  if (rope) {
    // the angle depends on the row's position and on the pair index c only; a thread whose elements all share one c
    // (the workgroup size is a multiple of half the head dim) takes its sine and cosine once
    const bool one_c = (blockDim.x % half) == 0;
    float sn = 0.f, cs = 1.f;
    if (one_c) {
      const float inv = powf(theta, -2.0f * (float)(threadIdx.x % half) / (float)dh);
      sincosf((float)pos * inv, &sn, &cs);
    }
    for (int idx = threadIdx.x; idx < n_rot_heads * half; idx += blockDim.x) {
      const int hd = idx / half, c = idx - hd * half;
      if (!one_c) {
        const float inv = powf(theta, -2.0f * (float)c / (float)dh);
        sincosf((float)pos * inv, &sn, &cs);
      }
      T* p = row + (size_t)hd * dh;
      const float a = to_f32(p[c]), bb = to_f32(p[c + half]);
      p[c] = from_f32<T>(a * cs - bb * sn);
      p[c + half] = from_f32<T>(bb * cs + a * sn);
    }
    __syncthreads();
  }
  const T* ksrc = row + (size_t)n_heads * dh;
  const T* vsrc = ksrc + (size_t)Hk * dh;
  const size_t head_elems = (size_t)kv.ctx_pad * dh;
  for (int idx = threadIdx.x; idx < Hk * dh; idx += blockDim.x) {
    const int hk = idx / dh, d = idx - hk * dh;
    const size_t base = ((size_t)b * Hk + hk) * head_elems;
    size_t ko, vo;
    if (kv.is_bf16) {
      ko = k_offset_bf16(pos, d, dh);
      vo = v_offset_bf16(pos, d, dh);
    } else {
      ko = vo = (size_t)pos * dh + d;
    }
    ((T*)kv.k)[base + ko] = ksrc[idx];
    ((T*)kv.v)[base + vo] = vsrc[idx];
  }
}

// The same from the K-slice planes of the QKV product (fp32 [n_parts][M, ld], bias in plane 0): sums the planes, rotates
// q and k in fp32, writes q as bf16 into qkv (what the attention kernel reads) and k, v into the cache.
// Grid (rows, head groups): a thread owns 4 consecutive dims c .. c+3 of the first half of one head and their partners
// c + d_head/2 ..; all its loads (2 x 16 bytes per plane, PMAX planes at most per batch) are requested before the first sum.
template <int PMAX>
__global__ __launch_bounds__(256) void rope_append_planes_kernel(const float* __restrict__ parts, int n_parts, size_t part_stride,
                                                                 bf16* __restrict__ qkv, int ld, int n_heads, KvGeom kv, int rope,
                                                                 float theta, const int* __restrict__ row_sample,
                                                                 const int* __restrict__ row_pos, int M, const int* m_dev) {
  const int Me = eff_rows(M, m_dev);
  const int r = blockIdx.x;
  if (r >= Me) return;
  const int dh = kv.d_head, Hk = kv.n_kv_heads, half = dh >> 1;
  const int tph = half >> 2;                               // threads per head
  const int hpw = 256 / tph;                               // heads per workgroup
  const int hd = blockIdx.y * hpw + threadIdx.x / tph;     // q heads, then k heads, then v heads
  if (hd >= n_heads + 2 * Hk) return;
  const int c = (threadIdx.x % tph) * 4;
  const int b = row_sample[r], pos = row_pos[r];
  const float* p0 = parts + (size_t)r * ld + (size_t)hd * dh + c;
  f32x4 lo = {0.f, 0.f, 0.f, 0.f}, hi = {0.f, 0.f, 0.f, 0.f};
  for (int pb = 0; pb < n_parts; pb += PMAX) {
    f32x4 tl[PMAX], th[PMAX];
#pragma unroll
    for (int p = 0; p < PMAX; ++p) {
      const int pp = pb + p < n_parts ? pb + p : pb;       // (a re-read that is not added)
      tl[p] = *(const f32x4*)(p0 + (size_t)pp * part_stride);
      th[p] = *(const f32x4*)(p0 + (size_t)pp * part_stride + half);
    }
#pragma unroll
    for (int p = 0; p < PMAX; ++p)
      if (pb + p < n_parts) { lo += tl[p]; hi += th[p]; }
  }
  const bool is_v = hd >= n_heads + Hk;
  if (rope && !is_v) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float sn, cs;
      const float inv = powf(theta, -2.0f * (float)(c + e) / (float)dh);
      sincosf((float)pos * inv, &sn, &cs);
      const float a = lo[e], bb = hi[e];
      lo[e] = a * cs - bb * sn;
      hi[e] = bb * cs + a * sn;
    }
  }
  bf16x4 blo, bhi;
#pragma unroll
  for (int e = 0; e < 4; ++e) { blo[e] = (bf16)lo[e]; bhi[e] = (bf16)hi[e]; }
  const size_t head_elems = (size_t)kv.ctx_pad * dh;
  if (hd < n_heads) {
    bf16* q = qkv + (size_t)r * ld + (size_t)hd * dh + c;
    *(bf16x4*)q = blo;
    *(bf16x4*)(q + half) = bhi;
  } else if (!is_v) {
    bf16* kc = (bf16*)kv.k + ((size_t)b * Hk + (hd - n_heads)) * head_elems;
    *(bf16x4*)(kc + k_offset_bf16(pos, c, dh)) = blo;      // 8 consecutive dims of a key are contiguous in the cache
    *(bf16x4*)(kc + k_offset_bf16(pos, c + half, dh)) = bhi;
  } else {
    bf16* vc = (bf16*)kv.v + ((size_t)b * Hk + (hd - n_heads - Hk)) * head_elems;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      vc[v_offset_bf16(pos, c + e, dh)] = blo[e];
      vc[v_offset_bf16(pos, c + half + e, dh)] = bhi[e];
    }
  }
}

template <typename T>
__global__ __launch_bounds__(256) void kv_load_kernel(KvGeom kv, const T* __restrict__ k, const T* __restrict__ v,
                                                      int B, int n) {
  const int dh = kv.d_head, Hk = kv.n_kv_heads;
  const size_t total = (size_t)B * Hk * n * dh;
  const size_t head_elems = (size_t)kv.ctx_pad * dh;
  for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (size_t)gridDim.x * blockDim.x) {
    const int d = (int)(idx % dh);
    const size_t t = idx / dh;
    const int pos = (int)(t % n);
    const size_t bh = t / n;                     // b * Hk + hk
    size_t ko, vo;
    if (kv.is_bf16) {
      ko = k_offset_bf16(pos, d, dh);
      vo = v_offset_bf16(pos, d, dh);
    } else {
      ko = vo = (size_t)pos * dh + d;
    }
    ((T*)kv.k)[bh * head_elems + ko] = k[idx];
    ((T*)kv.v)[bh * head_elems + vo] = v[idx];
  }
}

// ================================================================== entropy pre-filter
// Online softmax-entropy of one row held by one wave.  Every lane folds its elements into a running
// (m, l, a) kept in base-2 units: m = log2(e) * (reference value), l = sum 2^t, a = sum 2^t * t with
// t = log2(e) * x - m.  The reference cancels in H = ln l - ln(2) * a / l, so any m that avoids overflow is
// valid; lanes are merged through a wave maximum and two wave sums.
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;
struct Mla { float m, l, a; };
// Move the reference of s up to the element value mx (no-op when it is not larger).
__device__ __forceinline__ void mla_raise(Mla& s, float mx) {
  const float m2 = mx * LOG2E;
  if (m2 > s.m) {
    if (s.l > 0.f) {
      const float dl = s.m - m2, e = __builtin_amdgcn_exp2f(dl);
      s.a = e * (s.a + dl * s.l);
      s.l = e * s.l;
    }
    s.m = m2;
  }
}
__device__ __forceinline__ void mla_add(Mla& s, float x) {   // requires x * LOG2E <= s.m (up to rounding)
  const float t = fmaf(x, LOG2E, -s.m), e = __builtin_amdgcn_exp2f(t);
  s.l += e;
  s.a = fmaf(e, t, s.a);
}
__device__ __forceinline__ void mla_push(Mla& s, float x) {
  mla_raise(s, x);
  mla_add(s, x);
}
// Merge the lanes: common reference by a wave maximum, one rescale per lane, two wave sums.
__device__ __forceinline__ float mla_finish(Mla s) {
  const float M = wave_max(s.m);
  float l = 0.f, a = 0.f;
  if (s.l > 0.f) {
    const float dl = s.m - M, e = __builtin_amdgcn_exp2f(dl);
    l = e * s.l;
    a = e * (s.a + dl * s.l);
  }
  l = wave_sum(l);
  a = wave_sum(a);
  return __logf(l) - LN2 * a / l;
}

constexpr int ENT_NCH = 4;                        // 16-byte pieces a lane holds in flight
template <typename T> struct EntVec { using type = f32x4; };
template <> struct EntVec<bf16> { using type = bf16x8; };

// Issue the loads of up to ENT_NCH pieces per lane starting at piece c0 (addresses clamped, nvec >= 1).
template <typename T>
__device__ __forceinline__ void ent_fetch(const T* __restrict__ row, int c0, int nvec, int lane,
                                          typename EntVec<T>::type (&v)[ENT_NCH]) {
  using Vec = typename EntVec<T>::type;
  const Vec* rv = (const Vec*)row;
#pragma unroll
  for (int j = 0; j < ENT_NCH; ++j) {
    const int c = c0 + j * WAVE + lane;
    v[j] = rv[c < nvec ? c : nvec - 1];
  }
}
// Fold the fetched pieces: one maximum over the group, one rescale, then independent exponentials.
template <typename T>
__device__ __forceinline__ void ent_fold(Mla& s, const typename EntVec<T>::type (&v)[ENT_NCH], int c0, int nvec,
                                         int lane) {
  constexpr int VE = 16 / sizeof(T);
  float mx = -INFINITY;
#pragma unroll
  for (int j = 0; j < ENT_NCH; ++j) {
    if (c0 + j * WAVE + lane < nvec) {
#pragma unroll
      for (int i = 0; i < VE; ++i) mx = fmaxf(mx, (float)v[j][i]);
    }
  }
  mla_raise(s, mx);
#pragma unroll
  for (int j = 0; j < ENT_NCH; ++j) {
    if (c0 + j * WAVE + lane < nvec) {
#pragma unroll
      for (int i = 0; i < VE; ++i) mla_add(s, (float)v[j][i]);
    }
  }
}

// Entropy of a row that is entirely in the fetched registers (two passes: wave maximum, then sums).
template <typename T>
__device__ __forceinline__ float ent_row_regs(const typename EntVec<T>::type (&v)[ENT_NCH], int nvec, int lane) {
  constexpr int VE = 16 / sizeof(T);
  float mx = -INFINITY;
#pragma unroll
  for (int j = 0; j < ENT_NCH; ++j) {
    if (j * WAVE + lane < nvec) {
#pragma unroll
      for (int i = 0; i < VE; ++i) mx = fmaxf(mx, (float)v[j][i]);
    }
  }
  const float m2 = wave_max(mx) * LOG2E;
  float l = 0.f, a = 0.f;
#pragma unroll
  for (int j = 0; j < ENT_NCH; ++j) {
    if (j * WAVE + lane < nvec) {
#pragma unroll
      for (int i = 0; i < VE; ++i) {
        const float t = fmaf((float)v[j][i], LOG2E, -m2), e = __builtin_amdgcn_exp2f(t);
        l += e;
        a = fmaf(e, t, a);
      }
    }
  }
  l = wave_sum(l);
  a = wave_sum(a);
  return __logf(l) - LN2 * a / l;
}

// Half a wave per row: lane l32 of the half holds pieces l32, l32 + 32, ... (up to ENT_NCH2), so that the two halves
// of a wave fold two rows at once and share the reductions' instructions.
constexpr int ENT_NCH2 = 8;
template <typename T>
__device__ __forceinline__ void ent_fetch_half(const T* __restrict__ row, int nvec, int l32,
                                               typename EntVec<T>::type (&v)[ENT_NCH2]) {
  using Vec = typename EntVec<T>::type;
  const Vec* rv = (const Vec*)row;
#pragma unroll
  for (int j = 0; j < ENT_NCH2; ++j) {
    if (j * 32 < nvec) {                          // the same for every lane
      const int c = j * 32 + l32;
      v[j] = rv[c < nvec ? c : nvec - 1];
    }
  }
}
template <typename T>
__device__ __forceinline__ float ent_row_half(const typename EntVec<T>::type (&v)[ENT_NCH2], int nvec, int l32) {
  constexpr int VE = 16 / sizeof(T);
  float mx = -INFINITY;
#pragma unroll
  for (int j = 0; j < ENT_NCH2; ++j) {
    if (j * 32 < nvec) {
      if (j * 32 + l32 < nvec) {
#pragma unroll
        for (int i = 0; i < VE; ++i) mx = fmaxf(mx, (float)v[j][i]);
      }
    }
  }
  const float m2 = half_max(mx) * LOG2E;
  float l = 0.f, a = 0.f;
#pragma unroll
  for (int j = 0; j < ENT_NCH2; ++j) {
    if (j * 32 < nvec) {
      if (j * 32 + l32 < nvec) {
#pragma unroll
        for (int i = 0; i < VE; ++i) {
          const float t = fmaf((float)v[j][i], LOG2E, -m2), e = __builtin_amdgcn_exp2f(t);
          l += e;
          a = fmaf(e, t, a);
        }
      }
    }
  }
  l = half_sum(l);
  a = half_sum(a);
  return __logf(l) - LN2 * a / l;
}

template <typename T>
__device__ __forceinline__ float row_entropy_wave(const T* __restrict__ row, int L, int lane) {
  Mla s{-INFINITY, 0.f, 0.f};
  constexpr int VE = 16 / sizeof(T);              // elements per 16-byte piece
  const bool aligned = (((uintptr_t)row) & 15) == 0;
  const int nvec = aligned ? L / VE : 0;
  for (int c0 = 0; c0 < nvec; c0 += ENT_NCH * WAVE) {
    typename EntVec<T>::type v[ENT_NCH];
    ent_fetch<T>(row, c0, nvec, lane, v);
    ent_fold<T>(s, v, c0, nvec, lane);
  }
  for (int c = nvec * VE + lane; c < L; c += WAVE) mla_push(s, to_f32(row[c]));
  return mla_finish(s);
}

// Exclusive scan of one int per thread over a 256-thread workgroup; the workgroup total goes to *total.
__device__ __forceinline__ int block_excl_scan(int v, int* s_scan, int* total) {
  const int tid = threadIdx.x;
  s_scan[tid] = v;
  __syncthreads();
#pragma unroll
  for (int o = 1; o < 256; o <<= 1) {
    const int u = (tid >= o) ? s_scan[tid - o] : 0;
    __syncthreads();
    s_scan[tid] += u;
    __syncthreads();
  }
  const int incl = s_scan[tid];
  *total = s_scan[255];
  __syncthreads();
  return incl - v;
}

// H[r] = entropy of row r (one wave per row, rows `ld` elements apart).
// With n_parts > 0 (fp32 rows held in registers only; the host checks ent_rows_in_regs) the row is
// feat[r] + sum_p parts[p * part_stride + r * L + .]: pending partial planes of a K-sliced GEMM, added in
// plane order.
template <typename T>
__global__ __launch_bounds__(256) void entropy_rows_kernel(const T* __restrict__ feat, int ld, int rows, int L,
                                                           float* __restrict__ H, const float* __restrict__ parts = nullptr,
                                                           int n_parts = 0, size_t part_stride = 0) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = blockIdx.x * 4 + wave;
  if (r >= rows) return;
  const T* row = feat + (size_t)r * ld;
  constexpr int VE = 16 / sizeof(T);
  float h;
  if ((((uintptr_t)row) & 15) == 0 && L % VE == 0 && L >= VE && L / VE <= ENT_NCH * WAVE) {
    typename EntVec<T>::type v[ENT_NCH];
    ent_fetch<T>(row, 0, L / VE, lane, v);
    if constexpr (sizeof(T) == 4) {
      for (int p = 0; p < n_parts; ++p) {
        f32x4 w[ENT_NCH];
        ent_fetch<float>(parts + p * part_stride + (size_t)r * L, 0, L / VE, lane, w);
#pragma unroll
        for (int j = 0; j < ENT_NCH; ++j) v[j] += w[j];
      }
    }
    h = ent_row_regs<T>(v, L / VE, lane);
  } else {
    h = row_entropy_wave(row, L, lane);
  }
  if (lane == 0) H[r] = h;
}

// Threshold, prefix rule and compaction over [B, K] entropies, by one workgroup (small batches).
__global__ __launch_bounds__(256) void prefilter_tail_kernel(const float* __restrict__ H, int B, int K, float tau,
                                                             uint8_t* __restrict__ keep, int* __restrict__ n_keep,
                                                             int* __restrict__ surv_idx, int* __restrict__ n_surv) {
  __shared__ int s_scan[256];
  const int tid = threadIdx.x;
  int carry = 0;
  for (int base = 0; base < B; base += 256) {
    const int b = base + tid;
    int cnt = 0;
    if (b < B) {
      bool alive = true;
      for (int i = 0; i < K; ++i) {
        alive = alive && !(H[(size_t)b * K + i] < tau);
        keep[(size_t)b * K + i] = alive ? 1 : 0;
        cnt += alive ? 1 : 0;
      }
      n_keep[b] = cnt;
    }
    int total;
    const int start = carry + block_excl_scan(cnt, s_scan, &total);
    for (int i = 0; i < cnt; ++i) surv_idx[start + i] = b * K + i;   // kept drafts are a prefix
    carry += total;
  }
  if (tid == 0) *n_surv = carry;
}

// Large batches: a wave (PIPE: half a wave) per sample walks its K rows and applies the prefix rule itself;
// workgroup `blockIdx.x` owns the samples [blockIdx.x * spb, (blockIdx.x + 1) * spb) and records how many drafts
// they kept.  PIPE: every row is at most ENT_NCH2 * 32 aligned 16-byte pieces; the eight half waves of the
// workgroup take the samples b0 + slot, b0 + slot + 8, ..., and the loads of a half's next row are issued before its
// current row is folded (two register sets, taking turns).
template <typename T, bool PIPE>
__global__ __launch_bounds__(256) void entropy_samples_kernel(const T* __restrict__ feat, int B, int K, int L,
                                                              float tau, int spb, float* __restrict__ H,
                                                              uint8_t* __restrict__ keep, int* __restrict__ n_keep,
                                                              int* __restrict__ blk_cnt) {
  __shared__ int s_cnt[8];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int b0 = blockIdx.x * spb, b1 = min(B, b0 + spb);
  int total = 0;
  if constexpr (PIPE) {
    constexpr int VE = 16 / sizeof(T);
    using Vec = typename EntVec<T>::type;
    const int nvec = L / VE;
    const int l32 = lane & 31, slot = wave * 2 + (lane >> 5);
    const int nb = (b1 - b0 - wave * 2 + 7) / 8;   // samples of the wave's first half: never fewer than the second's
    const int nq = nb > 0 ? nb * K : 0;
    Vec va[ENT_NCH2], vb[ENT_NCH2];
    bool alive = true;
    int cnt = 0, i = 0, b = b0 + slot;
    // a half without a sample left reads the workgroup's last sample again and writes nothing
    auto row_of = [&](int bb, int ii) { return feat + ((size_t)min(bb, b1 - 1) * K + ii) * L; };
    auto step = [&](Vec (&cur)[ENT_NCH2], Vec (&nxt)[ENT_NCH2], bool more) {
      const int in = (i + 1 == K) ? 0 : i + 1, bn = (i + 1 == K) ? b + 8 : b;
      if (more) ent_fetch_half<T>(row_of(bn, in), nvec, l32, nxt);
      __builtin_amdgcn_sched_barrier(0);
      const float h = ent_row_half<T>(cur, nvec, l32);
      const bool live = b < b1;
      const size_t r = (size_t)b * K + i;
      alive = alive && !(h < tau);
      cnt += alive ? 1 : 0;
      if (l32 == 0 && live) {
        H[r] = h;
        keep[r] = alive ? 1 : 0;
      }
      if (in == 0) {
        if (l32 == 0 && live) n_keep[b] = cnt;
        total += live ? cnt : 0;
        cnt = 0;
        alive = true;
      }
      i = in;
      b = bn;
    };
    if (nq > 0) ent_fetch_half<T>(row_of(b, 0), nvec, l32, va);
    for (int q = 0; q < nq; q += 2) {
      step(va, vb, q + 1 < nq);
      if (q + 1 < nq) step(vb, va, q + 2 < nq);
    }
    if (l32 == 0) s_cnt[slot] = total;
  } else {
    for (int b = b0 + wave; b < b1; b += 4) {
      bool alive = true;
      int cnt = 0;
      for (int i = 0; i < K; ++i) {
        const size_t r = (size_t)b * K + i;
        const float h = row_entropy_wave(feat + r * L, L, lane);
        alive = alive && !(h < tau);
        cnt += alive ? 1 : 0;
        if (lane == 0) {
          H[r] = h;
          keep[r] = alive ? 1 : 0;
        }
      }
      if (lane == 0) n_keep[b] = cnt;
      total += cnt;
    }
    if ((lane & 31) == 0) s_cnt[wave * 2 + (lane >> 5)] = lane == 0 ? total : 0;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int t = 0;
    for (int w = 0; w < 8; ++w) t += s_cnt[w];
    blk_cnt[blockIdx.x] = t;
  }
}

// Second pass of the large-batch path: workgroup i sums the counts of the workgroups before it, then lists
// the kept drafts of its own samples.
__global__ __launch_bounds__(256) void entropy_compact_kernel(const int* __restrict__ n_keep,
                                                              const int* __restrict__ blk_cnt, int B, int K, int spb,
                                                              int* __restrict__ surv_idx, int* __restrict__ n_surv) {
  __shared__ int s_scan[256];
  const int tid = threadIdx.x;
  int part = 0;
  for (int j = tid; j < (int)blockIdx.x; j += 256) part += blk_cnt[j];
  int carry;
  block_excl_scan(part, s_scan, &carry);
  const int b0 = blockIdx.x * spb, b1 = min(B, b0 + spb);
  for (int base = b0; base < b1; base += 256) {
    const int b = base + tid;
    const int cnt = (b < b1) ? n_keep[b] : 0;
    int total;
    const int start = carry + block_excl_scan(cnt, s_scan, &total);
    for (int i = 0; i < cnt; ++i) surv_idx[start + i] = b * K + i;
    carry += total;
  }
  if (blockIdx.x == gridDim.x - 1 && tid == 0) *n_surv = carry;
}

__global__ __launch_bounds__(256) void entropy_step_kernel(const float* __restrict__ ent_heads, int n_heads,
                                                           const float* __restrict__ H_in, int B, int K, int step,
                                                           float tau, float* __restrict__ H, uint8_t* keep, int* alive,
                                                           int* n_keep, int* act_idx, int* n_act, int* emap,
                                                           int* omap) {
  __shared__ int s_scan[256];
  __shared__ int s_carry;
  const int tid = threadIdx.x;
  if (tid == 0) s_carry = 0;
  __syncthreads();
  for (int base = 0; base < B; base += 256) {
    const int b = base + tid;
    int now = 0;
    if (b < B) {
      float h;
      if (ent_heads) {
        float s = 0.f;
        for (int g = 0; g < n_heads; ++g) s += ent_heads[(size_t)b * n_heads + g];
        h = s / (float)n_heads;
      } else {
        h = H_in[b];
      }
      const int was = alive[b];
      now = (was && !(h < tau)) ? 1 : 0;
      H[(size_t)b * K + step] = was ? h : 0.f;
      keep[(size_t)b * K + step] = (uint8_t)now;
      alive[b] = now;
      n_keep[b] += now;
    }
    s_scan[tid] = now;
    __syncthreads();
    for (int o = 1; o < 256; o <<= 1) {
      int v = (tid >= o) ? s_scan[tid - o] : 0;
      __syncthreads();
      s_scan[tid] += v;
      __syncthreads();
    }
    const int carry = s_carry;
    if (now) {
      const int r = carry + s_scan[tid] - 1;
      act_idx[r] = b;
      emap[r] = b * (K + 1) + step;
      omap[r] = b * K + step;
    }
    __syncthreads();
    if (tid == 255) s_carry = carry + s_scan[255];
    __syncthreads();
  }
  if (tid == 0) *n_act = s_carry;
}

// ================================================================== end of a round (Alg. 1 Step 5)
// One wave per sample.  n_accept < n_keep: acceptance-rejection from the residual max(0, Sigma p - q) with
// proposals mu_p[n] + sigma_p eps_res[j], accepted when u_res[j] <= max(0, 1 - exp(-ln rho)); the last proposal
// is taken if none of the J is accepted.  Otherwise the target's own sample of row n_keep under the shared noise.
// Optionally appends the accepted drafts and the closing token to the sample's token list.
__global__ __launch_bounds__(64) void round_finish_kernel(const float* __restrict__ mu_p, const float* __restrict__ mu_q,
                                                          const float* __restrict__ eps_last,
                                                          const int* __restrict__ n_accept, const int* __restrict__ n_keep,
                                                          const float* __restrict__ eps_res, const float* __restrict__ u_res,
                                                          const float* __restrict__ x_draft, int K, int D, int J,
                                                          float log_sigma, float sigma_p, float sigma_q,
                                                          float* __restrict__ x_next, int* __restrict__ tries,
                                                          float* __restrict__ tokens, int tok_cap,
                                                          int* __restrict__ n_tokens) {
  const int b = blockIdx.x, lane = threadIdx.x;
  const int n = n_accept[b], nk = n_keep[b];
  const bool on = lane < D;
  float xn = 0.f;
  int t = 0;
  if (n < nk) {
    const float mp = on ? mu_p[((size_t)b * (K + 1) + n) * D + lane] : 0.f;
    const float mq = on ? mu_q[((size_t)b * K + n) * D + lane] : 0.f;
    const float cst = log_sigma + (float)D * (logf(sigma_q) - logf(sigma_p));
    const float ip = 1.0f / (2.0f * sigma_p * sigma_p), iq = 1.0f / (2.0f * sigma_q * sigma_q);
    for (int j = 0; j < J; ++j) {
      const float e = on ? eps_res[((size_t)b * J + j) * D + lane] : 0.f;
      xn = mp + sigma_p * e;
      const float a = xn - mp, c = xn - mq;
      const float dp = wave_sum(on ? a * a : 0.f), dq = wave_sum(on ? c * c : 0.f);
      const float lr = cst - dp * ip + dq * iq;
      const float alpha = fmaxf(0.f, 1.0f - expf(-lr));
      t = j + 1;
      if (u_res[(size_t)b * J + j] <= alpha) break;        // uniform across the wave
    }
  } else {
    const size_t o = ((size_t)b * (K + 1) + nk) * D + lane;
    xn = on ? mu_p[o] + sigma_p * eps_last[o] : 0.f;
  }
  if (on) x_next[(size_t)b * D + lane] = xn;
  if (lane == 0) tries[b] = t;
  if (tokens != nullptr) {
    const int pos = n_tokens[b];
    for (int i = 0; i < n; ++i)
      if (on && pos + i < tok_cap) tokens[((size_t)b * tok_cap + pos + i) * D + lane] = x_draft[((size_t)b * K + i) * D + lane];
    if (on && pos + n < tok_cap) tokens[((size_t)b * tok_cap + pos + n) * D + lane] = xn;
    if (lane == 0) n_tokens[b] = pos + n + 1;
  }
}

// Rows that the draft still has to read before the next round: draft K of the samples that accepted all K.
// One workgroup; nq[b] = (n_accept[b] == K), x_pack = those samples' last drafts in sample order.
__global__ __launch_bounds__(256) void catchup_pack_kernel(const int* __restrict__ n_accept, const float* __restrict__ x_draft,
                                                           int B, int K, int D, int* __restrict__ nq,
                                                           float* __restrict__ x_pack) {
  __shared__ int s_scan[256];
  int carry = 0;
  for (int base = 0; base < B; base += 256) {
    const int b = base + threadIdx.x;
    const int f = (b < B && n_accept[b] == K) ? 1 : 0;
    if (b < B) nq[b] = f;
    int total;
    const int r = carry + block_excl_scan(f, s_scan, &total);
    if (f)
      for (int c = 0; c < D; ++c) x_pack[(size_t)r * D + c] = x_draft[((size_t)b * K + K - 1) * D + c];
    carry += total;
  }
}

// ================================================================== head pieces
// First sampler step: hh = x_t W_in + b_in, x_t kept, and the conditioning silu(cz + temb_k) of all S steps
// (step k in rows [k n, (k + 1) n) of sc), so that one GEMM produces the modulations of every step.
template <typename T>
__global__ __launch_bounds__(256) void head_prep_kernel(const float* __restrict__ xsrc, const int* __restrict__ xmap,
                                                        float xscale, int D, const T* __restrict__ w_in,
                                                        const float* __restrict__ b_in, const float* __restrict__ cz,
                                                        const float* __restrict__ temb, int S, float* __restrict__ hh,
                                                        T* __restrict__ sc, float* __restrict__ xt_out, int w, int n,
                                                        const int* n_dev) {
  const int ne = eff_rows(n, n_dev);
  const int r = blockIdx.y;
  if (r >= ne) return;
  const int c = blockIdx.x * 256 + threadIdx.x;
  const float* xr = xsrc + (size_t)(xmap ? xmap[r] : r) * D;
  if (c < w) {
    const float czv = cz[(size_t)r * w + c];
    hh[(size_t)r * w + c] = in_proj<T>(b_in[c], xr, xscale, D, w_in, w, c);
    for (int k = 0; k < S; ++k) sc[((size_t)k * n + r) * w + c] = from_f32<T>(silu(czv + temb[(size_t)k * w + c]));
  }
  if (xt_out && blockIdx.x == 0 && (int)threadIdx.x < D) xt_out[(size_t)r * D + threadIdx.x] = xr[threadIdx.x] * xscale;
}

// One workgroup per row: final AdaLN, output projection to D <= 16 components, sampler update, and (when
// another step follows) the input projection of the new x_t into hh.  The row, its modulation and the
// projection rows are fetched with 16-byte loads issued up front (w <= 256 * 4 * HO_VPT).
constexpr int HO_VPT = 2;
template <typename T>
__device__ __forceinline__ void load_w16(const T* p, float (&o)[16]);
template <>
__device__ __forceinline__ void load_w16<float>(const float* p, float (&o)[16]) {
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const f32x4 v = ((const f32x4*)p)[q];
#pragma unroll
    for (int e = 0; e < 4; ++e) o[q * 4 + e] = v[e];
  }
}
template <>
__device__ __forceinline__ void load_w16<bf16>(const bf16* p, float (&o)[16]) {
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const bf16x8 v = ((const bf16x8*)p)[q];
#pragma unroll
    for (int e = 0; e < 8; ++e) o[q * 8 + e] = (float)v[e];
  }
}

template <typename T>
__global__ __launch_bounds__(256) void head_out_kernel(HeadStepArgs a) {
  __shared__ float red[8];
  __shared__ float part[4][16];
  __shared__ float xs[16];
  const int ne = eff_rows(a.n, a.n_dev);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = blockIdx.x;
  if (r >= ne) return;
  const int w = a.w, D = a.D, n4 = w >> 2;
  const float* row = a.hh + (size_t)r * w;
  const float* scp = a.scale + (size_t)r * a.ldm;
  const float* shp = a.shift + (size_t)r * a.ldm;
  f32x4 x[HO_VPT], sc[HO_VPT], sh[HO_VPT];
#pragma unroll
  for (int i = 0; i < HO_VPT; ++i) {
    const int c4 = threadIdx.x + i * 256;
    const bool ok = c4 < n4;
    const f32x4 z4 = {0.f, 0.f, 0.f, 0.f};
    x[i] = ok ? ((const f32x4*)row)[c4] : z4;
    sc[i] = ok ? ((const f32x4*)scp)[c4] : z4;
    sh[i] = ok ? ((const f32x4*)shp)[c4] : z4;
  }
  // Operands of the later phases (output projection, sampler update, next step's input projection) are requested
  // here, before the first barrier, when they fit in registers (bf16, D = 16, w <= 2048): the kernel then waits
  // for memory once instead of once per phase.
  constexpr bool CAN_PRE = sizeof(T) == 2;
  constexpr int NJ = 4 * HO_VPT;                          // columns per thread of the next step's input projection
  const bool pre = CAN_PRE && D == 16 && w <= 256 * NJ;
  const T* W = (const T*)a.w_out;
  const T* w_in = (const T*)a.w_in;
  bf16x8 wq[HO_VPT][4][2];
  T wvn[NJ][16];
  float bjn[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) bjn[j] = 0.f;
  float p_xt = 0.f, p_eps = 0.f, p_bout = 0.f;
  size_t p_oi = 0;
  if constexpr (CAN_PRE) {
    if (pre) {
#pragma unroll
      for (int i = 0; i < HO_VPT; ++i) {
        const int c4 = threadIdx.x + i * 256;
        const int cc = (c4 < n4) ? c4 : 0;
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
          for (int hq = 0; hq < 2; ++hq) wq[i][e][hq] = ((const bf16x8*)(W + (size_t)(cc * 4 + e) * 16))[hq];
      }
      if (threadIdx.x < 16) {
        const int k = threadIdx.x;
        p_bout = a.b_out[k];
        p_xt = a.xt[(size_t)r * 16 + k];
        p_oi = (size_t)(a.omap ? a.omap[r] : r) * 16 + k;
        if (a.last || a.renoise) p_eps = a.eps_next[(size_t)(a.emap ? a.emap[r] : r) * 16 + k];
      }
      if (!a.last) {
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
          const int c = ((int)threadIdx.x + 256 * j < w) ? (int)threadIdx.x + 256 * j : (int)threadIdx.x;
          bjn[j] = a.b_in[c];
#pragma unroll
          for (int k = 0; k < 16; ++k) wvn[j][k] = w_in[(size_t)k * w + c];
        }
      }
    }
  }
  // both moments in one reduction round, about a pivot (see norm_kernel)
  const float pivot = row[0];
  float s = 0.f, q = 0.f;
#pragma unroll
  for (int i = 0; i < HO_VPT; ++i) {
    if ((int)threadIdx.x + i * 256 < n4) {
#pragma unroll
      for (int e = 0; e < 4; ++e) { const float t = x[i][e] - pivot; s += t; q = fmaf(t, t, q); }
    }
  }
  block_sum2(s, q, red);
  const float m1 = s / (float)w;
  const float mean = pivot + m1;
  const float rstd = 1.0f / sqrtf(fmaxf(q / (float)w - m1 * m1, 0.f) + 1e-6f);
  float acc[16];
#pragma unroll
  for (int k = 0; k < 16; ++k) acc[k] = 0.f;
#pragma unroll
  for (int i = 0; i < HO_VPT; ++i) {
    const int c4 = threadIdx.x + i * 256;
    if (c4 >= n4) continue;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float y = (x[i][e] - mean) * rstd * (1.0f + sc[i][e]) + sh[i][e];
      const int c = c4 * 4 + e;
      if (CAN_PRE && pre) {
#pragma unroll
        for (int k = 0; k < 16; ++k) acc[k] += y * (float)wq[i][e][k >> 3][k & 7];
      } else if (D == 16) {
        float wr[16];
        load_w16<T>(W + (size_t)c * 16, wr);
#pragma unroll
        for (int k = 0; k < 16; ++k) acc[k] += y * wr[k];
      } else {
#pragma unroll
        for (int k = 0; k < 16; ++k)
          if (k < D) acc[k] += y * to_f32(W[(size_t)c * D + k]);
      }
    }
  }
#pragma unroll
  for (int k = 0; k < 16; ++k) acc[k] = wave_sum(acc[k]);
  if (lane == 0) {
#pragma unroll
    for (int k = 0; k < 16; ++k) part[wave][k] = acc[k];
  }
  __syncthreads();
  if ((int)threadIdx.x < D) {
    const int k = threadIdx.x;
    const float v = part[0][k] + part[1][k] + part[2][k] + part[3][k] + (pre ? p_bout : a.b_out[k]);
    const size_t xi = (size_t)r * D + k;
    const size_t ei = pre ? 0 : (size_t)(a.emap ? a.emap[r] : r) * D + k;
    const size_t oi = pre ? p_oi : (size_t)(a.omap ? a.omap[r] : r) * D + k;
    const float xt = pre ? p_xt : a.xt[xi];
    const float x0 = xt - a.t * v;
    if (a.last) {
      a.mu[oi] = x0;
      a.x[oi] = x0 + a.sigma * (pre ? p_eps : a.eps_next[ei]);
    } else {
      const float e = a.renoise ? (pre ? p_eps : a.eps_next[ei]) : xt + (1.0f - a.t) * v;
      const float xn = (1.0f - a.t_next) * x0 + a.t_next * e;
      a.xt[xi] = xn;
      xs[k] = xn;
    }
  }
  if (a.last) return;
  __syncthreads();
  // input projection of the next step
  if (CAN_PRE && pre) {
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int c = threadIdx.x + 256 * j;
      if (c >= w) continue;
      float v = bjn[j];
#pragma unroll
      for (int k = 0; k < 16; ++k) v += xs[k] * (float)wvn[j][k];
      a.hh_next[(size_t)r * w + c] = v;
    }
  } else if (D <= 16) {
    // 4 columns per thread and pass, all 64 weight loads in flight together
    float xr[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) xr[k] = (k < D) ? xs[k] : 0.f;
    for (int c0 = threadIdx.x; c0 < w; c0 += 1024) {
      float wv[4][16], bj[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int c = (c0 + 256 * j < w) ? c0 + 256 * j : c0;
        bj[j] = a.b_in[c];
#pragma unroll
        for (int k = 0; k < 16; ++k) wv[j][k] = to_f32(w_in[(size_t)(k < D ? k : 0) * w + c]);
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int c = c0 + 256 * j;
        if (c >= w) continue;
        float v = bj[j];
#pragma unroll
        for (int k = 0; k < 16; ++k) v += xr[k] * wv[j][k];
        a.hh_next[(size_t)r * w + c] = v;
      }
    }
  } else {
    for (int c = threadIdx.x; c < w; c += 256)
      a.hh_next[(size_t)r * w + c] = in_proj<T>(a.b_in[c], (const float*)xs, 1.0f, D, w_in, w, c);
  }
}

template <typename T>
__global__ __launch_bounds__(256) void matvec_kernel(const float* __restrict__ in, const T* __restrict__ W,
                                                     const float* __restrict__ b, int K, int N, int act,
                                                     float* __restrict__ out) {
  const int n = blockIdx.x * blockDim.x + threadIdx.x;
  if (n >= N) return;
  float v = b ? b[n] : 0.f;
  for (int k = 0; k < K; ++k) v += in[k] * to_f32(W[(size_t)k * N + n]);
  out[n] = apply_act(v, act);
}

// ================================================================== accept test
__global__ __launch_bounds__(64) void accept_kernel(const float* __restrict__ x, const float* __restrict__ mu_p,
                                                    const float* __restrict__ mu_q, const float* __restrict__ r,
                                                    const int* __restrict__ n_keep, float log_sigma, float sigma_p,
                                                    float sigma_q, int B, int K, int D, int* n_accept,
                                                    float* log_ratio, uint8_t* acc) {
  __shared__ int s_acc[256];
  const int b = blockIdx.x, i = threadIdx.x;
  const float cst = log_sigma + (float)D * (logf(sigma_q) - logf(sigma_p));
  const float ip = 1.0f / (2.0f * sigma_p * sigma_p), iq = 1.0f / (2.0f * sigma_q * sigma_q);
  for (int base = 0; base < K; base += 64) {
    const int t = base + i;
    if (t < K) {
      const float* xv = x + ((size_t)b * K + t) * D;
      const float* mp = mu_p + ((size_t)b * (K + 1) + t) * D;
      const float* mq = mu_q + ((size_t)b * K + t) * D;
      float dp = 0.f, dq = 0.f;
      for (int c = 0; c < D; ++c) {
        const float a = xv[c] - mp[c], e = xv[c] - mq[c];
        dp += a * a;
        dq += e * e;
      }
      const float lr = cst - dp * ip + dq * iq;
      const int ok = (logf(r[(size_t)b * K + t]) <= lr) ? 1 : 0;
      log_ratio[(size_t)b * K + t] = lr;
      acc[(size_t)b * K + t] = (uint8_t)ok;
      s_acc[t] = ok;
    }
  }
  __syncthreads();
  if (i == 0) {
    const int lim = n_keep[b] < K ? n_keep[b] : K;
    int n = 0;
    while (n < lim && s_acc[n]) ++n;
    n_accept[b] = n;
  }
}

__global__ void len_add_kernel(int* cache_len, const int* n, int base, int B, int* row_pos) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < B) {
    const int v = cache_len[b] + base + (n ? n[b] : 0);
    cache_len[b] = v;
    if (row_pos) row_pos[b] = v;             // one row per sample: row b's next position
  }
}
__global__ void fill_i32_kernel(int* p, int v, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}
__global__ void fill_f32_kernel(float* p, float v, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}
template <typename E>
__global__ void scatter_rows_kernel(const E* __restrict__ src, E* __restrict__ dst, const int* __restrict__ dmap,
                                    int width, int n, const int* n_dev) {
  const int ne = eff_rows(n, n_dev);
  const int r = blockIdx.y;
  if (r >= ne) return;
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c < width) dst[(size_t)(dmap ? dmap[r] : r) * width + c] = src[(size_t)r * width + c];
}

}  // namespace

// ====================================================================== launchers
hipError_t launch_build_rows(hipStream_t s, const int* n_base, int add, int B, int K, int D, const int* cache_len,
                             RowMaps maps, const float* x_first, const float* x_rest, float* x_out, int* aux_row,
                             int m_max, int nq_cap) {
  build_rows_kernel<<<1, 256, 0, s>>>(n_base, add, B, K, D, cache_len, maps, x_first, x_rest, x_out, aux_row, m_max,
                                      nq_cap);
  return hipGetLastError();
}

hipError_t launch_embed(hipStream_t s, int is_bf16, const float* x, int ldx, int D, const void* w_in, const float* b_in,
                        const void* pos_table, const int* row_pos, const void* cond_table, const int* cond_id,
                        float* h, int d, int M, const int* m_dev) {
  if (M <= 0) return hipSuccess;
  dim3 grid((d + 255) / 256, M);
  if (is_bf16)
    embed_kernel<bf16><<<grid, 256, 0, s>>>(x, ldx, D, (const bf16*)w_in, b_in, (const bf16*)pos_table, row_pos,
                                            (const bf16*)cond_table, cond_id, h, d, M, m_dev);
  else
    embed_kernel<float><<<grid, 256, 0, s>>>(x, ldx, D, (const float*)w_in, b_in, (const float*)pos_table, row_pos,
                                             (const float*)cond_table, cond_id, h, d, M, m_dev);
  return hipGetLastError();
}

// h[r, :] += sum_p parts[p][r, :] for r < M (device-side count honoured): the residual update that a K-sliced GEMM
// left undone, for consumers of the stream that are not a norm.
__global__ __launch_bounds__(256) void add_parts_kernel(float* __restrict__ h, const float* __restrict__ parts, int n_parts,
                                                        size_t part_stride, int d, int M, const int* m_dev) {
  const int Me = eff_rows(M, m_dev);
  const int r = blockIdx.x;
  if (r >= Me) return;
  for (int c4 = threadIdx.x; c4 < (d >> 2); c4 += 256) {
    const size_t o = (size_t)r * d + c4 * 4;
    f32x4 v = *(const f32x4*)(h + o);
    for (int p = 0; p < n_parts; ++p) v += *(const f32x4*)(parts + (size_t)p * part_stride + o);
    *(f32x4*)(h + o) = v;
  }
}

template <typename T>
__device__ __forceinline__ f32x4 load4f(const T* p);
template <>
__device__ __forceinline__ f32x4 load4f<float>(const float* p) { return *(const f32x4*)p; }
template <>
__device__ __forceinline__ f32x4 load4f<bf16>(const bf16* p) {
  const bf16x4 t = *(const bf16x4*)p;
  return f32x4{(float)t[0], (float)t[1], (float)t[2], (float)t[3]};
}

// embed + the first norm of layer 0 in one launch: one workgroup per row computes h[r, :] as embed_kernel does,
// keeps it in registers, writes it, and writes u[r, :] = norm(h[r, :]) g + b (what norm_kernel would).
template <typename T, int VPT>
__global__ __launch_bounds__(256) void embed_norm_kernel(const float* __restrict__ x, int ldx, int D, const T* __restrict__ w_in,
                                                         const float* __restrict__ b_in, const T* __restrict__ pos_table,
                                                         const int* __restrict__ row_pos, const T* __restrict__ cond_table,
                                                         const int* __restrict__ cond_id, float* __restrict__ h, int d, int M,
                                                         const int* m_dev, int norm_type, float eps, const float* __restrict__ g,
                                                         const float* __restrict__ b, T* __restrict__ u, int u_tiled) {
  __shared__ float red[8];
  const int Me = eff_rows(M, m_dev);
  const int r = blockIdx.x;
  if (r >= Me) return;
  const int n4 = d >> 2;
  const int id = cond_id ? cond_id[r] : -1;
  const int pos = (pos_table && id < 0) ? row_pos[r] : 0;
  f32x4 v[VPT];
  float s = 0.f;
  float xr[16];                                            // D <= 16 (checked on the host)
#pragma unroll
  for (int k = 0; k < 16; ++k) xr[k] = (k < D) ? x[(size_t)r * ldx + k] : 0.f;
#pragma unroll
  for (int i = 0; i < VPT; ++i) {
    const int c4 = threadIdx.x + i * 256;
    v[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (c4 < n4) {
      if (id >= 0) {
        v[i] = load4f<T>(cond_table + (size_t)id * d + c4 * 4);
      } else {
        // four columns at a time: all 16 weight loads of the group are issued before the first use
        f32x4 w[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) w[k] = load4f<T>(w_in + (size_t)(k < D ? k : 0) * d + c4 * 4);
        if (b_in) v[i] = ((const f32x4*)b_in)[c4];
        if (pos_table) v[i] += load4f<T>(pos_table + (size_t)pos * d + c4 * 4);
#pragma unroll
        for (int k = 0; k < 16; ++k) v[i] += w[k] * xr[k];
      }
      *(f32x4*)(h + (size_t)r * d + c4 * 4) = v[i];
      s += v[i][0] + v[i][1] + v[i][2] + v[i][3];
    }
  }
  float mean = 0.f;
  if (norm_type == 0) mean = block_sum(s, red) / (float)d;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < VPT; ++i) {
    if ((int)threadIdx.x + i * 256 < n4) {
#pragma unroll
      for (int e = 0; e < 4; ++e) { const float t = v[i][e] - mean; q += t * t; }
    }
  }
  const float rstd = 1.0f / sqrtf(block_sum(q, red) / (float)d + eps);
#pragma unroll
  for (int i = 0; i < VPT; ++i) {
    const int c4 = threadIdx.x + i * 256;
    if (c4 >= n4) continue;
    f32x4 y;
#pragma unroll
    for (int e = 0; e < 4; ++e) y[e] = (v[i][e] - mean) * rstd;
    if (g) y *= ((const f32x4*)g)[c4];
    if (b) y += ((const f32x4*)b)[c4];
    store4<T>(u + (u_tiled ? tile_offset(r, c4 * 4, d) : (size_t)r * d + c4 * 4), y[0], y[1], y[2], y[3]);
  }
}

hipError_t launch_embed_norm(hipStream_t s, int is_bf16, const float* x, int ldx, int D, const void* w_in, const float* b_in,
                             const void* pos_table, const int* row_pos, const void* cond_table, const int* cond_id, float* h,
                             int d, int M, const int* m_dev, int norm_type, float eps, const float* g, const float* b, void* u,
                             int u_tiled) {
  if (M <= 0) return hipSuccess;
  if (d % 4 != 0 || d > 256 * 4 * NORM_VPT || (u_tiled && (!is_bf16 || d % 32 != 0))) return hipErrorInvalidValue;
#define FARD_EN(VPT)                                                                                                       \
  do {                                                                                                                     \
    if (is_bf16)                                                                                                           \
      embed_norm_kernel<bf16, VPT><<<M, 256, 0, s>>>(x, ldx, D, (const bf16*)w_in, b_in, (const bf16*)pos_table, row_pos,  \
                                                     (const bf16*)cond_table, cond_id, h, d, M, m_dev, norm_type, eps, g, b, \
                                                     (bf16*)u, u_tiled);                                                   \
    else                                                                                                                   \
      embed_norm_kernel<float, VPT><<<M, 256, 0, s>>>(x, ldx, D, (const float*)w_in, b_in, (const float*)pos_table, row_pos, \
                                                      (const float*)cond_table, cond_id, h, d, M, m_dev, norm_type, eps, g, b, \
                                                      (float*)u, 0);                                                       \
  } while (0)
  const int n4 = d >> 2;
  if (n4 <= 256) FARD_EN(1);
  else if (n4 <= 512) FARD_EN(2);
  else if (n4 <= 1024) FARD_EN(4);
  else FARD_EN(8);
#undef FARD_EN
  return hipGetLastError();
}

hipError_t launch_add_parts(hipStream_t s, float* h, const float* parts, int n_parts, size_t part_stride, int d, int M,
                            const int* m_dev) {
  if (M <= 0 || n_parts <= 0) return hipSuccess;
  add_parts_kernel<<<M, 256, 0, s>>>(h, parts, n_parts, part_stride, d, M, m_dev);
  return hipGetLastError();
}

hipError_t launch_norm(hipStream_t s, int is_bf16, const float* h, int d, int M, const int* m_dev, int norm_type,
                       float eps, const float* g, const float* b, const float* shift, const float* scale, int ldm,
                       const int* in_map, void* out, const float* parts, int n_parts, size_t part_stride, float* h_wb,
                       int out_tiled) {
  if (M <= 0) return hipSuccess;
  if (d % 4 != 0 || d > 256 * 4 * NORM_VPT || ldm % 4 != 0 || (out_tiled && (!is_bf16 || d % 32 != 0))) return hipErrorInvalidValue;
#define FARD_NORM(VPT)                                                                                                 \
  do {                                                                                                                 \
    if (is_bf16)                                                                                                       \
      norm_kernel<bf16, VPT><<<M, 256, 0, s>>>(h, d, M, m_dev, norm_type, eps, g, b, shift, scale, ldm, in_map, (bf16*)out, parts, n_parts, part_stride, h_wb, out_tiled);  \
    else                                                                                                               \
      norm_kernel<float, VPT><<<M, 256, 0, s>>>(h, d, M, m_dev, norm_type, eps, g, b, shift, scale, ldm, in_map, (float*)out, parts, n_parts, part_stride, h_wb, 0); \
  } while (0)
  if (d <= 1024) FARD_NORM(1);
  else if (d <= 2048) FARD_NORM(2);
  else if (d <= 4096) FARD_NORM(4);
  else FARD_NORM(8);
#undef FARD_NORM
  return hipGetLastError();
}

hipError_t launch_rope_append(hipStream_t s, void* qkv, int ld, int n_heads, KvGeom kv, int rope, float rope_theta,
                              const int* row_sample, const int* row_pos, int M, const int* m_dev) {
  if (M <= 0) return hipSuccess;
  if (kv.is_bf16)
    rope_append_kernel<bf16><<<M, 256, 0, s>>>((bf16*)qkv, ld, n_heads, kv, rope, rope_theta, row_sample, row_pos, M, m_dev);
  else
    rope_append_kernel<float><<<M, 256, 0, s>>>((float*)qkv, ld, n_heads, kv, rope, rope_theta, row_sample, row_pos, M, m_dev);
  return hipGetLastError();
}

hipError_t launch_rope_append_planes(hipStream_t s, const float* parts, int n_parts, size_t part_stride, void* qkv, int ld,
                                     int n_heads, KvGeom kv, int rope, float rope_theta, const int* row_sample,
                                     const int* row_pos, int M, const int* m_dev) {
  if (M <= 0) return hipSuccess;
  const int dh = kv.d_head;
  // a head's first half in groups of 4 dims; 16-byte loads of the planes, 8-byte stores of q and k
  if (!kv.is_bf16 || n_parts < 1 || dh % 16 != 0 || dh > 2048 || 256 % (dh / 8) != 0 || ld % 4 != 0 || part_stride % 4 != 0 ||
      (((uintptr_t)parts) & 15) != 0 || (((uintptr_t)qkv) & 7) != 0)
    return hipErrorInvalidValue;
  const int hpw = 256 / (dh / 8);
  const dim3 grid(M, (n_heads + 2 * kv.n_kv_heads + hpw - 1) / hpw);
  rope_append_planes_kernel<8><<<grid, 256, 0, s>>>(parts, n_parts, part_stride, (bf16*)qkv, ld, n_heads, kv, rope, rope_theta,
                                                    row_sample, row_pos, M, m_dev);
  return hipGetLastError();
}

hipError_t launch_kv_load(hipStream_t s, KvGeom kv, const void* k, const void* v, int B, int n) {
  const size_t total = (size_t)B * kv.n_kv_heads * n * kv.d_head;
  if (total == 0) return hipSuccess;
  size_t blocks = (total + 255) / 256;
  if (blocks > 65535) blocks = 65535;
  if (kv.is_bf16)
    kv_load_kernel<bf16><<<(unsigned)blocks, 256, 0, s>>>(kv, (const bf16*)k, (const bf16*)v, B, n);
  else
    kv_load_kernel<float><<<(unsigned)blocks, 256, 0, s>>>(kv, (const float*)k, (const float*)v, B, n);
  return hipGetLastError();
}

template <typename T>
static void launch_entropy_prefilter_t(hipStream_t s, const T* feat, int B, int K, int L, float tau, float* H,
                                       uint8_t* keep, int* n_keep, int* surv_idx, int* n_surv, int* blk_cnt) {
  if (B <= ENT_SAMPLE_MODE_MIN_B) {
    const int rows = B * K;
    if (rows > 0) entropy_rows_kernel<T><<<(rows + 3) / 4, 256, 0, s>>>(feat, L, rows, L, H);
    prefilter_tail_kernel<<<1, 256, 0, s>>>(H, B, K, tau, keep, n_keep, surv_idx, n_surv);
    return;
  }
  int spb = (B + ENT_MAX_BLOCKS - 1) / ENT_MAX_BLOCKS;
  spb = (spb + 7) & ~7;
  const unsigned blocks = (unsigned)((B + spb - 1) / spb);
  constexpr int VE = 16 / (int)sizeof(T);
  const bool pipe = (((uintptr_t)feat) & 15) == 0 && L % VE == 0 && L >= VE && L / VE <= ENT_NCH2 * 32;
  if (pipe)
    entropy_samples_kernel<T, true><<<blocks, 256, 0, s>>>(feat, B, K, L, tau, spb, H, keep, n_keep, blk_cnt);
  else
    entropy_samples_kernel<T, false><<<blocks, 256, 0, s>>>(feat, B, K, L, tau, spb, H, keep, n_keep, blk_cnt);
  entropy_compact_kernel<<<blocks, 256, 0, s>>>(n_keep, blk_cnt, B, K, spb, surv_idx, n_surv);
}

hipError_t launch_entropy_prefilter(hipStream_t s, int is_bf16, const void* feat, int B, int K, int L, float tau,
                                    float* H, uint8_t* keep, int* n_keep, int* surv_idx, int* n_surv, int* blk_cnt) {
  if (is_bf16)
    launch_entropy_prefilter_t<bf16>(s, (const bf16*)feat, B, K, L, tau, H, keep, n_keep, surv_idx, n_surv, blk_cnt);
  else
    launch_entropy_prefilter_t<float>(s, (const float*)feat, B, K, L, tau, H, keep, n_keep, surv_idx, n_surv, blk_cnt);
  return hipGetLastError();
}

bool ent_rows_in_regs_f32(const float* feat, int ld, int L) {
  return (((uintptr_t)feat) & 15) == 0 && ld % 4 == 0 && L % 4 == 0 && L >= 4 && L / 4 <= ENT_NCH * WAVE;
}

hipError_t launch_entropy_rows_f32(hipStream_t s, const float* feat, int ld, int rows, int L, float* H, const float* parts,
                                   int n_parts, size_t part_stride) {
  if (rows <= 0) return hipSuccess;
  if (n_parts > 0 && (!ent_rows_in_regs_f32(feat, ld, L) || (((uintptr_t)parts) & 15) != 0 || part_stride % 4 != 0))
    return hipErrorInvalidValue;
  entropy_rows_kernel<float><<<(rows + 3) / 4, 256, 0, s>>>(feat, ld, rows, L, H, parts, n_parts, part_stride);
  return hipGetLastError();
}

hipError_t launch_entropy_step(hipStream_t s, const float* ent_heads, int n_heads, const float* H_in, int B, int K,
                               int step, float tau, float* H, uint8_t* keep, int* alive, int* n_keep, int* act_idx,
                               int* n_act, int* emap, int* omap) {
  entropy_step_kernel<<<1, 256, 0, s>>>(ent_heads, n_heads, H_in, B, K, step, tau, H, keep, alive, n_keep, act_idx,
                                        n_act, emap, omap);
  return hipGetLastError();
}

hipError_t launch_head_prep(hipStream_t s, int is_bf16, const float* xsrc, const int* xmap, float xscale, int D,
                            const void* w_in, const float* b_in, const float* cz, const float* temb, int S, float* hh,
                            void* sc, float* xt_out, int w, int n, const int* n_dev) {
  if (n <= 0) return hipSuccess;
  dim3 grid((w + 255) / 256, n);
  if (is_bf16)
    head_prep_kernel<bf16><<<grid, 256, 0, s>>>(xsrc, xmap, xscale, D, (const bf16*)w_in, b_in, cz, temb, S, hh,
                                                (bf16*)sc, xt_out, w, n, n_dev);
  else
    head_prep_kernel<float><<<grid, 256, 0, s>>>(xsrc, xmap, xscale, D, (const float*)w_in, b_in, cz, temb, S, hh,
                                                 (float*)sc, xt_out, w, n, n_dev);
  return hipGetLastError();
}

hipError_t launch_head_out(hipStream_t s, int is_bf16, const HeadStepArgs& a) {
  if (a.n <= 0) return hipSuccess;
  if (a.D > 16 || a.w % 4 != 0 || a.w > 256 * 4 * HO_VPT || a.ldm % 4 != 0) return hipErrorInvalidValue;
  if (is_bf16)
    head_out_kernel<bf16><<<a.n, 256, 0, s>>>(a);
  else
    head_out_kernel<float><<<a.n, 256, 0, s>>>(a);
  return hipGetLastError();
}

hipError_t launch_round_finish(hipStream_t s, const float* mu_p, const float* mu_q, const float* eps_last, const int* n_accept,
                               const int* n_keep, const float* eps_res, const float* u_res, const float* x_draft, int B, int K,
                               int D, int J, float log_sigma, float sigma_p, float sigma_q, float* x_next, int* tries,
                               float* tokens, int tok_cap, int* n_tokens) {
  if (B <= 0) return hipSuccess;
  if (D > 64 || J < 1) return hipErrorInvalidValue;
  round_finish_kernel<<<B, 64, 0, s>>>(mu_p, mu_q, eps_last, n_accept, n_keep, eps_res, u_res, x_draft, K, D, J, log_sigma,
                                       sigma_p, sigma_q, x_next, tries, tokens, tok_cap, n_tokens);
  return hipGetLastError();
}

hipError_t launch_catchup_pack(hipStream_t s, const int* n_accept, const float* x_draft, int B, int K, int D, int* nq,
                               float* x_pack) {
  if (B <= 0) return hipSuccess;
  catchup_pack_kernel<<<1, 256, 0, s>>>(n_accept, x_draft, B, K, D, nq, x_pack);
  return hipGetLastError();
}

hipError_t launch_matvec(hipStream_t s, int is_bf16, const float* in, const void* W, const float* b, int K, int N,
                         int act, float* out) {
  if (is_bf16)
    matvec_kernel<bf16><<<(N + 255) / 256, 256, 0, s>>>(in, (const bf16*)W, b, K, N, act, out);
  else
    matvec_kernel<float><<<(N + 255) / 256, 256, 0, s>>>(in, (const float*)W, b, K, N, act, out);
  return hipGetLastError();
}

hipError_t launch_accept(hipStream_t s, const float* x, const float* mu_p, const float* mu_q, const float* r,
                         const int* n_keep, float log_sigma, float sigma_p, float sigma_q, int B, int K, int D,
                         int* n_accept, float* log_ratio, uint8_t* acc) {
  if (B <= 0) return hipSuccess;
  accept_kernel<<<B, 64, 0, s>>>(x, mu_p, mu_q, r, n_keep, log_sigma, sigma_p, sigma_q, B, K, D, n_accept, log_ratio, acc);
  return hipGetLastError();
}

hipError_t launch_len_add(hipStream_t s, int* cache_len, const int* n, int base, int B, int* row_pos) {
  len_add_kernel<<<(B + 255) / 256, 256, 0, s>>>(cache_len, n, base, B, row_pos);
  return hipGetLastError();
}
hipError_t launch_fill_i32(hipStream_t s, int* p, int v, int n) {
  if (n <= 0) return hipSuccess;
  fill_i32_kernel<<<(n + 255) / 256, 256, 0, s>>>(p, v, n);
  return hipGetLastError();
}
hipError_t launch_fill_f32(hipStream_t s, float* p, float v, size_t n) {
  if (n == 0) return hipSuccess;
  size_t blocks = (n + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  fill_f32_kernel<<<(unsigned)blocks, 256, 0, s>>>(p, v, n);
  return hipGetLastError();
}
hipError_t launch_scatter_rows(hipStream_t s, const void* src, void* dst, const int* dmap, int width, int elem_size,
                               int n, const int* n_dev) {
  if (n <= 0) return hipSuccess;
  dim3 grid((width + 255) / 256, n);
  if (elem_size == 4)
    scatter_rows_kernel<float><<<grid, 256, 0, s>>>((const float*)src, (float*)dst, dmap, width, n, n_dev);
  else
    scatter_rows_kernel<bf16><<<grid, 256, 0, s>>>((const bf16*)src, (bf16*)dst, dmap, width, n, n_dev);
  return hipGetLastError();
}

}  // namespace fard

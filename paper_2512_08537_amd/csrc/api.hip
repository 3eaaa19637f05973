// C-ABI entry points and host-side orchestration of the speculative round (see include/fastardiff.h).
// No kernel in this file touches the method's arithmetic except two tiny helpers (type conversion
// at weight upload, cache-length commit); everything else is launched from gemm.hip, attn.hip,
// rowops.hip.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <map>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/fastardiff.h"
#include "gemm.h"
#include "kernels.h"

using namespace fard;

namespace {

// ------------------------------------------------------------------------------ small kernels
template <typename TS, typename TD>
__global__ void convert_kernel(const TS* __restrict__ src, TD* __restrict__ dst, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    dst[i] = from_f32<TD>(to_f32(src[i]));
}
// dst[k, col0 + n] = src[k, n] for a [K, N] block placed inside a [K, ldd] matrix
template <typename TS, typename TD>
__global__ void place_kernel(const TS* __restrict__ src, TD* __restrict__ dst, int K, int N, int ldd, int col0) {
  const size_t total = (size_t)K * N;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const size_t k = i / N, n = i - k * N;
    dst[k * ldd + col0 + n] = from_f32<TD>(to_f32(src[i]));
  }
}
__global__ void len_commit_kernel(int* len, const int* base, const int* n_accept, int cap_extra, int B) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < B) {
    int add = 1 + n_accept[b];
    if (add > cap_extra) add = cap_extra;      // never beyond what was written this round
    if (add < 1) add = 1;
    len[b] = base[b] + add;
  }
}
// len[b] = src[b] clamped to [0, hi]: the device values can never exceed the bound the host checks capacity with
__global__ void len_restore_kernel(const int* __restrict__ src, int* __restrict__ len, int B, int hi) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < B) len[b] = min(max(src[b], 0), hi);
}
__global__ void copy_i32_kernel(const int* src, int* dst, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src[i];
}
// Attention passes over the rows of a forward with more rows per sample than one attention workgroup holds: pass p
// takes rows [p cap, (p + 1) cap) of every sample.  start / cnt / len are [n_pass][B].
__global__ void attn_pass_kernel(const int* __restrict__ row_start, const int* __restrict__ cache_len, int B, int cap, int n_pass,
                                 int* __restrict__ start, int* __restrict__ cnt, int* __restrict__ len) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= B * n_pass) return;
  const int p = i / B, b = i - p * B;
  const int nq = row_start[b + 1] - row_start[b];
  const int lo = min(p * cap, nq);
  start[i] = row_start[b] + lo;
  cnt[i] = min(max(nq - lo, 0), cap);
  len[i] = cache_len[b] + lo;
}
// Prefill, one chunk: sample b contributes nq[b] = clamp(n[b] - c0, 0, chunk) rows.
__global__ void prefill_chunk_kernel(const int* __restrict__ n, int c0, int chunk, int* __restrict__ nq, int B) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < B) nq[b] = min(max(n[b] - c0, 0), chunk);
}
// Packed row (sample b, j) <- x[b, c0 + j, :]; its id is first_id[b] at position 0 of the prefix, else -1 (a
// latent row).  One workgroup per sample; the sample's first packed row is the sum of the counts before it.
__global__ __launch_bounds__(64) void prefill_pack_kernel(const float* __restrict__ x, int n_max, int D, int c0,
                                                          const int* __restrict__ nq, const int* __restrict__ first_id,
                                                          float* __restrict__ x_out, int* __restrict__ ids) {
  const int b = blockIdx.x, lane = threadIdx.x;
  int start = 0;
  for (int i = lane; i < b; i += 64) start += nq[i];
  for (int o = 32; o > 0; o >>= 1) start += __shfl_xor(start, o, 64);
  const int cnt = nq[b];
  for (int e = lane; e < cnt * D; e += 64) {
    const int j = e / D, k = e - j * D;
    x_out[(size_t)(start + j) * D + k] = x[((size_t)b * n_max + c0 + j) * D + k];
  }
  for (int j = lane; j < cnt; j += 64) ids[start + j] = (first_id && c0 + j == 0) ? first_id[b] : -1;
}
// z_last[b, :] <- the packed feature row of sample b's last prefix position, in the chunk that holds it.
template <typename T>
__global__ __launch_bounds__(64) void prefill_last_kernel(const T* __restrict__ z, int ldz, const int* __restrict__ n, int c0,
                                                          const int* __restrict__ nq, T* __restrict__ z_last) {
  const int b = blockIdx.x, lane = threadIdx.x;
  const int cnt = nq[b];
  if (cnt == 0 || c0 + cnt != n[b]) return;
  int start = 0;
  for (int i = lane; i < b; i += 64) start += nq[i];
  for (int o = 32; o > 0; o >>= 1) start += __shfl_xor(start, o, 64);
  for (int k = lane; k < ldz; k += 64) z_last[(size_t)b * ldz + k] = z[(size_t)(start + cnt - 1) * ldz + k];
}
// Folding a norm's affine part into the GEMM that follows it: scaled[k, n] = bf16(g[k] w[k, n]),
// cs[n] = sum_k scaled[k, n], bf[n] = b0[n] + sum_k beta[k] w[k, n].  One thread per column.
template <typename TS>
__global__ void ln_fold_kernel(const TS* __restrict__ w, const float* __restrict__ g, const float* __restrict__ beta,
                               const float* __restrict__ b0, int K, int N, bf16* __restrict__ scaled, float* __restrict__ cs,
                               float* __restrict__ bf) {
  const int n = blockIdx.x * blockDim.x + threadIdx.x;
  if (n >= N) return;
  float c = 0.f, bb = b0 ? b0[n] : 0.f;
  for (int k = 0; k < K; ++k) {
    const float wv = to_f32(w[(size_t)k * N + n]);
    const bf16 ws = (bf16)(g[k] * wv);
    scaled[(size_t)k * N + n] = ws;
    c += (float)ws;
    if (beta) bb = fmaf(beta[k], wv, bb);
  }
  cs[n] = c;
  bf[n] = bb;
}
// Multi-round generation as graph replays: the noise of round t is copied to fixed staging buffers before the round's
// graph, and the round's per-sample records are copied out after it.
__global__ void gen_stage_in_kernel(const float* __restrict__ eps, const float* __restrict__ r, const float* __restrict__ eres,
                                    const float* __restrict__ ures, size_t n_eps, size_t n_r, size_t n_eres, size_t n_ures,
                                    float* __restrict__ d_eps, float* __restrict__ d_r, float* __restrict__ d_eres,
                                    float* __restrict__ d_ures) {
  const size_t total = n_eps + n_r + n_eres + n_ures;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    if (i < n_eps) d_eps[i] = eps[i];
    else if (i < n_eps + n_r) d_r[i - n_eps] = r[i - n_eps];
    else if (i < n_eps + n_r + n_eres) d_eres[i - n_eps - n_r] = eres[i - n_eps - n_r];
    else d_ures[i - n_eps - n_r - n_eres] = ures[i - n_eps - n_r - n_eres];
  }
}
__global__ void gen_stage_out_kernel(const float* __restrict__ s_H, const int* __restrict__ s_nk, const int* __restrict__ s_na,
                                     const int* __restrict__ s_tr, int BK, int B, float* __restrict__ H, int* __restrict__ nk,
                                     int* __restrict__ na, int* __restrict__ tr) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < BK) H[i] = s_H[i];
  if (i < B) {
    nk[i] = s_nk[i];
    na[i] = s_na[i];
    tr[i] = s_tr[i];
  }
}
__global__ void temb_feat_kernel(float t, float t_scale, int half, float* out) {
  const int k = blockIdx.x * blockDim.x + threadIdx.x;
  if (k < half) {
    const float omega = powf(10000.0f, -(float)k / (float)half);
    const float arg = t * t_scale * omega;
    out[k] = cosf(arg);
    out[half + k] = sinf(arg);
  }
}
__global__ void mean_heads_kernel(const float* __restrict__ ent_heads, int n_heads, float* __restrict__ out, int M,
                                  const int* m_dev) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r < eff_rows(M, m_dev)) {
    float s = 0.f;
    for (int g = 0; g < n_heads; ++g) s += ent_heads[(size_t)r * n_heads + g];
    out[r] = s / (float)n_heads;
  }
}

// ------------------------------------------------------------------------------ context
struct LayerW {
  float *n1g = nullptr, *n1b = nullptr, *n2g = nullptr, *n2b = nullptr;
  void *wqkv = nullptr, *wo = nullptr, *w1 = nullptr, *w2 = nullptr;   // w1 = up (GELU) or gate|up (SwiGLU), w2 = down
  float *bqkv = nullptr, *bo = nullptr, *b1 = nullptr, *b2 = nullptr;
  // norm 2 folded into the up-projection (bf16, GELU layers): diag(n2g) w1 packed, its column sums, b1 + n2b w1
  void* w1f = nullptr;
  float *cs1 = nullptr, *b1f = nullptr;
};
struct Model {
  fard_tf_cfg c;
  void *in_w = nullptr, *pos = nullptr, *cond = nullptr, *up = nullptr;
  float *in_b = nullptr, *nfg = nullptr, *nfb = nullptr;
  std::vector<LayerW> L;
  void *kc = nullptr, *vc = nullptr;       // [layer][B][Hkv][ctx_pad][dh]
  size_t layer_elems = 0;
  int ctx_pad = 0;
  int *len = nullptr, *len_base = nullptr; // device [max_batch]
  int len_hi = 0;                          // host upper bound of any sample's length
  int written = 0;                         // rows per sample written since len_base was recorded
  int d_out() const { return c.d_out ? c.d_out : c.d_model; }
  int qkv_n() const { return (c.n_heads + 2 * c.n_kv_heads) * c.d_head; }
};
struct BlockW {
  void *w1 = nullptr, *w2 = nullptr;
  float *b1 = nullptr, *b2 = nullptr;
};
struct HeadW {
  void *in_w = nullptr, *c_w = nullptr, *mod_all = nullptr, *out_w = nullptr;
  float *in_b = nullptr, *c_b = nullptr, *mod_b_all = nullptr, *out_b = nullptr, *temb = nullptr;
  std::vector<BlockW> B;
  int mod_n = 0;
  // bf16 path: per block j the mod GEMM also yields c0_j = shift_j W1_j and c1_j = (1 + scale_j) W1_j (columns
  // fold_base + 2 w j and + w), so that the block's modulated norm can be folded into its first GEMM; 0: not built
  int fold_base = 0;
};
struct Prof {
  bool on = false;
  std::vector<std::pair<hipEvent_t, hipEvent_t>> pool;
  std::vector<int> cls;
  size_t used = 0;
  double flops[5] = {0, 0, 0, 0, 0}, bytes[5] = {0, 0, 0, 0, 0};
};

// A captured round: spec_round called again with the arguments of `key` replays `exec` instead of launching
// its kernels one by one.
struct RoundKey {
  const void* ptr[13];
  float f[4];
  int32_t B;
  int32_t pad;
};
struct RoundGraph {
  bool on = false;
  bool have_key = false;                   // key = the arguments of the last eager spec_round call
  RoundKey key;
  hipGraph_t graph = nullptr;
  hipGraphExec_t exec = nullptr;           // non-null: replays key
  void drop() {
    if (exec) (void)hipGraphExecDestroy(exec);
    if (graph) (void)hipGraphDestroy(graph);
    exec = nullptr;
    graph = nullptr;
    have_key = false;
  }
};

}  // namespace

struct fard_ctx {
  fard_round_cfg cfg;
  hipStream_t stream = nullptr;
  int bf16 = 1;
  size_t esz = 2;
  int m_max = 0;                           // rows of a round: max_batch * (K + 1)
  int m_rows = 0;                          // rows of the transformer workspace: max_batch * max(K + 1, prefill chunk)
  int *pf_n = nullptr, *pf_nq = nullptr;   // prefill: prefix lengths and the current chunk's row counts
  int *ap_start = nullptr, *ap_cnt = nullptr, *ap_len = nullptr;   // attention passes [n_pass][B], ap_max entries each
  int ap_max = 0;
  Model mdl[2];
  HeadW head;
  std::vector<void*> allocs;
  std::string err;
  Prof prof;
  // workspace
  float *h = nullptr, *x_in = nullptr, *ent_heads = nullptr, *h_row = nullptr;
  void* hv = nullptr;            // head: bf16 rows h (1 + scale of the next block), written by a block's second GEMM
  float* hmom = nullptr;         // head: [rows][w / 16] (mean, centred squares) of h per 16-column tile
  void *u = nullptr, *qkv = nullptr, *ao = nullptr, *ff = nullptr, *z = nullptr, *ztmp = nullptr;
  RowMaps maps{};
  int *aux_row = nullptr, *row_ids = nullptr;
  float* x_scratch = nullptr;
  // multi-round generation: outputs of the current round, the closing token, catch-up rows
  float *g_x = nullptr, *g_mu_q = nullptr, *g_mu_p = nullptr, *g_lr = nullptr, *g_next = nullptr, *g_cu_x = nullptr;
  int* g_cu_nq = nullptr;
  uint8_t* g_keep = nullptr;
  // deferred residual update: K-slice partial sums of the last down-projection, folded in by the next norm
  // keys of one (sample, kv head) split over several attention workgroups: their partial results (see AttnSplit)
  float *attn_o = nullptr, *attn_mla = nullptr;
  int attn_rows = 0;
  float* parts = nullptr;
  size_t parts_cap = 0;                    // floats that parts holds
  int pend_n = 0;
  size_t pend_stride = 0;
  RoundGraph rgraph;
  RoundGraph ggraph;                       // one round of spec_generate on the staging buffers below
  float *s_eps = nullptr, *s_r = nullptr, *s_eres = nullptr, *s_ures = nullptr, *s_H = nullptr;
  int *s_pid = nullptr, *s_nk = nullptr, *s_na = nullptr, *s_tr = nullptr;
  void* loss_tmp = nullptr;                // scratch of the training-side losses, grown on demand
  size_t loss_tmp_bytes = 0;
  uint8_t* acc_tmp = nullptr;
  float *cz = nullptr, *hh = nullptr, *mod = nullptr, *xt = nullptr;
  void *sc = nullptr, *a1 = nullptr, *a2 = nullptr;
  int *alive = nullptr, *act_idx = nullptr, *n_act = nullptr, *emap = nullptr, *omap = nullptr;
  int* ent_blk = nullptr;
  void* gemm_tmp = nullptr;
  size_t gemm_tmp_bytes = 0;
};

namespace {

int fail(fard_ctx* c, int code, const std::string& msg) {
  if (c) c->err = msg;
  return code;
}
#define HIPCHK(ctx, expr)                                                                      \
  do {                                                                                         \
    hipError_t e__ = (expr);                                                                   \
    if (e__ != hipSuccess)                                                                     \
      return fail(ctx, FARD_EHIP, std::string(#expr) + ": " + hipGetErrorString(e__));         \
  } while (0)

template <typename T>
int dalloc(fard_ctx* c, T** p, size_t count) {
  void* q = nullptr;
  size_t bytes = count * sizeof(T);
  if (bytes == 0) bytes = 16;
  hipError_t e = hipMalloc(&q, bytes);
  if (e != hipSuccess) return fail(c, FARD_ENOMEM, std::string("hipMalloc: ") + hipGetErrorString(e));
  c->allocs.push_back(q);
  *p = (T*)q;
  return FARD_OK;
}
int dalloc_bytes(fard_ctx* c, void** p, size_t bytes) {
  char* q = nullptr;
  int rc = dalloc<char>(c, &q, bytes);
  *p = q;
  return rc;
}

// Launch bracket: when profiling is on, every launch of a class sits between two events.
struct Bracket {
  fard_ctx* c;
  int cls;
  size_t slot = (size_t)-1;
  Bracket(fard_ctx* ctx, int k, double fl = 0, double by = 0) : c(ctx), cls(k) {
    Prof& p = c->prof;
    if (!p.on) return;
    if (p.used == p.pool.size()) {
      hipEvent_t a, b;
      if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return;
      p.pool.push_back({a, b});
      p.cls.push_back(0);
    }
    slot = p.used++;
    p.cls[slot] = k;
    p.flops[k] += fl;
    p.bytes[k] += by;
    (void)hipEventRecord(p.pool[slot].first, c->stream);
  }
  ~Bracket() {
    if (slot != (size_t)-1) (void)hipEventRecord(c->prof.pool[slot].second, c->stream);
  }
};
enum { CLS_GEMM = 0, CLS_ATTN = 1, CLS_ENT = 2, CLS_OTHER = 3, CLS_GEMM_NARROW = 4, CLS_COUNT = 5 };

// ------------------------------------------------------------------------------ weight upload
struct Loader {
  fard_ctx* c;
  std::map<std::string, const fard_tensor*> byname;
  std::vector<void*> staging;

  const fard_tensor* find(const std::string& n) const {
    auto it = byname.find(n);
    return it == byname.end() ? nullptr : it->second;
  }
  // device pointer to the tensor's data (uploads host tensors to a staging buffer)
  int device_src(const fard_tensor* t, const void** out) {
    if (t->on_device) { *out = t->data; return FARD_OK; }
    const size_t bytes = (size_t)t->numel * (t->dtype == FARD_BF16 ? 2 : 4);
    void* p = nullptr;
    hipError_t e = hipMalloc(&p, bytes ? bytes : 16);
    if (e != hipSuccess) return fail(c, FARD_ENOMEM, "staging hipMalloc failed");
    staging.push_back(p);
    HIPCHK(c, hipMemcpy(p, t->data, bytes, hipMemcpyHostToDevice));
    *out = p;
    return FARD_OK;
  }
  void release_staging() {
    (void)hipStreamSynchronize(c->stream);
    for (void* p : staging) (void)hipFree(p);
    staging.clear();
  }
  int need(const std::string& n, int64_t numel, const fard_tensor** out) {
    const fard_tensor* t = find(n);
    if (!t) return fail(c, FARD_EINVAL, "missing weight " + n);
    if (t->numel != numel)
      return fail(c, FARD_ESHAPE, "weight " + n + ": numel " + std::to_string(t->numel) + " != " + std::to_string(numel));
    if (t->dtype != FARD_F32 && t->dtype != FARD_BF16) return fail(c, FARD_EINVAL, "weight " + n + ": bad dtype");
    if (!t->data) return fail(c, FARD_EINVAL, "weight " + n + ": null data");
    *out = t;
    return FARD_OK;
  }
  // fp32 vector; optional (absent -> filled with `dflt`, or nullptr when allow_null)
  int vec(const std::string& n, int64_t numel, float dflt, bool required, float** out) {
    const fard_tensor* t = find(n);
    if (!t) {
      if (required) return fail(c, FARD_EINVAL, "missing weight " + n);
      int rc = dalloc<float>(c, out, (size_t)numel);
      if (rc) return rc;
      HIPCHK(c, launch_fill_f32(c->stream, *out, dflt, (size_t)numel));
      return FARD_OK;
    }
    int rc = need(n, numel, &t);
    if (rc) return rc;
    const void* src;
    if ((rc = device_src(t, &src))) return rc;
    if ((rc = dalloc<float>(c, out, (size_t)numel))) return rc;
    const unsigned blocks = (unsigned)std::min<size_t>(((size_t)numel + 255) / 256, 4096);
    if (t->dtype == FARD_BF16)
      convert_kernel<bf16, float><<<blocks, 256, 0, c->stream>>>((const bf16*)src, *out, (size_t)numel);
    else
      convert_kernel<float, float><<<blocks, 256, 0, c->stream>>>((const float*)src, *out, (size_t)numel);
    HIPCHK(c, hipGetLastError());
    return FARD_OK;
  }
  // table in storage type, row-major as given
  int table(const std::string& n, int64_t numel, void** out) {
    const fard_tensor* t;
    int rc = need(n, numel, &t);
    if (rc) return rc;
    const void* src;
    if ((rc = device_src(t, &src))) return rc;
    if ((rc = dalloc_bytes(c, out, (size_t)numel * c->esz))) return rc;
    const unsigned blocks = (unsigned)std::min<size_t>(((size_t)numel + 255) / 256, 4096);
    const size_t n_ = (size_t)numel;
    if (c->bf16) {
      if (t->dtype == FARD_BF16) convert_kernel<bf16, bf16><<<blocks, 256, 0, c->stream>>>((const bf16*)src, (bf16*)*out, n_);
      else convert_kernel<float, bf16><<<blocks, 256, 0, c->stream>>>((const float*)src, (bf16*)*out, n_);
    } else {
      if (t->dtype == FARD_BF16) convert_kernel<bf16, float><<<blocks, 256, 0, c->stream>>>((const bf16*)src, (float*)*out, n_);
      else convert_kernel<float, float><<<blocks, 256, 0, c->stream>>>((const float*)src, (float*)*out, n_);
    }
    HIPCHK(c, hipGetLastError());
    return FARD_OK;
  }
  // GEMM operand: a list of [K, N_i] matrices laid side by side along N (interleave = 32-column
  // blocks of two matrices alternate, for the SwiGLU epilogue).
  int gemm_weight(const std::vector<std::string>& names, int K, const std::vector<int>& Ns, bool interleave, void** out) {
    int Ntot = 0;
    for (int n : Ns) Ntot += n;
    int rc = dalloc_bytes(c, out, (size_t)K * Ntot * c->esz);
    if (rc) return rc;
    int col0 = 0;
    for (size_t i = 0; i < names.size(); ++i) {
      const fard_tensor* t;
      if ((rc = need(names[i], (int64_t)K * Ns[i], &t))) return rc;
      const void* src;
      if ((rc = device_src(t, &src))) return rc;
      if (c->bf16) {
        if (K % 64 != 0 || Ns[i] % 32 != 0)
          return fail(c, FARD_ESHAPE, "weight " + names[i] + ": bf16 GEMM needs K % 64 == 0 and N % 32 == 0");
        const int off = interleave ? (int)i : col0 / 32;
        const int stride = interleave ? (int)names.size() : 1;
        HIPCHK(c, launch_pack_weight(c->stream, src, t->dtype == FARD_BF16, Ns[i], K, Ns[i], *out, off, stride));
      } else {
        const size_t total = (size_t)K * Ns[i];
        const unsigned blocks = (unsigned)std::min<size_t>((total + 255) / 256, 4096);
        if (t->dtype == FARD_BF16)
          place_kernel<bf16, float><<<blocks, 256, 0, c->stream>>>((const bf16*)src, (float*)*out, K, Ns[i], Ntot, col0);
        else
          place_kernel<float, float><<<blocks, 256, 0, c->stream>>>((const float*)src, (float*)*out, K, Ns[i], Ntot, col0);
        HIPCHK(c, hipGetLastError());
      }
      col0 += Ns[i];
      // keep peak staging memory low for the big models
      if (staging.size() > 8) release_staging();
    }
    return FARD_OK;
  }
};

// w1f / cs1 / b1f of a layer (see LayerW) from the layer's w1 [K, N], norm gain g, norm bias beta (or null), b1 (or null).
int fold_norm_into(fard_ctx* c, Loader& ld, const std::string& name, int K, int N, const float* g, const float* beta,
                   const float* b0, void** w_out, float** cs_out, float** bf_out) {
  const fard_tensor* t;
  int rc = ld.need(name, (int64_t)K * N, &t);
  if (rc) return rc;
  const void* src;
  if ((rc = ld.device_src(t, &src))) return rc;
  void* scaled = nullptr;
  if (hipMalloc(&scaled, (size_t)K * N * 2) != hipSuccess) return fail(c, FARD_ENOMEM, "staging hipMalloc failed");
  ld.staging.push_back(scaled);
  if ((rc = dalloc_bytes(c, w_out, (size_t)K * N * 2)) || (rc = dalloc<float>(c, cs_out, (size_t)N)) ||
      (rc = dalloc<float>(c, bf_out, (size_t)N)))
    return rc;
  const unsigned blocks = (unsigned)((N + 127) / 128);
  if (t->dtype == FARD_BF16)
    ln_fold_kernel<bf16><<<blocks, 128, 0, c->stream>>>((const bf16*)src, g, beta, b0, K, N, (bf16*)scaled, *cs_out, *bf_out);
  else
    ln_fold_kernel<float><<<blocks, 128, 0, c->stream>>>((const float*)src, g, beta, b0, K, N, (bf16*)scaled, *cs_out, *bf_out);
  HIPCHK(c, hipGetLastError());
  HIPCHK(c, launch_pack_weight(c->stream, scaled, 1, N, K, N, *w_out, 0, 1));
  if (ld.staging.size() > 8) ld.release_staging();
  return FARD_OK;
}

int check_tf(fard_ctx* c, const fard_tf_cfg& t, const char* who) {
  std::string w(who);
  if (t.n_layers < 1 || t.d_model < 1 || t.n_heads < 1 || t.n_kv_heads < 1 || t.d_head < 1 || t.d_ff < 1 || t.d_latent < 1)
    return fail(c, FARD_EINVAL, w + ": non-positive size");
  if (t.n_heads % t.n_kv_heads != 0) return fail(c, FARD_ESHAPE, w + ": n_heads % n_kv_heads != 0");
  if (t.d_latent > 16) return fail(c, FARD_ESHAPE, w + ": d_latent > 16 unsupported");
  if (t.d_head % 2 != 0) return fail(c, FARD_ESHAPE, w + ": odd d_head");
  if (c->bf16) {
    if (t.d_head != 32 && t.d_head != 64 && t.d_head != 128) return fail(c, FARD_ESHAPE, w + ": bf16 d_head must be 32, 64 or 128");
    if (t.d_model % 64 != 0 || t.d_ff % 64 != 0 || (t.n_heads * t.d_head) % 64 != 0)
      return fail(c, FARD_ESHAPE, w + ": bf16 widths must be multiples of 64");
    if (t.d_out && t.d_out % 32 != 0) return fail(c, FARD_ESHAPE, w + ": d_out % 32 != 0");
  }
  if (t.act != FARD_ACT_GELU && t.act != FARD_ACT_SWIGLU) return fail(c, FARD_EINVAL, w + ": act");
  if (t.norm != FARD_NORM_LAYER && t.norm != FARD_NORM_RMS) return fail(c, FARD_EINVAL, w + ": norm");
  if (t.pos != FARD_POS_LEARNED && t.pos != FARD_POS_ROPE) return fail(c, FARD_EINVAL, w + ": pos");
  if (t.pos == FARD_POS_LEARNED && t.max_pos < 1) return fail(c, FARD_EINVAL, w + ": learned positions need max_pos");
  return FARD_OK;
}

int load_model(fard_ctx* c, Loader& ld, int which) {
  Model& m = c->mdl[which];
  const fard_tf_cfg& t = m.c;
  const std::string p = which == FARD_TARGET ? "target." : "draft.";
  const int d = t.d_model, F = t.d_ff, D = t.d_latent, HD = t.n_heads * t.d_head, QN = m.qkv_n();
  int rc;
  if ((rc = ld.table(p + "in.w", (int64_t)D * d, &m.in_w))) return rc;
  if ((rc = ld.vec(p + "in.b", d, 0.f, false, &m.in_b))) return rc;
  if (t.pos == FARD_POS_LEARNED && (rc = ld.table(p + "pos", (int64_t)t.max_pos * d, &m.pos))) return rc;
  if (t.n_cond_ids > 0 && (rc = ld.table(p + "cond", (int64_t)t.n_cond_ids * d, &m.cond))) return rc;
  m.L.resize(t.n_layers);
  const bool ln = t.norm == FARD_NORM_LAYER;
  for (int i = 0; i < t.n_layers; ++i) {
    LayerW& L = m.L[i];
    const std::string q = p + "L" + std::to_string(i) + ".";
    if ((rc = ld.vec(q + "n1.g", d, 1.f, false, &L.n1g))) return rc;
    if ((rc = ld.vec(q + "n2.g", d, 1.f, false, &L.n2g))) return rc;
    if (ln) {
      if ((rc = ld.vec(q + "n1.b", d, 0.f, false, &L.n1b))) return rc;
      if ((rc = ld.vec(q + "n2.b", d, 0.f, false, &L.n2b))) return rc;
    }
    if ((rc = ld.gemm_weight({q + "wqkv"}, d, {QN}, false, &L.wqkv))) return rc;
    if ((rc = ld.gemm_weight({q + "wo"}, HD, {d}, false, &L.wo))) return rc;
    if (t.has_bias) {
      if ((rc = ld.vec(q + "bqkv", QN, 0.f, false, &L.bqkv))) return rc;
      if ((rc = ld.vec(q + "bo", d, 0.f, false, &L.bo))) return rc;
    }
    if (t.act == FARD_ACT_GELU) {
      if ((rc = ld.gemm_weight({q + "w1"}, d, {F}, false, &L.w1))) return rc;
      if ((rc = ld.gemm_weight({q + "w2"}, F, {d}, false, &L.w2))) return rc;
      if (t.has_bias) {
        if ((rc = ld.vec(q + "b1", F, 0.f, false, &L.b1))) return rc;
        if ((rc = ld.vec(q + "b2", d, 0.f, false, &L.b2))) return rc;
      }
      if (c->bf16 && (rc = fold_norm_into(c, ld, q + "w1", d, F, L.n2g, ln ? L.n2b : nullptr, L.b1, &L.w1f, &L.cs1, &L.b1f)))
        return rc;
    } else {
      if ((rc = ld.gemm_weight({q + "wg", q + "wu"}, d, {F, F}, true, &L.w1))) return rc;
      if ((rc = ld.gemm_weight({q + "wd"}, F, {d}, false, &L.w2))) return rc;
    }
  }
  if ((rc = ld.vec(p + "nf.g", d, 1.f, false, &m.nfg))) return rc;
  if (ln && (rc = ld.vec(p + "nf.b", d, 0.f, false, &m.nfb))) return rc;
  if (t.d_out && t.d_out != d && (rc = ld.gemm_weight({p + "up.w"}, d, {t.d_out}, false, &m.up))) return rc;

  // KV cache, zeroed: masked positions multiply V by an exact 0, which needs finite V
  m.ctx_pad = c->bf16 ? ((c->cfg.max_ctx + 31) / 32) * 32 : c->cfg.max_ctx;
  m.layer_elems = (size_t)c->cfg.max_batch * t.n_kv_heads * m.ctx_pad * t.d_head;
  const size_t bytes = m.layer_elems * t.n_layers * c->esz;
  if ((rc = dalloc_bytes(c, &m.kc, bytes))) return rc;
  if ((rc = dalloc_bytes(c, &m.vc, bytes))) return rc;
  HIPCHK(c, hipMemsetAsync(m.kc, 0, bytes, c->stream));
  HIPCHK(c, hipMemsetAsync(m.vc, 0, bytes, c->stream));
  if ((rc = dalloc<int>(c, &m.len, c->cfg.max_batch))) return rc;
  if ((rc = dalloc<int>(c, &m.len_base, c->cfg.max_batch))) return rc;
  HIPCHK(c, launch_fill_i32(c->stream, m.len, 0, c->cfg.max_batch));
  HIPCHK(c, launch_fill_i32(c->stream, m.len_base, 0, c->cfg.max_batch));
  m.len_hi = 0;
  return FARD_OK;
}

// Which GEMMs of the bf16 path go to the narrow-tile kernel (no K split, no atomics, any epilogue).
bool routes_narrow(int M, int N, int K, int epi) {
  if (epi == EPI_SWIGLU || N % 32 != 0 || K % 64 != 0 || M < 1) return false;
  // a few dozen rows against a weight matrix that 16-column tiles spread over enough workgroups: the
  // narrow-tile kernel finishes in one memory round trip
  if (M <= 64 && K <= 2048 && N <= 8192) return true;
  // up to about 300 rows against a small square-ish matrix: still ahead of the streaming kernel's 32-row tiles
  // (measured at 288 x 1024 x 1024: 6.0-6.4 us against 6.2-6.9; at 576 x 1280 x 1280 13 us against 8-9)
  if (M <= 320 && K <= 1536 && N <= 1536) return true;
  // ... or a wide one with a store epilogue, through 64-column workgroups
  if (M <= 640 && K <= 1024 && N <= 8192 && N % 64 == 0 && (epi == EPI_STORE || epi == EPI_STORE_F32)) return true;
  return false;
}

// Extras of the narrow kernel: a bf16 copy of a residual update; the preceding norm applied in the epilogue.
struct GemmExtra {
  void* copy_bf16 = nullptr;
  const float* ln_cs = nullptr;
  float ln_eps = 0.f;
  int ln_rms = 0;
  // modulated-norm fold (GemmArgs): producer side, consumer side
  const float* copy_scale = nullptr;
  int copy_ld = 0;
  float* mom_out = nullptr;
  int mom_ld = 0;
  const float *ada_mom = nullptr, *ada_c1 = nullptr, *ada_c0 = nullptr;
  int ada_mom_ld = 0, ada_ld = 0;
  float ada_eps = 0.f;
  int a_tiled = 0, out_tiled = 0;
};

hipError_t gemm(fard_ctx* c, const void* A, int lda, const void* W, const float* bias, void* out, int ldo, int M,
                int N, int K, const int* m_dev, int epi, int act, const float* gate = nullptr, int ldg = 0,
                const GemmExtra* ex = nullptr) {
  GemmArgs a;
  a.A = A; a.lda = lda; a.W = W; a.bias = bias; a.out = out; a.ldo = ldo; a.gate = gate; a.ldg = ldg;
  a.M = M; a.N = N; a.K = K; a.m_dev = m_dev; a.act = act; a.epi = epi;
  if (ex) {
    if (!c->bf16 || !routes_narrow(M, N, K, epi)) return hipErrorInvalidValue;   // only the narrow kernel has them
    a.copy_bf16 = ex->copy_bf16; a.ln_cs = ex->ln_cs; a.ln_eps = ex->ln_eps; a.ln_rms = ex->ln_rms;
    a.copy_scale = ex->copy_scale; a.copy_ld = ex->copy_ld; a.mom_out = ex->mom_out; a.mom_ld = ex->mom_ld;
    a.ada_mom = ex->ada_mom; a.ada_mom_ld = ex->ada_mom_ld; a.ada_c1 = ex->ada_c1; a.ada_c0 = ex->ada_c0; a.ada_ld = ex->ada_ld;
    a.ada_eps = ex->ada_eps; a.a_tiled = ex->a_tiled; a.out_tiled = ex->out_tiled;
  }
  const double fl = 2.0 * M * (double)N * K;
  const double by = (double)K * N * c->esz + (double)M * K * c->esz + (double)M * (epi == EPI_SWIGLU ? N / 2 : N) * 4;
  const bool narrow = c->bf16 && routes_narrow(M, N, K, epi) && narrow_supported(a);
  if (ex && !narrow) return hipErrorInvalidValue;
  Bracket br(c, narrow ? CLS_GEMM_NARROW : CLS_GEMM, fl, by);
  if (!c->bf16) return launch_gemm_f32(c->stream, a);
  if (narrow) return launch_gemm_narrow(c->stream, a);
  return launch_gemm_bf16(c->stream, a);
}

int load_head(fard_ctx* c, Loader& ld) {
  const fard_head_cfg& hc = c->cfg.head;
  HeadW& hw = c->head;
  const int w = hc.width, D = hc.d_latent, Nb = hc.n_blocks, S = hc.n_steps;
  int rc;
  if ((rc = ld.table("head.in.w", (int64_t)D * w, &hw.in_w))) return rc;
  if ((rc = ld.vec("head.in.b", w, 0.f, false, &hw.in_b))) return rc;
  if ((rc = ld.gemm_weight({"head.c.w"}, hc.d_cond, {w}, false, &hw.c_w))) return rc;
  if ((rc = ld.vec("head.c.b", w, 0.f, false, &hw.c_b))) return rc;
  // all modulation projections share their input silu(c): one wide GEMM [w, (3 Nb + 2) w]; on the bf16 path 2 Nb w
  // more columns follow (fold_base), see below
  const bool fold = c->bf16 && w % 64 == 0 && w <= 2048;
  std::vector<std::string> names;
  std::vector<int> Ns;
  for (int j = 0; j < Nb; ++j) { names.push_back("head.B" + std::to_string(j) + ".mod.w"); Ns.push_back(3 * w); }
  names.push_back("head.f.mod.w");
  Ns.push_back(2 * w);
  const int base_n = (3 * Nb + 2) * w;
  hw.mod_n = base_n + (fold ? 2 * Nb * w : 0);
  hw.fold_base = fold ? base_n : 0;
  if (!fold) {
    if ((rc = ld.gemm_weight(names, w, Ns, false, &hw.mod_all))) return rc;
  } else {
    if ((rc = dalloc_bytes(c, &hw.mod_all, (size_t)w * hw.mod_n * c->esz))) return rc;
    int col0 = 0;
    for (size_t i = 0; i < names.size(); ++i) {
      const fard_tensor* t;
      if ((rc = ld.need(names[i], (int64_t)w * Ns[i], &t))) return rc;
      const void* src;
      if ((rc = ld.device_src(t, &src))) return rc;
      HIPCHK(c, launch_pack_weight(c->stream, src, t->dtype == FARD_BF16, Ns[i], w, Ns[i], hw.mod_all, col0 / 32, 1));
      col0 += Ns[i];
      if (ld.staging.size() > 8) ld.release_staging();
    }
  }
  if ((rc = dalloc<float>(c, &hw.mod_b_all, hw.mod_n))) return rc;
  HIPCHK(c, launch_fill_f32(c->stream, hw.mod_b_all, 0.f, hw.mod_n));
  for (int j = 0; j <= Nb; ++j) {
    const std::string n = j < Nb ? "head.B" + std::to_string(j) + ".mod.b" : std::string("head.f.mod.b");
    const int cnt = j < Nb ? 3 * w : 2 * w;
    if (!ld.find(n)) continue;
    float* tmp;
    if ((rc = ld.vec(n, cnt, 0.f, true, &tmp))) return rc;
    HIPCHK(c, hipMemcpyAsync(hw.mod_b_all + (size_t)3 * w * j, tmp, (size_t)cnt * 4, hipMemcpyDeviceToDevice, c->stream));
  }
  hw.B.resize(Nb);
  for (int j = 0; j < Nb; ++j) {
    const std::string q = "head.B" + std::to_string(j) + ".";
    if ((rc = ld.gemm_weight({q + "w1"}, w, {w}, false, &hw.B[j].w1))) return rc;
    if ((rc = ld.gemm_weight({q + "w2"}, w, {w}, false, &hw.B[j].w2))) return rc;
    if ((rc = ld.vec(q + "b1", w, 0.f, false, &hw.B[j].b1))) return rc;
    if ((rc = ld.vec(q + "b2", w, 0.f, false, &hw.B[j].b2))) return rc;
  }
  if ((rc = ld.table("head.out.w", (int64_t)w * D, &hw.out_w))) return rc;
  if ((rc = ld.vec("head.out.b", D, 0.f, false, &hw.out_b))) return rc;

  if (fold) {
    // The modulated norm of block j, a1 = LN(h)(1 + scale) + shift, times W1 with the row-wise factors outside the sum:
    //   a1 W1 = rstd ((h (1 + scale)) W1 - mean (1 + scale) W1) + shift W1.
    // (1 + scale) W1 and shift W1 are affine in the conditioning s = silu(c) like scale and shift themselves
    // (scale = s Wsc + bsc): (1 + scale) W1 = s (Wsc W1) + (1 + bsc) W1, shift W1 = s (Wsh W1) + bsh W1.  The products
    // Wsc W1 and Wsh W1 are formed here, once, and packed as further columns of the mod GEMM.
    void *tmod = nullptr, *tw1 = nullptr, *tf = nullptr;
    float *ones = nullptr, *tv = nullptr;
    HIPCHK(c, hipMalloc(&tmod, (size_t)w * 3 * w * 2));
    HIPCHK(c, hipMalloc(&tw1, (size_t)w * w * 2));
    HIPCHK(c, hipMalloc(&tf, (size_t)w * w * 2));
    HIPCHK(c, hipMalloc((void**)&ones, (size_t)w * 4));
    HIPCHK(c, hipMalloc((void**)&tv, (size_t)w * 4));
    HIPCHK(c, launch_fill_f32(c->stream, ones, 1.f, (size_t)w));
    auto to_bf16 = [&](const std::string& name, int64_t numel, void* dst) -> int {
      const fard_tensor* t;
      int r = ld.need(name, numel, &t);
      if (r) return r;
      const void* src;
      if ((r = ld.device_src(t, &src))) return r;
      const unsigned blocks = (unsigned)std::min<size_t>(((size_t)numel + 255) / 256, 4096);
      if (t->dtype == FARD_BF16) convert_kernel<bf16, bf16><<<blocks, 256, 0, c->stream>>>((const bf16*)src, (bf16*)dst, (size_t)numel);
      else convert_kernel<float, bf16><<<blocks, 256, 0, c->stream>>>((const float*)src, (bf16*)dst, (size_t)numel);
      HIPCHK(c, hipGetLastError());
      return FARD_OK;
    };
    for (int j = 0; j < Nb && rc == FARD_OK; ++j) {
      const std::string q = "head.B" + std::to_string(j) + ".";
      if ((rc = to_bf16(q + "mod.w", (int64_t)w * 3 * w, tmod))) break;
      if ((rc = to_bf16(q + "w1", (int64_t)w * w, tw1))) break;
      float* bj = hw.mod_b_all + (size_t)3 * w * j;                      // shift, scale, gate biases of block j
      float* fb = hw.mod_b_all + (size_t)hw.fold_base + (size_t)2 * w * j;   // c0, c1 biases
      for (int which = 0; which < 2; ++which) {                          // 0: shift -> c0, 1: scale -> c1
        GemmArgs a;
        a.A = (const bf16*)tmod + (size_t)which * w; a.lda = 3 * w; a.W = hw.B[j].w1; a.bias = nullptr; a.out = tf; a.ldo = w;
        a.gate = nullptr; a.ldg = 0; a.M = w; a.N = w; a.K = w; a.m_dev = nullptr; a.act = ACT_NONE; a.epi = EPI_STORE;
        HIPCHK(c, launch_gemm_bf16(c->stream, a));
        HIPCHK(c, launch_pack_weight(c->stream, tf, 1, w, w, w, hw.mod_all, (hw.fold_base + 2 * w * j + which * w) / 32, 1));
        // bias row: bsh W1, or (1 + bsc) W1 = ones W1 + bsc W1
        HIPCHK(c, launch_matvec(c->stream, 1, bj + (size_t)which * w, tw1, nullptr, w, w, ACT_NONE, which ? tv : fb));
        if (which) HIPCHK(c, launch_matvec(c->stream, 1, ones, tw1, tv, w, w, ACT_NONE, fb + w));
      }
      ld.release_staging();
    }
    (void)hipStreamSynchronize(c->stream);
    (void)hipFree(tmod); (void)hipFree(tw1); (void)hipFree(tf); (void)hipFree(ones); (void)hipFree(tv);
    if (rc) return rc;
  }

  // time embedding of the S fixed sampler times t_k = 1 - k/S, computed once
  void *t1w, *t2w;
  float *t1b, *t2b, *feat, *hid;
  if ((rc = ld.table("head.t1.w", (int64_t)hc.t_freq_dim * w, &t1w))) return rc;
  if ((rc = ld.table("head.t2.w", (int64_t)w * w, &t2w))) return rc;
  if ((rc = ld.vec("head.t1.b", w, 0.f, false, &t1b))) return rc;
  if ((rc = ld.vec("head.t2.b", w, 0.f, false, &t2b))) return rc;
  if ((rc = dalloc<float>(c, &feat, hc.t_freq_dim))) return rc;
  if ((rc = dalloc<float>(c, &hid, w))) return rc;
  if ((rc = dalloc<float>(c, &hw.temb, (size_t)S * w))) return rc;
  for (int k = 0; k < S; ++k) {
    const float t = 1.0f - (float)k / (float)S;
    const int half = hc.t_freq_dim / 2;
    temb_feat_kernel<<<(half + 255) / 256, 256, 0, c->stream>>>(t, hc.t_scale, half, feat);
    HIPCHK(c, hipGetLastError());
    HIPCHK(c, launch_matvec(c->stream, c->bf16, feat, t1w, t1b, hc.t_freq_dim, w, ACT_SILU, hid));
    HIPCHK(c, launch_matvec(c->stream, c->bf16, hid, t2w, t2b, w, w, ACT_NONE, hw.temb + (size_t)k * w));
  }
  return FARD_OK;
}

constexpr int GEN_J_MAX = 64;            // resampling tries that the staged (graph) generation path holds
constexpr int PART_MAX_SLICES = 16;     // K slices of a deferred residual update
constexpr int PART_MAX_ROWS = 640;
constexpr int ATTN_MAX_SPLIT = 8;        // attention workgroups per (sample, kv head) at most

int cap_nq(const fard_ctx* c, int which);

int alloc_workspace(fard_ctx* c) {
  const fard_round_cfg& g = c->cfg;
  const int M = c->m_max, MR = c->m_rows;
  int dmax = 0, qmax = 0, hdmax = 0, fmax = 0, omax = 0, hmax = 0;
  for (int i = 0; i < 2; ++i) {
    const Model& m = c->mdl[i];
    dmax = std::max(dmax, m.c.d_model);
    qmax = std::max(qmax, m.qkv_n());
    hdmax = std::max(hdmax, m.c.n_heads * m.c.d_head);
    fmax = std::max(fmax, m.c.d_ff);
    omax = std::max(omax, m.d_out());
    hmax = std::max(hmax, m.c.n_heads);
  }
  const int w = g.head.width, D = g.head.d_latent;
  int rc;
  if ((rc = dalloc<float>(c, &c->h, (size_t)MR * dmax))) return rc;
  if ((rc = dalloc<float>(c, &c->x_in, (size_t)MR * 16))) return rc;
  if ((rc = dalloc<float>(c, &c->ent_heads, (size_t)MR * hmax))) return rc;
  if ((rc = dalloc<float>(c, &c->h_row, (size_t)MR))) return rc;
  const size_t MRt = ((size_t)MR + 15) / 16 * 16;          // whole 16-row tiles for the buffers that may hold tile order
  if ((rc = dalloc_bytes(c, &c->u, MRt * dmax * c->esz))) return rc;
  if ((rc = dalloc_bytes(c, &c->qkv, (size_t)MR * qmax * c->esz))) return rc;
  if ((rc = dalloc_bytes(c, &c->ao, MRt * hdmax * c->esz))) return rc;
  if ((rc = dalloc_bytes(c, &c->ff, MRt * fmax * c->esz))) return rc;
  if ((rc = dalloc_bytes(c, &c->z, (size_t)MR * omax * c->esz))) return rc;
  if ((rc = dalloc_bytes(c, &c->ztmp, (size_t)MR * dmax * c->esz))) return rc;
  if ((rc = dalloc<int>(c, &c->maps.row_start, g.max_batch + 2))) return rc;
  if ((rc = dalloc<int>(c, &c->maps.row_sample, MR))) return rc;
  if ((rc = dalloc<int>(c, &c->maps.row_j, MR))) return rc;
  if ((rc = dalloc<int>(c, &c->maps.row_pos, MR))) return rc;
  if ((rc = dalloc<int>(c, &c->maps.m_total, 4))) return rc;
  if ((rc = dalloc<int>(c, &c->aux_row, MR))) return rc;
  if ((rc = dalloc<int>(c, &c->row_ids, MR))) return rc;
  if ((rc = dalloc<float>(c, &c->x_scratch, (size_t)M * 16))) return rc;
  if ((rc = dalloc<uint8_t>(c, &c->acc_tmp, (size_t)g.max_batch * g.K))) return rc;
  if ((rc = dalloc<float>(c, &c->cz, (size_t)M * w))) return rc;
  if ((rc = dalloc<float>(c, &c->hh, (size_t)M * w))) return rc;
  if ((rc = dalloc<float>(c, &c->mod, (size_t)g.head.n_steps * M * c->head.mod_n))) return rc;
  if ((rc = dalloc<float>(c, &c->xt, (size_t)M * D))) return rc;
  if ((rc = dalloc_bytes(c, &c->sc, (size_t)g.head.n_steps * M * w * c->esz))) return rc;
  if ((rc = dalloc_bytes(c, &c->a1, (size_t)((M + 15) / 16 * 16) * w * c->esz))) return rc;
  if ((rc = dalloc_bytes(c, &c->a2, (size_t)((M + 15) / 16 * 16) * w * c->esz))) return rc;   // (whole 16-row tiles)
  if ((rc = dalloc_bytes(c, &c->hv, (size_t)((M + 15) / 16 * 16) * w * c->esz))) return rc;
  if ((rc = dalloc<float>(c, &c->hmom, (size_t)(w / 16 + 1) * M * 2))) return rc;
  if ((rc = dalloc<int>(c, &c->alive, g.max_batch))) return rc;
  if ((rc = dalloc<int>(c, &c->act_idx, g.max_batch))) return rc;
  if ((rc = dalloc<int>(c, &c->n_act, 4))) return rc;
  if ((rc = dalloc<int>(c, &c->emap, g.max_batch))) return rc;
  if ((rc = dalloc<int>(c, &c->omap, g.max_batch))) return rc;
  if ((rc = dalloc<int>(c, &c->ent_blk, ENT_MAX_BLOCKS))) return rc;
  // entries of the attention-pass arrays: n_pass * B <= rows / (rows of a pass) + B for any batch that fits
  c->ap_max = c->m_rows / std::max(1, std::min(std::min(cap_nq(c, 0), cap_nq(c, 1)), c->m_rows)) + 2 * g.max_batch;
  if ((rc = dalloc<int>(c, &c->ap_start, (size_t)c->ap_max))) return rc;
  if ((rc = dalloc<int>(c, &c->ap_cnt, (size_t)c->ap_max))) return rc;
  if ((rc = dalloc<int>(c, &c->ap_len, (size_t)c->ap_max))) return rc;
  if ((rc = dalloc<int>(c, &c->pf_n, g.max_batch))) return rc;
  if ((rc = dalloc<int>(c, &c->pf_nq, g.max_batch))) return rc;
  const size_t bk = (size_t)g.max_batch * g.K;
  if ((rc = dalloc<float>(c, &c->g_x, bk * D))) return rc;
  if ((rc = dalloc<float>(c, &c->g_mu_q, bk * D))) return rc;
  if ((rc = dalloc<float>(c, &c->g_mu_p, (size_t)g.max_batch * (g.K + 1) * D))) return rc;
  if ((rc = dalloc<float>(c, &c->g_lr, bk))) return rc;
  if ((rc = dalloc<float>(c, &c->g_next, (size_t)g.max_batch * D))) return rc;
  if ((rc = dalloc<float>(c, &c->g_cu_x, (size_t)g.max_batch * D))) return rc;
  if ((rc = dalloc<int>(c, &c->g_cu_nq, g.max_batch))) return rc;
  if ((rc = dalloc<uint8_t>(c, &c->g_keep, bk))) return rc;
  if ((rc = dalloc<float>(c, &c->s_eps, (size_t)(g.head.n_steps + 1) * g.max_batch * (g.K + 1) * D))) return rc;
  if ((rc = dalloc<float>(c, &c->s_r, bk))) return rc;
  if ((rc = dalloc<float>(c, &c->s_eres, (size_t)g.max_batch * GEN_J_MAX * D))) return rc;
  if ((rc = dalloc<float>(c, &c->s_ures, (size_t)g.max_batch * GEN_J_MAX))) return rc;
  if ((rc = dalloc<float>(c, &c->s_H, bk))) return rc;
  if ((rc = dalloc<int>(c, &c->s_pid, g.max_batch))) return rc;
  if ((rc = dalloc<int>(c, &c->s_nk, g.max_batch))) return rc;
  if ((rc = dalloc<int>(c, &c->s_na, g.max_batch))) return rc;
  if ((rc = dalloc<int>(c, &c->s_tr, g.max_batch))) return rc;
  // split-key attention: only contexts whose full batch leaves most of the chip idle (samples x kv heads < 256)
  if (c->bf16) {
    int hk_min = std::min(c->mdl[0].c.n_kv_heads, c->mdl[1].c.n_kv_heads), dh_max = std::max(c->mdl[0].c.d_head, c->mdl[1].c.d_head);
    if ((long)g.max_batch * hk_min < 256) {
      c->attn_rows = M;
      if ((rc = dalloc<float>(c, &c->attn_o, (size_t)ATTN_MAX_SPLIT * M * hmax * dh_max))) return rc;
      if ((rc = dalloc<float>(c, &c->attn_mla, (size_t)ATTN_MAX_SPLIT * M * hmax * 4))) return rc;
    }
  }
  // planes for any forward the workspace admits (a prefill pass has more rows than a round), up to the row limit
  if (c->bf16) {
    c->parts_cap = (size_t)PART_MAX_SLICES * std::min(std::max(M, MR), PART_MAX_ROWS) * dmax;
    if ((rc = dalloc<float>(c, &c->parts, c->parts_cap))) return rc;
  }
  return FARD_OK;
}

KvGeom kv_geom(fard_ctx* c, Model& m, int layer) {
  KvGeom g;
  g.k = (char*)m.kc + (size_t)layer * m.layer_elems * c->esz;
  g.v = (char*)m.vc + (size_t)layer * m.layer_elems * c->esz;
  g.n_kv_heads = m.c.n_kv_heads;
  g.d_head = m.c.d_head;
  g.ctx_pad = m.ctx_pad;
  g.is_bf16 = c->bf16;
  return g;
}

// GEMMs of 65 to 128 rows against tens of MB of weights (the verify stage of the 5120-wide configuration: 72 rows,
// 52-283 MB per matrix): K is split over workgroups of the streaming kernel on 128-column tiles and every split writes
// its own plane; the kernel that follows (RoPE + cache append, the next norm) sums the planes.  Returns the number of
// planes, 0 when the shape does not call for it.  Measured at 72 rows: QKV 7168 x 5120 35 -> 25 us, output projection
// 26.5 -> 20.6 us, down-projection 49.5 -> 39 us.
int plane_splits(const fard_ctx* c, int M, int N, int K) {
  if (!c->bf16 || c->parts == nullptr || M <= 64 || M > 128 || K % 256 != 0 || N % 32 != 0) return 0;
  if ((size_t)K * N * 2 < ((size_t)16 << 20)) return 0;
  const int tiles = (N + 127) / 128;
  if (tiles >= 200) return 0;                              // the column tiles alone cover the chip
  int want = (200 + tiles - 1) / tiles;
  want = std::min(want, std::min(PART_MAX_SLICES, K / 256));
  const int n = gemm_plane_count(K, want);
  if (n < 2 || (size_t)n * M * N > c->parts_cap) return 0;
  return n;
}

// The down-projection with a long K and a few hundred rows at most: K slices of 1024 as separate workgroups of
// the narrow kernel, each writing its partial sums to its own plane; no atomics.  The planes stay pending until
// the next norm (or flush_parts) adds them to the residual stream.
bool parts_eligible(const fard_ctx* c, int M, int N, int K) {
  if (plane_splits(c, M, N, K) > 0) return true;
  return c->bf16 && c->parts != nullptr && M <= PART_MAX_ROWS && K > 2048 && (K + 1023) / 1024 <= 8 && N <= 8192 &&
         N % 32 == 0 && K % 64 == 0 && (size_t)((K + 1023) / 1024) * M * N <= c->parts_cap;
}

// out planes <- A W (+ bias in plane 0); *n_planes and *stride describe them.  The planes are c->parts.
hipError_t gemm_planes(fard_ctx* c, const void* A, int lda, const void* W, const float* bias, int M, int N, int K,
                       const int* m_dev, int* n_planes, size_t* stride, int a_tiled = 0) {
  GemmArgs a;
  a.A = A; a.lda = lda; a.W = W; a.bias = bias; a.out = c->parts; a.ldo = N; a.gate = nullptr; a.ldg = 0;
  a.M = M; a.N = N; a.K = K; a.m_dev = m_dev; a.act = ACT_NONE; a.epi = EPI_PARTIAL;
  const int wide = plane_splits(c, M, N, K);
  if (a_tiled && wide > 0) return hipErrorInvalidValue;      // (only the narrow kernel reads tile order)
  a.a_tiled = a_tiled;
  a.k_slices = wide > 0 ? wide : (K + 1023) / 1024;
  a.part_stride = (size_t)M * N;
  if ((size_t)a.k_slices * a.part_stride > c->parts_cap) return hipErrorInvalidValue;   // never launch past the planes
  const double fl = 2.0 * M * (double)N * K;
  const double by = (double)K * N * c->esz + (double)M * K * c->esz + (double)M * N * 4;
  Bracket br(c, wide > 0 ? CLS_GEMM : CLS_GEMM_NARROW, fl, by);
  hipError_t e = wide > 0 ? launch_gemm_bf16_planes(c->stream, a) : launch_gemm_narrow(c->stream, a);
  if (e == hipSuccess) {
    *n_planes = a.k_slices;
    *stride = a.part_stride;
  }
  return e;
}

// A residual update left as pending planes: the next norm adds them to the stream.
hipError_t gemm_parts(fard_ctx* c, const void* A, int lda, const void* W, const float* bias, int M, int N, int K,
                      const int* m_dev, int a_tiled = 0) {
  int n = 0;
  size_t stride = 0;
  hipError_t e = gemm_planes(c, A, lda, W, bias, M, N, K, m_dev, &n, &stride, a_tiled);
  if (e == hipSuccess) {
    c->pend_n = n;
    c->pend_stride = stride;
  }
  return e;
}

int flush_parts(fard_ctx* c, int d, int M, const int* m_dev) {
  if (c->pend_n == 0) return FARD_OK;
  Bracket br(c, CLS_OTHER);
  HIPCHK(c, launch_add_parts(c->stream, c->h, c->parts, c->pend_n, c->pend_stride, d, M, m_dev));
  c->pend_n = 0;
  return FARD_OK;
}

// The bf16 activations that a narrow-tile GEMM reads (first-norm rows for QKV, attention output for the output
// projection, second-norm rows and the MLP's hidden rows) are written in tile order (common.h: tile_offset) by their
// producers; whether a buffer is tiled is a function of the consumer's route, i.e. of the shapes alone.
bool qkv_reads_tiles(fard_ctx* c, const Model& m, int M) {
  const fard_tf_cfg& t = m.c;
  if (!c->bf16) return false;
  const bool fused_append = t.pos != FARD_POS_ROPE;
  if (!fused_append && plane_splits(c, M, m.qkv_n(), t.d_model) > 0) return false;
  return routes_narrow(M, m.qkv_n(), t.d_model, EPI_STORE);
}

// Layers [l0, l1) of one model over the packed rows described by c->maps (h in, h out).
// first_norm_done: c->u already holds the first norm of layer l0 (the embedding kernel wrote it).
int run_layers(fard_ctx* c, int which, int l0, int l1, int B, int M, int nq_max, const int* m_dev, int ent_layer,
               bool first_norm_done = false) {
  Model& m = c->mdl[which];
  const fard_tf_cfg& t = m.c;
  hipStream_t s = c->stream;
  const int d = t.d_model, F = t.d_ff, HD = t.n_heads * t.d_head, QN = m.qkv_n();
  // tile order of the bf16 buffers between the kernels (see qkv_reads_tiles): by the routes of the GEMMs that read them
  const bool gelu = t.act == FARD_ACT_GELU;
  const bool u1_tiled = qkv_reads_tiles(c, m, M);
  const bool up_narrow = c->bf16 && gelu && routes_narrow(M, F, d, EPI_STORE);
  const bool down_narrow = c->bf16 && (parts_eligible(c, M, d, F) ? plane_splits(c, M, d, F) == 0 : routes_narrow(M, d, F, EPI_RESID));
  const bool ff_tiled = up_narrow && down_narrow;
  for (int l = l0; l < l1; ++l) {
    const LayerW& L = m.L[l];
    if (!(first_norm_done && l == l0 && c->pend_n == 0)) {
      Bracket br(c, CLS_OTHER);
      HIPCHK(c, launch_norm(s, c->bf16, c->h, d, M, m_dev, t.norm, t.norm_eps, L.n1g, L.n1b, nullptr, nullptr, 0, nullptr, c->u,
                            c->parts, c->pend_n, c->pend_stride, c->h, u1_tiled));
      c->pend_n = 0;
    }
    KvGeom kg = kv_geom(c, m, l);
    // learned positions, bf16: the attention kernel stores the new K / V rows itself
    const bool fused_append = c->bf16 && t.pos != FARD_POS_ROPE;
    if (!fused_append && c->bf16 && plane_splits(c, M, QN, d) > 0) {
      // the QKV product as K-slice planes, summed by the kernel that rotates q, k and appends k, v to the cache
      int n_pl = 0;
      size_t pl_stride = 0;
      HIPCHK(c, gemm_planes(c, c->u, d, L.wqkv, L.bqkv, M, QN, d, m_dev, &n_pl, &pl_stride));
      Bracket br(c, CLS_OTHER);
      HIPCHK(c, launch_rope_append_planes(s, c->parts, n_pl, pl_stride, c->qkv, QN, t.n_heads, kg, t.pos == FARD_POS_ROPE,
                                          t.rope_theta, c->maps.row_sample, c->maps.row_pos, M, m_dev));
    } else {
      if (u1_tiled) {
        GemmExtra ex;
        ex.a_tiled = 1;
        HIPCHK(c, gemm(c, c->u, d, L.wqkv, L.bqkv, c->qkv, QN, M, QN, d, m_dev, EPI_STORE, ACT_NONE, nullptr, 0, &ex));
      } else {
        HIPCHK(c, gemm(c, c->u, d, L.wqkv, L.bqkv, c->qkv, QN, M, QN, d, m_dev, EPI_STORE, ACT_NONE));
      }
      if (!fused_append) {
        Bracket br(c, CLS_OTHER);
        HIPCHK(c, launch_rope_append(s, c->qkv, QN, t.n_heads, kg, t.pos == FARD_POS_ROPE, t.rope_theta, c->maps.row_sample,
                                     c->maps.row_pos, M, m_dev));
      }
    }
    const bool fold2 = c->bf16 && L.w1f != nullptr && gelu && routes_narrow(M, d, HD, EPI_RESID) &&
                       routes_narrow(M, F, d, EPI_STORE);
    const bool ao_tiled = fold2 || (c->bf16 && plane_splits(c, M, d, HD) == 0 && routes_narrow(M, d, HD, EPI_RESID));
    const int acap = cap_nq(c, which);
    if (nq_max <= acap) {
      // few samples x kv heads against a long cache: the key blocks of each are dealt to several workgroups (the
      // count depends on the batch and the cache capacity only, so that every call of a shape takes the same path)
      AttnSplit sp{};
      const int pairs = B * t.n_kv_heads;
      if (c->attn_o != nullptr && !fused_append && pairs < 256 && M <= c->attn_rows) {
        const int n = std::min(std::min(ATTN_MAX_SPLIT, 256 / pairs), (c->cfg.max_ctx + 31) / 32 / 2);
        if (n >= 2) { sp.n = n; sp.rows = c->attn_rows; sp.o = c->attn_o; sp.mla = c->attn_mla; }
      }
      Bracket br(c, CLS_ATTN);
      HIPCHK(c, launch_attention(s, c->qkv, QN, t.n_heads, kg, m.len, c->maps.row_start, B, nq_max, c->ao, HD,
                                 (l + 1 == ent_layer) ? c->ent_heads : nullptr, fused_append ? 1 : 0, nullptr, 1,
                                 sp.n > 1 ? &sp : nullptr, M, m_dev, ao_tiled));
    } else {
      // more rows per sample than one attention workgroup holds: passes of acap rows (c->ap_* hold their row ranges
      // and first positions), all in one launch once every row's K / V is in the cache
      const int n_pass = (nq_max + acap - 1) / acap;
      if (fused_append) {
        Bracket br(c, CLS_OTHER);
        HIPCHK(c, launch_rope_append(s, c->qkv, QN, t.n_heads, kg, 0, t.rope_theta, c->maps.row_sample, c->maps.row_pos, M, m_dev));
      }
      Bracket br(c, CLS_ATTN);
      HIPCHK(c, launch_attention(s, c->qkv, QN, t.n_heads, kg, c->ap_len, c->ap_start, B, acap, c->ao, HD,
                                 (l + 1 == ent_layer) ? c->ent_heads : nullptr, 0, c->ap_cnt, n_pass, nullptr, 0, nullptr, ao_tiled));
    }
    // norm 2 without a launch of its own, when both GEMMs around it run in the narrow kernel: the output
    // projection also leaves the updated stream as bf16, and the up-projection (weights pre-scaled by the norm's
    // gain) sums the row statistics from its activation fragments and applies them in its epilogue
    if (fold2) {
      GemmExtra ex_o, ex_1;
      ex_o.copy_bf16 = c->u;
      ex_o.a_tiled = 1; ex_o.out_tiled = 1;                // (ao and the bf16 copy of the stream in tile order)
      ex_1.a_tiled = 1; ex_1.out_tiled = ff_tiled;
      HIPCHK(c, gemm(c, c->ao, HD, L.wo, L.bo, c->h, d, M, d, HD, m_dev, EPI_RESID, ACT_NONE, nullptr, 0, &ex_o));
      ex_1.ln_cs = L.cs1; ex_1.ln_eps = t.norm_eps; ex_1.ln_rms = t.norm == FARD_NORM_RMS;
      HIPCHK(c, gemm(c, c->u, d, L.w1f, L.b1f, c->ff, F, M, F, d, m_dev, EPI_STORE, ACT_GELU, nullptr, 0, &ex_1));
    } else {
      // (the output projection of the wide 72-row layers also leaves planes, which the second norm adds to the stream)
      if (plane_splits(c, M, d, HD) > 0) {
        HIPCHK(c, gemm_parts(c, c->ao, HD, L.wo, L.bo, M, d, HD, m_dev));
      } else if (ao_tiled) {
        GemmExtra ex;
        ex.a_tiled = 1;
        HIPCHK(c, gemm(c, c->ao, HD, L.wo, L.bo, c->h, d, M, d, HD, m_dev, EPI_RESID, ACT_NONE, nullptr, 0, &ex));
      } else {
        HIPCHK(c, gemm(c, c->ao, HD, L.wo, L.bo, c->h, d, M, d, HD, m_dev, EPI_RESID, ACT_NONE));
      }
      { Bracket br(c, CLS_OTHER);
        HIPCHK(c, launch_norm(s, c->bf16, c->h, d, M, m_dev, t.norm, t.norm_eps, L.n2g, L.n2b, nullptr, nullptr, 0, nullptr, c->u,
                              c->parts, c->pend_n, c->pend_stride, c->h, up_narrow));
        c->pend_n = 0; }
      if (up_narrow) {
        GemmExtra ex;
        ex.a_tiled = 1; ex.out_tiled = ff_tiled;
        HIPCHK(c, gemm(c, c->u, d, L.w1, L.b1, c->ff, F, M, F, d, m_dev, EPI_STORE, ACT_GELU, nullptr, 0, &ex));
      } else if (gelu) {
        HIPCHK(c, gemm(c, c->u, d, L.w1, L.b1, c->ff, F, M, F, d, m_dev, EPI_STORE, ACT_GELU));
      } else {
        HIPCHK(c, gemm(c, c->u, d, L.w1, nullptr, c->ff, F, M, 2 * F, d, m_dev, EPI_SWIGLU, ACT_NONE));
      }
    }
    if (parts_eligible(c, M, d, F)) {
      HIPCHK(c, gemm_parts(c, c->ff, F, L.w2, L.b2, M, d, F, m_dev, ff_tiled));
    } else if (ff_tiled) {
      GemmExtra ex;
      ex.a_tiled = 1;
      HIPCHK(c, gemm(c, c->ff, F, L.w2, L.b2, c->h, d, M, d, F, m_dev, EPI_RESID, ACT_NONE, nullptr, 0, &ex));
    } else {
      HIPCHK(c, gemm(c, c->ff, F, L.w2, L.b2, c->h, d, M, d, F, m_dev, EPI_RESID, ACT_NONE));
    }
  }
  return FARD_OK;
}

// Embedding of the packed rows into c->h together with the first norm of layer 0 into c->u.
hipError_t embed_first_norm(fard_ctx* c, int which, const float* x, int ldx, const int* cond_id, int M, const int* m_dev) {
  Model& m = c->mdl[which];
  const fard_tf_cfg& t = m.c;
  const LayerW& L = m.L[0];
  Bracket br(c, CLS_OTHER);
  return launch_embed_norm(c->stream, c->bf16, x, ldx, t.d_latent, m.in_w, m.in_b, m.pos, c->maps.row_pos, m.cond, cond_id, c->h,
                           t.d_model, M, m_dev, t.norm, t.norm_eps, L.n1g, L.n1b, c->u, qkv_reads_tiles(c, m, M));
}

// Final norm (optionally gathering rows through in_map) and up-projection -> z [n, d_out] storage type.
int run_final(fard_ctx* c, int which, int n, const int* n_dev, const int* in_map, void* z_out) {
  Model& m = c->mdl[which];
  const fard_tf_cfg& t = m.c;
  const bool up = m.up != nullptr;
  { Bracket br(c, CLS_OTHER);
    HIPCHK(c, launch_norm(c->stream, c->bf16, c->h, t.d_model, n, n_dev, t.norm, t.norm_eps, m.nfg, m.nfb, nullptr, nullptr,
                          0, in_map, up ? c->ztmp : z_out, c->parts, c->pend_n, c->pend_stride, nullptr));
    c->pend_n = 0; }
  if (up) HIPCHK(c, gemm(c, c->ztmp, t.d_model, m.up, nullptr, z_out, t.d_out, n, t.d_out, t.d_model, n_dev, EPI_STORE, ACT_NONE));
  return FARD_OK;
}

int cap_nq(const fard_ctx* c, int which) {
  const fard_tf_cfg& t = c->mdl[which].c;
  return c->bf16 ? 64 / (t.n_heads / t.n_kv_heads) : 1 << 20;
}
// Rows of the transformer workspace: a round's rows, or up to PREFILL_ROWS rows of a prefill pass (whole prefixes when
// they fit, so that the GEMMs of a prefill see thousands of rows whatever the attention kernel's own row limit is).
constexpr int PREFILL_ROWS = 8192;
int workspace_rows(const fard_round_cfg& g) {
  const long all = (long)g.max_batch * g.max_ctx;
  return (int)std::max<long>((long)g.max_batch * (g.K + 1), std::min<long>(all, PREFILL_ROWS));
}

// S sampler steps of the head over n rows of z (compact), noise / output rows through emap / omap.
int run_head(fard_ctx* c, const void* z, int n, const int* n_dev, const float* eps, size_t eps_step_stride,
             const int* emap, const int* omap, float* mu, float* x) {
  const fard_head_cfg& hc = c->cfg.head;
  HeadW& hw = c->head;
  hipStream_t s = c->stream;
  const int w = hc.width, D = hc.d_latent, Nb = hc.n_blocks, S = hc.n_steps;
  HIPCHK(c, gemm(c, z, hc.d_cond, hw.c_w, hw.c_b, c->cz, w, n, w, hc.d_cond, n_dev, EPI_STORE_F32, ACT_NONE));
  { Bracket br(c, CLS_OTHER);
    HIPCHK(c, launch_head_prep(s, c->bf16, eps, emap, hc.temperature, D, hw.in_w, hw.in_b, c->cz, hw.temb, S, c->hh, c->sc,
                               c->xt, w, n, n_dev)); }
  // From the second block of a step on the modulated norm has no launch of its own when the rows are few (the launch
  // is then the cost; measured: a gain up to 64 rows, none above): the gate-residual GEMM of block j - 1 leaves
  // v = bf16(h (1 + scale_j)) and the tile moments of h, and block j's first GEMM multiplies v and applies mean, rstd,
  // c1_j = (1 + scale_j) W1_j and c0_j = shift_j W1_j (columns fold_base.. of the mod GEMM, computed only then).
  const bool fold = hw.fold_base > 0 && n <= 64 && routes_narrow(n, w, w, EPI_GATE_RESID) && routes_narrow(n, w, w, EPI_STORE) &&
                    w / 32 <= 48;
  // the bf16 rows a narrow-tile GEMM of a block reads are in tile order: a1 (norm -> first GEMM), a2 and, with the fold, v
  const bool g1_narrow = c->bf16 && routes_narrow(n, w, w, EPI_STORE), g2_narrow = c->bf16 && routes_narrow(n, w, w, EPI_GATE_RESID);
  const bool a2_tiled = g1_narrow && g2_narrow;
  // the modulations of all S steps in one GEMM over S n rows (rows past the device-side count are unused)
  const int mod_cols = fold ? hw.mod_n : (hw.fold_base > 0 ? hw.fold_base : hw.mod_n);
  HIPCHK(c, gemm(c, c->sc, w, hw.mod_all, hw.mod_b_all, c->mod, hw.mod_n, S * n, mod_cols, w, nullptr, EPI_STORE_F32, ACT_NONE));
  for (int k = 0; k < S; ++k) {
    const float t = 1.0f - (float)k / (float)S;
    const float t_next = 1.0f - (float)(k + 1) / (float)S;
    const float* modk = c->mod + (size_t)k * n * hw.mod_n;
    for (int j = 0; j < Nb; ++j) {
      const float* mj = modk + (size_t)3 * w * j;
      const bool folded = fold && j > 0;
      if (!folded) {
        { Bracket br(c, CLS_OTHER);
          HIPCHK(c, launch_norm(s, c->bf16, c->hh, w, n, n_dev, 0, 1e-6f, nullptr, nullptr, mj, mj + w, hw.mod_n, nullptr, c->a1,
                                nullptr, 0, 0, nullptr, g1_narrow)); }
        if (g1_narrow) {
          GemmExtra ex;
          ex.a_tiled = 1; ex.out_tiled = a2_tiled;
          HIPCHK(c, gemm(c, c->a1, w, hw.B[j].w1, hw.B[j].b1, c->a2, w, n, w, w, n_dev, EPI_STORE, ACT_SILU, nullptr, 0, &ex));
        } else {
          HIPCHK(c, gemm(c, c->a1, w, hw.B[j].w1, hw.B[j].b1, c->a2, w, n, w, w, n_dev, EPI_STORE, ACT_SILU));
        }
      } else {
        GemmExtra ex;
        ex.a_tiled = 1; ex.out_tiled = 1;
        ex.ada_mom = c->hmom; ex.ada_mom_ld = w / 16;
        ex.ada_c0 = modk + (size_t)hw.fold_base + (size_t)2 * w * j; ex.ada_c1 = ex.ada_c0 + w; ex.ada_ld = hw.mod_n;
        ex.ada_eps = 1e-6f;
        HIPCHK(c, gemm(c, c->hv, w, hw.B[j].w1, hw.B[j].b1, c->a2, w, n, w, w, n_dev, EPI_STORE, ACT_SILU, nullptr, 0, &ex));
      }
      if (fold && j + 1 < Nb) {
        GemmExtra ex;
        ex.a_tiled = 1; ex.out_tiled = 1;
        ex.copy_bf16 = c->hv; ex.copy_scale = modk + (size_t)3 * w * (j + 1) + w; ex.copy_ld = hw.mod_n;
        ex.mom_out = c->hmom; ex.mom_ld = w / 16;
        HIPCHK(c, gemm(c, c->a2, w, hw.B[j].w2, hw.B[j].b2, c->hh, w, n, w, w, n_dev, EPI_GATE_RESID, ACT_NONE, mj + 2 * w, hw.mod_n, &ex));
      } else if (a2_tiled) {
        GemmExtra ex;
        ex.a_tiled = 1;
        HIPCHK(c, gemm(c, c->a2, w, hw.B[j].w2, hw.B[j].b2, c->hh, w, n, w, w, n_dev, EPI_GATE_RESID, ACT_NONE, mj + 2 * w, hw.mod_n, &ex));
      } else {
        HIPCHK(c, gemm(c, c->a2, w, hw.B[j].w2, hw.B[j].b2, c->hh, w, n, w, w, n_dev, EPI_GATE_RESID, ACT_NONE, mj + 2 * w, hw.mod_n));
      }
    }
    HeadStepArgs a;
    a.hh = c->hh; a.w = w;
    a.shift = modk + (size_t)3 * w * Nb; a.scale = a.shift + w; a.ldm = hw.mod_n;
    a.w_out = hw.out_w; a.b_out = hw.out_b; a.D = D;
    a.xt = c->xt;
    a.eps_next = eps + (size_t)(k + 1) * eps_step_stride;
    a.emap = emap; a.omap = omap;
    a.t = t; a.t_next = t_next;
    a.last = (k == S - 1);
    a.renoise = hc.renoise;
    a.sigma = hc.sigma_last * hc.temperature;
    a.mu = mu; a.x = x;
    a.w_in = hw.in_w; a.b_in = hw.in_b; a.hh_next = c->hh;
    a.n = n; a.n_dev = n_dev;
    { Bracket br(c, CLS_OTHER);
      HIPCHK(c, launch_head_out(s, c->bf16, a)); }
  }
  return FARD_OK;
}

int check_ctx(fard_ctx* c) { return c ? FARD_OK : FARD_EINVAL; }

}  // namespace

// ====================================================================================== C ABI
extern "C" {

int spec_round_init(const fard_round_cfg* cfg, const fard_tensor* weights, int32_t n_weights, void* hip_stream,
                    fard_ctx** out) {
  if (!cfg || !out || (!weights && n_weights > 0) || n_weights < 0) return FARD_EINVAL;
  *out = nullptr;
  fard_ctx* c = new (std::nothrow) fard_ctx();
  if (!c) return FARD_ENOMEM;
  c->cfg = *cfg;
  c->stream = (hipStream_t)hip_stream;
  int rc = FARD_OK;
  auto bail = [&](int code) {
    // keep the message reachable: the caller gets no context on failure, so print it
    fprintf(stderr, "spec_round_init: %s\n", c->err.c_str());
    for (void* p : c->allocs) (void)hipFree(p);
    delete c;
    return code;
  };
  if (cfg->dtype != FARD_F32 && cfg->dtype != FARD_BF16) return bail(fail(c, FARD_EINVAL, "dtype"));
  c->bf16 = cfg->dtype == FARD_BF16;
  c->esz = c->bf16 ? 2 : 4;
  if (cfg->K < 1 || cfg->K > 64 || cfg->max_batch < 1 || cfg->max_ctx < cfg->K + 1)
    return bail(fail(c, FARD_EINVAL, "K in [1,64], max_batch >= 1, max_ctx >= K+1 required"));
  if (cfg->prefix_rule != 1) return bail(fail(c, FARD_EINVAL, "prefix_rule must be 1"));
  if (cfg->entropy_mode != FARD_ENT_FEATURE && cfg->entropy_mode != FARD_ENT_ATTN) return bail(fail(c, FARD_EINVAL, "entropy_mode"));
  if (cfg->entropy_layer < 1 || cfg->entropy_layer > cfg->draft.n_layers) return bail(fail(c, FARD_EINVAL, "entropy_layer outside the draft"));
  c->mdl[0].c = cfg->target;
  c->mdl[1].c = cfg->draft;
  if ((rc = check_tf(c, cfg->target, "target")) || (rc = check_tf(c, cfg->draft, "draft"))) return bail(rc);
  const fard_head_cfg& hc = cfg->head;
  if (hc.n_blocks < 1 || hc.width < 1 || hc.n_steps < 1 || hc.t_freq_dim < 2 || hc.t_freq_dim % 2)
    return bail(fail(c, FARD_EINVAL, "head sizes"));
  if (hc.d_latent != cfg->target.d_latent || hc.d_latent != cfg->draft.d_latent) return bail(fail(c, FARD_ESHAPE, "d_latent differs"));
  if (hc.d_cond != c->mdl[0].d_out() || hc.d_cond != c->mdl[1].d_out())
    return bail(fail(c, FARD_ESHAPE, "head.d_cond must equal both models' feature width"));
  if (c->bf16 && (hc.width % 64 != 0 || hc.d_cond % 64 != 0)) return bail(fail(c, FARD_ESHAPE, "bf16 head widths must be multiples of 64"));
  if (!(hc.sigma_last > 0.f)) return bail(fail(c, FARD_EINVAL, "sigma_last must be > 0"));
  c->m_max = cfg->max_batch * (cfg->K + 1);
  c->m_rows = workspace_rows(*cfg);

  Loader ld;
  ld.c = c;
  for (int i = 0; i < n_weights; ++i) {
    if (!weights[i].name) return bail(fail(c, FARD_EINVAL, "unnamed weight"));
    ld.byname[weights[i].name] = &weights[i];
  }
  if ((rc = load_model(c, ld, FARD_TARGET)) || (rc = load_model(c, ld, FARD_DRAFT)) || (rc = load_head(c, ld)) ||
      (rc = alloc_workspace(c))) {
    ld.release_staging();
    return bail(rc);
  }
  ld.release_staging();
  hipError_t e = hipStreamSynchronize(c->stream);
  if (e != hipSuccess) return bail(fail(c, FARD_EHIP, std::string("init sync: ") + hipGetErrorString(e)));
  *out = c;
  return FARD_OK;
}

int spec_round_destroy(fard_ctx* c) {
  if (!c) return FARD_EINVAL;
  (void)hipStreamSynchronize(c->stream);
  for (auto& ev : c->prof.pool) { (void)hipEventDestroy(ev.first); (void)hipEventDestroy(ev.second); }
  c->rgraph.drop();
  c->ggraph.drop();
  if (c->gemm_tmp) (void)hipFree(c->gemm_tmp);
  if (c->loss_tmp) (void)hipFree(c->loss_tmp);
  for (void* p : c->allocs) (void)hipFree(p);
  delete c;
  return FARD_OK;
}

const char* spec_last_error(const fard_ctx* c) { return c ? c->err.c_str() : "null context"; }

float entropy_threshold(float mean_H, float std_H) { return 0.3f * mean_H - 0.1f * std_H; }

int spec_kv_reset(fard_ctx* c, int32_t which, const int32_t* cache_len, int32_t B) {
  if (check_ctx(c)) return FARD_EINVAL;
  if (which != FARD_TARGET && which != FARD_DRAFT) return fail(c, FARD_EINVAL, "which");
  if (B < 0 || B > c->cfg.max_batch) return fail(c, FARD_ECAPACITY, "B > max_batch");
  Model& m = c->mdl[which];
  int hi = 0;
  if (cache_len) {
    for (int b = 0; b < B; ++b) {
      if (cache_len[b] < 0 || cache_len[b] > c->cfg.max_ctx) return fail(c, FARD_ECAPACITY, "cache_len outside [0, max_ctx]");
      hi = std::max(hi, cache_len[b]);
    }
    HIPCHK(c, hipMemcpyAsync(m.len, cache_len, (size_t)B * 4, hipMemcpyHostToDevice, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));   // the host array may go away after return
  } else {
    HIPCHK(c, launch_fill_i32(c->stream, m.len, 0, c->cfg.max_batch));
  }
  m.len_hi = hi;
  m.written = 0;
  return FARD_OK;
}

int spec_kv_restore(fard_ctx* c, int32_t which, const int32_t* cache_len_dev, int32_t B, int32_t len_hi) {
  if (check_ctx(c)) return FARD_EINVAL;
  if (which != FARD_TARGET && which != FARD_DRAFT) return fail(c, FARD_EINVAL, "which");
  if (B < 0 || B > c->cfg.max_batch) return fail(c, FARD_ECAPACITY, "B > max_batch");
  if (len_hi < 0 || len_hi > c->cfg.max_ctx) return fail(c, FARD_ECAPACITY, "len_hi outside [0, max_ctx]");
  if (B > 0 && !cache_len_dev) return fail(c, FARD_EINVAL, "null cache_len_dev");
  Model& m = c->mdl[which];
  if (B > 0) {
    len_restore_kernel<<<(B + 255) / 256, 256, 0, c->stream>>>(cache_len_dev, m.len, B, len_hi);
    HIPCHK(c, hipGetLastError());
  }
  m.len_hi = len_hi;
  m.written = 0;
  return FARD_OK;
}

int spec_kv_load(fard_ctx* c, int32_t which, int32_t layer, const void* k, const void* v, int32_t B, int32_t n) {
  if (check_ctx(c)) return FARD_EINVAL;
  if (which != FARD_TARGET && which != FARD_DRAFT) return fail(c, FARD_EINVAL, "which");
  Model& m = c->mdl[which];
  if (layer < 0 || layer >= m.c.n_layers) return fail(c, FARD_EINVAL, "layer");
  if (B < 0 || B > c->cfg.max_batch || n < 0 || n > c->cfg.max_ctx) return fail(c, FARD_ECAPACITY, "B or n beyond capacity");
  if (B == 0 || n == 0) return FARD_OK;
  if (!k || !v) return fail(c, FARD_EINVAL, "null k/v");
  HIPCHK(c, launch_kv_load(c->stream, kv_geom(c, m, layer), k, v, B, n));
  return FARD_OK;
}

int spec_kv_lengths(fard_ctx* c, int32_t which, int32_t* out_host, int32_t B) {
  if (check_ctx(c)) return FARD_EINVAL;
  if ((which != FARD_TARGET && which != FARD_DRAFT) || !out_host) return fail(c, FARD_EINVAL, "which/out");
  if (B < 0 || B > c->cfg.max_batch) return fail(c, FARD_ECAPACITY, "B > max_batch");
  // all max_batch lengths come back: the host's upper bound (which a round can only raise by K + 1, whatever was
  // accepted) is reset to the true maximum, so that a caller looping over rounds does not run into FARD_ECAPACITY early
  Model& m = c->mdl[which];
  std::vector<int32_t> all((size_t)c->cfg.max_batch);
  HIPCHK(c, hipMemcpyAsync(all.data(), m.len, all.size() * 4, hipMemcpyDeviceToHost, c->stream));
  HIPCHK(c, hipStreamSynchronize(c->stream));
  int hi = 0;
  for (int32_t v : all) hi = std::max(hi, (int)v);
  if (m.written == 0) m.len_hi = hi;       // (between a draft / verify and its commit the bound covers uncommitted rows)
  for (int b = 0; b < B; ++b) out_host[b] = all[b];
  return FARD_OK;
}

int spec_kv_commit(fard_ctx* c, int32_t which, const int32_t* n_accept, int32_t B) {
  if (check_ctx(c)) return FARD_EINVAL;
  if (!n_accept) return fail(c, FARD_EINVAL, "n_accept");
  if (B < 0 || B > c->cfg.max_batch) return fail(c, FARD_ECAPACITY, "B > max_batch");
  if (B == 0) return FARD_OK;
  for (int w = 0; w < 2; ++w) {
    if (which != -1 && which != w) continue;
    Model& m = c->mdl[w];
    if (m.written < 1) return fail(c, FARD_ESTATE, "spec_kv_commit without a preceding spec_draft / spec_verify");
    len_commit_kernel<<<(B + 255) / 256, 256, 0, c->stream>>>(m.len, m.len_base, n_accept, m.written, B);
    HIPCHK(c, hipGetLastError());
    m.written = 0;
  }
  return FARD_OK;
}

int spec_forward(fard_ctx* c, int32_t which, const float* x_in, const int32_t* cond_id, const int32_t* n_q, int32_t nq_max,
                 int32_t B, int32_t M, int32_t commit, void* z_out, float* shallow_out, float* h_attn_out) {
  if (check_ctx(c)) return FARD_EINVAL;
  if (which != FARD_TARGET && which != FARD_DRAFT) return fail(c, FARD_EINVAL, "which");
  if (B < 0 || B > c->cfg.max_batch) return fail(c, FARD_ECAPACITY, "B > max_batch");
  if (M < 0 || M > c->m_rows) return fail(c, FARD_ECAPACITY, "M beyond the workspace rows");
  if (B == 0 || M == 0) return FARD_OK;
  if (!x_in || !n_q || !z_out) return fail(c, FARD_EINVAL, "null x_in / n_q / z_out");
  Model& m = c->mdl[which];
  if (cond_id && !m.cond) return fail(c, FARD_EINVAL, "cond_id given but the model has no id table");
  if (nq_max < 1) return fail(c, FARD_EINVAL, "nq_max < 1");
  const int acap = cap_nq(c, which);
  const int n_pass = (std::min(nq_max, M) + acap - 1) / acap;
  if ((long)n_pass * B > c->ap_max) return fail(c, FARD_ESHAPE, "nq_max beyond the attention passes the workspace holds");
  const int cap = std::min(nq_max, M);
  if (m.len_hi + cap > c->cfg.max_ctx) return fail(c, FARD_ECAPACITY, "cache_len + n_q may exceed max_ctx");
  if (m.c.pos == FARD_POS_LEARNED && m.len_hi + cap > m.c.max_pos) return fail(c, FARD_ECAPACITY, "position beyond the learned table");
  hipStream_t s = c->stream;
  { Bracket br(c, CLS_OTHER);
    HIPCHK(c, launch_build_rows(s, n_q, 0, B, c->cfg.K, m.c.d_latent, m.len, c->maps, nullptr, nullptr, nullptr, nullptr, M, cap)); }
  const int* md = c->maps.m_total;
  if (n_pass > 1) {
    Bracket br(c, CLS_OTHER);
    attn_pass_kernel<<<(B * n_pass + 255) / 256, 256, 0, s>>>(c->maps.row_start, m.len, B, acap, n_pass, c->ap_start, c->ap_cnt,
                                                               c->ap_len);
    HIPCHK(c, hipGetLastError());
  }
  HIPCHK(c, embed_first_norm(c, which, x_in, m.c.d_latent, cond_id, M, md));
  const int ls = c->cfg.entropy_layer;
  const bool want_sh = (shallow_out || h_attn_out) && ls <= m.c.n_layers;
  int rc;
  if (want_sh) {
    if ((rc = run_layers(c, which, 0, ls, B, M, cap, md, h_attn_out ? ls : 0, true))) return rc;
    if ((rc = flush_parts(c, m.c.d_model, M, md))) return rc;
    if (shallow_out) {
      Bracket br(c, CLS_OTHER);
      HIPCHK(c, launch_scatter_rows(s, c->h, shallow_out, nullptr, m.c.d_model, 4, M, md));
    }
    if (h_attn_out) {
      Bracket br(c, CLS_ENT);
      mean_heads_kernel<<<(M + 255) / 256, 256, 0, s>>>(c->ent_heads, m.c.n_heads, h_attn_out, M, md);
      HIPCHK(c, hipGetLastError());
    }
    if ((rc = run_layers(c, which, ls, m.c.n_layers, B, M, cap, md, 0))) return rc;
  } else {
    if ((rc = run_layers(c, which, 0, m.c.n_layers, B, M, cap, md, 0, true))) return rc;
  }
  if ((rc = run_final(c, which, M, md, nullptr, z_out))) return rc;
  if (commit) {
    HIPCHK(c, launch_len_add(s, m.len, n_q, 0, B));
    m.len_hi += cap;
  }
  return FARD_OK;
}

int spec_prefill(fard_ctx* c, int32_t which, const float* x, const int32_t* first_id, const int32_t* n, int32_t n_max,
                 int32_t B, void* z_last) {
  if (check_ctx(c)) return FARD_EINVAL;
  if (which != FARD_TARGET && which != FARD_DRAFT) return fail(c, FARD_EINVAL, "which");
  if (B < 0 || B > c->cfg.max_batch) return fail(c, FARD_ECAPACITY, "B > max_batch");
  if (n_max < 0) return fail(c, FARD_EINVAL, "n_max < 0");
  if (B == 0 || n_max == 0) return FARD_OK;
  if (!x || !n) return fail(c, FARD_EINVAL, "null x / n");
  Model& m = c->mdl[which];
  if (first_id && !m.cond) return fail(c, FARD_EINVAL, "first_id given but the model has no id table");
  int n_hi = 0;
  for (int b = 0; b < B; ++b) {
    if (n[b] < 0 || n[b] > n_max) return fail(c, FARD_EINVAL, "n[b] outside [0, n_max]");
    n_hi = std::max(n_hi, n[b]);
  }
  if (n_hi == 0) return FARD_OK;
  if (m.len_hi + n_hi > c->cfg.max_ctx) return fail(c, FARD_ECAPACITY, "cache_len + n exceeds max_ctx");
  if (m.c.pos == FARD_POS_LEARNED && m.len_hi + n_hi > m.c.max_pos) return fail(c, FARD_ECAPACITY, "position beyond the learned table");
  hipStream_t s = c->stream;
  HIPCHK(c, hipMemcpyAsync(c->pf_n, n, (size_t)B * 4, hipMemcpyHostToDevice, s));
  HIPCHK(c, hipStreamSynchronize(s));      // the host array may go away after return
  // rows per sample of one pass through the layers: whole prefixes when B of them fit into the workspace
  const int chunk = std::max(1, std::min(c->m_rows / B, c->cfg.max_ctx)), D = m.c.d_latent, ldz = m.d_out();
  for (int c0 = 0; c0 < n_hi; c0 += chunk) {
    const int cap = std::min(chunk, n_hi - c0);
    int M = 0;
    for (int b = 0; b < B; ++b) M += std::min(std::max(n[b] - c0, 0), cap);
    { Bracket br(c, CLS_OTHER);
      prefill_chunk_kernel<<<(B + 255) / 256, 256, 0, s>>>(c->pf_n, c0, cap, c->pf_nq, B);
      HIPCHK(c, hipGetLastError());
      prefill_pack_kernel<<<B, 64, 0, s>>>(x, n_max, D, c0, c->pf_nq, first_id, c->x_in, c->row_ids);
      HIPCHK(c, hipGetLastError()); }
    int rc = spec_forward(c, which, c->x_in, m.cond ? c->row_ids : nullptr, c->pf_nq, cap, B, M, 1, c->z, nullptr, nullptr);
    if (rc) return rc;
    if (z_last) {
      Bracket br(c, CLS_OTHER);
      if (c->bf16) prefill_last_kernel<bf16><<<B, 64, 0, s>>>((const bf16*)c->z, ldz, c->pf_n, c0, c->pf_nq, (bf16*)z_last);
      else prefill_last_kernel<float><<<B, 64, 0, s>>>((const float*)c->z, ldz, c->pf_n, c0, c->pf_nq, (float*)z_last);
      HIPCHK(c, hipGetLastError());
    }
  }
  return FARD_OK;
}

static int loss_scratch(fard_ctx* c, size_t bytes) {
  if (bytes <= c->loss_tmp_bytes) return FARD_OK;
  HIPCHK(c, hipStreamSynchronize(c->stream));
  if (c->loss_tmp) (void)hipFree(c->loss_tmp);
  c->loss_tmp = nullptr;
  c->loss_tmp_bytes = 0;
  if (hipMalloc(&c->loss_tmp, bytes) != hipSuccess) return fail(c, FARD_ENOMEM, "loss scratch hipMalloc failed");
  c->loss_tmp_bytes = bytes;
  return FARD_OK;
}

int spec_entropy_loss(fard_ctx* c, const void* q, const void* k, int32_t B, int32_t H, int32_t H_kv, int32_t R, int32_t d_head,
                      float* loss, float* h_rows, float* dq, float* dk) {
  if (check_ctx(c)) return FARD_EINVAL;
  if (!c->bf16) return fail(c, FARD_ESTATE, "spec_entropy_loss needs a bf16 context");
  if (B < 1 || H < 1 || H_kv < 1 || R < 1 || H % H_kv != 0) return fail(c, FARD_ESHAPE, "B, H, H_kv, R >= 1 and H % H_kv == 0 required");
  if (d_head != 32 && d_head != 64 && d_head != 128) return fail(c, FARD_ESHAPE, "d_head must be 32, 64 or 128");
  if (!q || !k || !loss) return fail(c, FARD_EINVAL, "null argument");
  if ((((uintptr_t)q) | ((uintptr_t)k)) & 15) return fail(c, FARD_EINVAL, "q and k must be 16-byte aligned");
  const EntLossScratch lay = entropy_loss_scratch(B, H, H_kv, R, d_head);
  int rc = loss_scratch(c, lay.bytes);
  if (rc) return rc;
  // score tiles: forward once, once more per gradient; second products: one per gradient
  const double tiles = (double)B * H * 0.5 * R * (double)R;
  const double fl = 2.0 * d_head * tiles * (1.0 + (dq ? 2.0 : 0.0) + (dk ? 2.0 : 0.0));
  Bracket br(c, CLS_ATTN, fl, (double)B * (H + H_kv) * R * d_head * 2.0);
  HIPCHK(c, launch_entropy_loss(c->stream, q, k, B, H, H_kv, R, d_head, c->loss_tmp, loss, h_rows, dq, dk));
  return FARD_OK;
}

int spec_smooth_l1(fard_ctx* c, const void* pred, const void* target, int64_t n, float beta, float* loss, float* dpred) {
  if (check_ctx(c)) return FARD_EINVAL;
  if (n < 1) return fail(c, FARD_ESHAPE, "n >= 1 required");
  if (!(beta > 0.f)) return fail(c, FARD_EINVAL, "beta > 0 required");
  if (!pred || !target || !loss) return fail(c, FARD_EINVAL, "null argument");
  const int n_part = (int)std::min<int64_t>(1024, (n + 255) / 256);
  int rc = loss_scratch(c, (size_t)n_part * 4);
  if (rc) return rc;
  Bracket br(c, CLS_OTHER);
  HIPCHK(c, launch_smooth_l1(c->stream, c->bf16, pred, target, (long)n, beta, (float*)c->loss_tmp, n_part, loss, dpred));
  return FARD_OK;
}

int entropy_prefilter(fard_ctx* c, const void* feat, int32_t B, int32_t K, int32_t L, float tau, float* H, uint8_t* keep,
                      int32_t* n_keep, int32_t* surv_idx, int32_t* n_surv) {
  if (check_ctx(c)) return FARD_EINVAL;
  if (B < 0 || K < 0 || L < 1) return fail(c, FARD_ESHAPE, "B, K >= 0 and L >= 1 required");
  if (!n_surv) return fail(c, FARD_EINVAL, "null n_surv");
  if ((long)B * K == 0) {
    HIPCHK(c, launch_fill_i32(c->stream, n_surv, 0, 1));
    if (B > 0 && n_keep) HIPCHK(c, launch_fill_i32(c->stream, n_keep, 0, B));
    return FARD_OK;
  }
  if (!feat || !H || !keep || !n_keep || !surv_idx) return fail(c, FARD_EINVAL, "null argument");
  Bracket br(c, CLS_ENT, 0, (double)B * K * L * c->esz);
  HIPCHK(c, launch_entropy_prefilter(c->stream, c->bf16, feat, B, K, L, tau, H, keep, n_keep, surv_idx, n_surv, c->ent_blk));
  return FARD_OK;
}

// ---- the pre-filter for callers that cannot allocate: no context, scratch in a file-scope device array
constexpr int STATIC_PF_MAX_B = 1 << 21;                 // samples
constexpr long STATIC_PF_MAX_ROWS = 1L << 24;            // B * K
constexpr int STATIC_PF_MAX_DEVICES = 64;
}  // extern "C"
// per-workgroup survivor counts of the large-batch path (entropy_samples_kernel -> entropy_compact_kernel); every
// GPU the library runs on holds its own copy until the process ends
static __device__ __align__(256) int scratch[fard::ENT_MAX_BLOCKS];
static int* g_scratch_ptr[STATIC_PF_MAX_DEVICES];        // the array's device address, per device (nullptr: not asked yet)
static std::mutex g_scratch_mu;
extern "C" {

int entropy_prefilter_static(const void* feat, int32_t dtype, int32_t B, int32_t K, int32_t L, float tau, float* H,
                             uint8_t* keep, int32_t* n_keep, int32_t* surv_idx, int32_t* n_surv, void* hip_stream) {
  if (dtype != FARD_F32 && dtype != FARD_BF16) return FARD_EINVAL;
  if (B < 0 || K < 0 || L < 1) return FARD_ESHAPE;
  if (B > STATIC_PF_MAX_B || (long)B * K > STATIC_PF_MAX_ROWS) return FARD_ECAPACITY;
  if (!n_surv) return FARD_EINVAL;
  hipStream_t s = (hipStream_t)hip_stream;
  if ((long)B * K == 0) {
    if (launch_fill_i32(s, n_surv, 0, 1) != hipSuccess) return FARD_EHIP;
    if (B > 0 && n_keep && launch_fill_i32(s, n_keep, 0, B) != hipSuccess) return FARD_EHIP;
    return FARD_OK;
  }
  if (!feat || !H || !keep || !n_keep || !surv_idx) return FARD_EINVAL;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= STATIC_PF_MAX_DEVICES) return FARD_EHIP;
  int* blk = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (g_scratch_ptr[dev] == nullptr) {
      // the array's name is only a host-side handle: its address on the current device has to be asked for
      int* p = nullptr;
      if (hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return FARD_EHIP;
      g_scratch_ptr[dev] = p;
    }
    blk = g_scratch_ptr[dev];
  }
  // every workgroup of the first launch overwrites its own count before the second launch reads it: nothing to clear
  if (launch_entropy_prefilter(s, dtype == FARD_BF16, feat, B, K, L, tau, H, keep, n_keep, surv_idx, n_surv, blk) != hipSuccess)
    return FARD_EHIP;
  return FARD_OK;
}

int diffhead_decode(fard_ctx* c, const void* z, const int32_t* n_rows, int32_t n_max, const float* eps, float* mu, float* x) {
  if (check_ctx(c)) return FARD_EINVAL;
  if (n_max < 0 || n_max > c->m_max) return fail(c, FARD_ECAPACITY, "n_max > max_batch*(K+1)");
  if (n_max == 0) return FARD_OK;
  if (!z || !eps || !mu || !x) return fail(c, FARD_EINVAL, "null argument");
  return run_head(c, z, n_max, n_rows, eps, (size_t)n_max * c->cfg.head.d_latent, nullptr, nullptr, mu, x);
}

int spec_accept(fard_ctx* c, const float* x_draft, const float* mu_p, const float* mu_q, const float* r, const int32_t* n_keep,
                float log_sigma_factor, float sigma_p, float sigma_q, int32_t B, int32_t* n_accept, float* log_ratio,
                uint8_t* acc) {
  if (check_ctx(c)) return FARD_EINVAL;
  if (B < 0) return fail(c, FARD_ESHAPE, "B < 0");
  if (B == 0) return FARD_OK;
  if (!x_draft || !mu_p || !mu_q || !r || !n_keep || !n_accept || !log_ratio || !acc) return fail(c, FARD_EINVAL, "null argument");
  if (!(sigma_p > 0.f) || !(sigma_q > 0.f)) return fail(c, FARD_EINVAL, "sigma must be > 0");
  Bracket br(c, CLS_OTHER);
  HIPCHK(c, launch_accept(c->stream, x_draft, mu_p, mu_q, r, n_keep, log_sigma_factor, sigma_p, sigma_q, B, c->cfg.K,
                          c->cfg.head.d_latent, n_accept, log_ratio, acc));
  return FARD_OK;
}

// Start of a draft stage: the lengths to roll back to, every sample alive, outputs cleared.
static int draft_begin(fard_ctx* c, int B, int32_t* n_keep, float* x_draft, float* mu_q) {
  Model& m = c->mdl[FARD_DRAFT];
  const int K = c->cfg.K, D = m.c.d_latent;
  hipStream_t s = c->stream;
  Bracket br(c, CLS_OTHER);
  copy_i32_kernel<<<(B + 255) / 256, 256, 0, s>>>(m.len, m.len_base, B);
  HIPCHK(c, hipGetLastError());
  HIPCHK(c, launch_fill_i32(s, c->alive, 1, B));
  HIPCHK(c, launch_fill_i32(s, n_keep, 0, B));
  // dropped drafts keep finite values: they still travel through the dense draft rows
  HIPCHK(c, launch_fill_f32(s, x_draft, 0.f, (size_t)B * K * D));
  HIPCHK(c, launch_fill_f32(s, mu_q, 0.f, (size_t)B * K * D));
  m.written = 0;
  return FARD_OK;
}

// One row per sample: the row maps of a draft step (positions = current lengths).
static int draft_maps(fard_ctx* c, int B) {
  Model& m = c->mdl[FARD_DRAFT];
  Bracket br(c, CLS_OTHER);
  HIPCHK(c, launch_build_rows(c->stream, nullptr, 1, B, c->cfg.K, m.c.d_latent, m.len, c->maps, nullptr, nullptr, nullptr, nullptr, B, 1));
  return FARD_OK;
}

// Draft step i: reads the previous token of every sample (xs, row stride ldx), produces draft i of the samples that
// are still speculating, advances the draft cache by one position.
static int draft_step(fard_ctx* c, int i, const float* xs, int ldx, const int32_t* ids, const float* eps, float tau, int B,
                      float* H, uint8_t* keep, int32_t* n_keep, float* x_draft, float* mu_q) {
  Model& m = c->mdl[FARD_DRAFT];
  const int K = c->cfg.K, D = m.c.d_latent, d = m.c.d_model, ls = c->cfg.entropy_layer;
  hipStream_t s = c->stream;
  const size_t eps_stride = (size_t)B * (K + 1) * D;
  int rc;
  HIPCHK(c, embed_first_norm(c, FARD_DRAFT, xs, ldx, ids, B, nullptr));
  const bool attn_mode = c->cfg.entropy_mode == FARD_ENT_ATTN;
  if ((rc = run_layers(c, FARD_DRAFT, 0, ls, B, B, 1, nullptr, attn_mode ? ls : 0, true))) return rc;
  // pending partial planes of the last shallow layer: the entropy rows add them on the fly and the next norm
  // folds them into the stream; otherwise they are folded here
  const bool ent_folds = !attn_mode && ls < m.c.n_layers && ent_rows_in_regs_f32(c->h, d, d);
  if (!ent_folds && (rc = flush_parts(c, d, B, nullptr))) return rc;
  { Bracket br(c, CLS_ENT, 0, (double)B * d * 4);
    if (!attn_mode)
      HIPCHK(c, launch_entropy_rows_f32(s, c->h, d, B, d, c->h_row, c->parts, ent_folds ? c->pend_n : 0, c->pend_stride));
    HIPCHK(c, launch_entropy_step(s, attn_mode ? c->ent_heads : nullptr, m.c.n_heads, c->h_row, B, K, i, tau, H, keep, c->alive,
                                  n_keep, c->act_idx, c->n_act, c->emap, c->omap)); }
  if ((rc = run_layers(c, FARD_DRAFT, ls, m.c.n_layers, B, B, 1, nullptr, 0))) return rc;
  // only samples that are still speculating reach the head
  if ((rc = run_final(c, FARD_DRAFT, B, c->n_act, c->act_idx, c->z))) return rc;
  if ((rc = run_head(c, c->z, B, c->n_act, eps, eps_stride, c->emap, c->omap, mu_q, x_draft))) return rc;
  HIPCHK(c, launch_len_add(s, m.len, nullptr, 1, B, c->maps.row_pos));
  m.len_hi += 1;
  m.written += 1;
  return FARD_OK;
}

static int draft_checks(fard_ctx* c, const float* x_first, const int32_t* id, const float* eps, int B, const float* H,
                        const uint8_t* keep, const int32_t* n_keep, const float* x_draft, const float* mu_q, int steps) {
  if (B < 0 || B > c->cfg.max_batch) return fail(c, FARD_ECAPACITY, "B > max_batch");
  if (!x_first || !eps || !H || !keep || !n_keep || !x_draft || !mu_q) return fail(c, FARD_EINVAL, "null argument");
  Model& m = c->mdl[FARD_DRAFT];
  if (id && !m.cond) return fail(c, FARD_EINVAL, "pending_id given but the draft has no id table");
  if (m.len_hi + steps > c->cfg.max_ctx) return fail(c, FARD_ECAPACITY, "draft cache_len + K exceeds max_ctx");
  if (m.c.pos == FARD_POS_LEARNED && m.len_hi + steps > m.c.max_pos) return fail(c, FARD_ECAPACITY, "draft position beyond the learned table");
  return FARD_OK;
}

int spec_draft(fard_ctx* c, const float* x_pending, const int32_t* pending_id, const float* eps, float tau, int32_t B,
               float* H, uint8_t* keep, int32_t* n_keep, float* x_draft, float* mu_q) {
  if (check_ctx(c)) return FARD_EINVAL;
  if (B == 0) return FARD_OK;
  int rc = draft_checks(c, x_pending, pending_id, eps, B, H, keep, n_keep, x_draft, mu_q, c->cfg.K);
  if (rc) return rc;
  const int K = c->cfg.K, D = c->mdl[FARD_DRAFT].c.d_latent;
  if ((rc = draft_begin(c, B, n_keep, x_draft, mu_q))) return rc;
  // one row per sample in every step: the row maps are built once, the positions move on with the lengths
  if ((rc = draft_maps(c, B))) return rc;
  for (int i = 0; i < K; ++i) {
    const float* xs = (i == 0) ? x_pending : x_draft + (size_t)(i - 1) * D;
    const int ldx = (i == 0) ? D : K * D;
    if ((rc = draft_step(c, i, xs, ldx, i == 0 ? pending_id : nullptr, eps, tau, B, H, keep, n_keep, x_draft, mu_q))) return rc;
  }
  return FARD_OK;
}

int spec_draft_step(fard_ctx* c, int32_t i, const float* x_prev, const int32_t* prev_id, const float* eps, float tau, int32_t B,
                    float* H, uint8_t* keep, int32_t* n_keep, float* x_draft, float* mu_q) {
  if (check_ctx(c)) return FARD_EINVAL;
  if (i < 0 || i >= c->cfg.K) return fail(c, FARD_EINVAL, "step index outside [0, K)");
  if (B == 0) return FARD_OK;
  const int K = c->cfg.K, D = c->mdl[FARD_DRAFT].c.d_latent;
  if (i > 0 && c->mdl[FARD_DRAFT].written != i) return fail(c, FARD_ESTATE, "draft steps must be taken in order, from step 0");
  const float* xs = x_prev ? x_prev : (i > 0 ? x_draft + (size_t)(i - 1) * D : nullptr);
  const int ldx = x_prev ? D : K * D;
  int rc = draft_checks(c, xs, prev_id, eps, B, H, keep, n_keep, x_draft, mu_q, 1);
  if (rc) return rc;
  if (i == 0 && (rc = draft_begin(c, B, n_keep, x_draft, mu_q))) return rc;
  if ((rc = draft_maps(c, B))) return rc;                // other calls may have used the row maps in between
  return draft_step(c, i, xs, ldx, prev_id, eps, tau, B, H, keep, n_keep, x_draft, mu_q);
}

int spec_verify(fard_ctx* c, const float* x_pending, const int32_t* pending_id, const float* x_draft, const float* mu_q,
                const int32_t* n_keep, const float* r, const float* eps, float log_sigma_factor, float sigma_p, float sigma_q,
                int32_t B, int32_t* n_accept, float* log_ratio, float* mu_p, void* z_p) {
  if (check_ctx(c)) return FARD_EINVAL;
  if (B < 0 || B > c->cfg.max_batch) return fail(c, FARD_ECAPACITY, "B > max_batch");
  if (B == 0) return FARD_OK;
  if (!x_pending || !x_draft || !mu_q || !n_keep || !r || !eps || !n_accept || !log_ratio || !mu_p)
    return fail(c, FARD_EINVAL, "null argument");
  if (!(sigma_p > 0.f) || !(sigma_q > 0.f)) return fail(c, FARD_EINVAL, "sigma must be > 0");
  Model& m = c->mdl[FARD_TARGET];
  if (pending_id && !m.cond) return fail(c, FARD_EINVAL, "pending_id given but the target has no id table");
  const int K = c->cfg.K, D = m.c.d_latent, M = B * (K + 1);
  if (K + 1 > cap_nq(c, FARD_TARGET)) return fail(c, FARD_ESHAPE, "(K+1) * (n_heads / n_kv_heads) > 64");
  if (m.len_hi + K + 1 > c->cfg.max_ctx) return fail(c, FARD_ECAPACITY, "target cache_len + K + 1 exceeds max_ctx");
  if (m.c.pos == FARD_POS_LEARNED && m.len_hi + K + 1 > m.c.max_pos) return fail(c, FARD_ECAPACITY, "target position beyond the learned table");
  hipStream_t s = c->stream;
  int rc;
  { Bracket br(c, CLS_OTHER);
    copy_i32_kernel<<<(B + 255) / 256, 256, 0, s>>>(m.len, m.len_base, B);
    HIPCHK(c, hipGetLastError());
    HIPCHK(c, launch_build_rows(s, n_keep, 1, B, K, D, m.len, c->maps, x_pending, x_draft, c->x_in, c->aux_row, M, K + 1));
    HIPCHK(c, launch_fill_f32(s, mu_p, 0.f, (size_t)B * (K + 1) * D)); }
  const int* md = c->maps.m_total;
  int* cid = nullptr;
  { Bracket br(c, CLS_OTHER);
    if (pending_id) {
      // per-row ids: row 0 of each sample carries the pending id, every other row is a latent row
      cid = c->row_ids;
      HIPCHK(c, launch_fill_i32(s, cid, -1, M));
      HIPCHK(c, launch_scatter_rows(s, pending_id, cid, c->maps.row_start, 1, 4, B, nullptr));
    }
  }
  HIPCHK(c, embed_first_norm(c, FARD_TARGET, c->x_in, D, cid, M, md));
  if ((rc = run_layers(c, FARD_TARGET, 0, m.c.n_layers, B, M, K + 1, md, 0, true))) return rc;
  if ((rc = run_final(c, FARD_TARGET, M, md, nullptr, c->z))) return rc;
  if (z_p) {
    Bracket br(c, CLS_OTHER);
    HIPCHK(c, launch_scatter_rows(s, c->z, z_p, c->aux_row, m.d_out(), (int)c->esz, M, md));
  }
  if ((rc = run_head(c, c->z, M, md, eps, (size_t)B * (K + 1) * D, c->aux_row, c->aux_row, mu_p, c->x_scratch)))
    return rc;
  { Bracket br(c, CLS_OTHER);
    HIPCHK(c, launch_accept(s, x_draft, mu_p, mu_q, r, n_keep, log_sigma_factor, sigma_p, sigma_q, B, K, D, n_accept, log_ratio,
                            c->acc_tmp)); }
  m.len_hi += K + 1;                       // what a commit may keep at most
  m.written = K + 1;
  return FARD_OK;
}

static int round_eager(fard_ctx* c, const float* x_pending, const int32_t* pending_id, const float* eps, const float* r,
                       float tau, float log_sigma_factor, float sigma_p, float sigma_q, int32_t B, float* H, uint8_t* keep,
                       int32_t* n_keep, float* x_draft, float* mu_q, int32_t* n_accept, float* log_ratio, float* mu_p) {
  int rc = spec_draft(c, x_pending, pending_id, eps, tau, B, H, keep, n_keep, x_draft, mu_q);
  if (rc) return rc;
  rc = spec_verify(c, x_pending, pending_id, x_draft, mu_q, n_keep, r, eps, log_sigma_factor, sigma_p, sigma_q, B, n_accept,
                   log_ratio, mu_p, nullptr);
  if (rc) return rc;
  return spec_kv_commit(c, -1, n_accept, B);
}

// The cache-capacity rules of spec_draft and spec_verify, for a round that launches no kernel of its own.
static int round_capacity(fard_ctx* c) {
  const int K = c->cfg.K;
  for (int w = 0; w < 2; ++w) {
    const Model& m = c->mdl[w];
    const int add = (w == FARD_TARGET) ? K + 1 : K;
    if (m.len_hi + add > c->cfg.max_ctx) return fail(c, FARD_ECAPACITY, "cache_len + K (+ 1) exceeds max_ctx");
    if (m.c.pos == FARD_POS_LEARNED && m.len_hi + add > m.c.max_pos) return fail(c, FARD_ECAPACITY, "position beyond the learned table");
  }
  return FARD_OK;
}

int spec_graph_enable(fard_ctx* c, int32_t on) {
  if (check_ctx(c)) return FARD_EINVAL;
  if (on && c->stream == nullptr) return fail(c, FARD_ESTATE, "rounds on the default stream cannot be captured");
  c->rgraph.drop();
  c->ggraph.drop();
  c->rgraph.on = on != 0;
  return FARD_OK;
}

int spec_round(fard_ctx* c, const float* x_pending, const int32_t* pending_id, const float* eps, const float* r, float tau,
               float log_sigma_factor, float sigma_p, float sigma_q, int32_t B, float* H, uint8_t* keep, int32_t* n_keep,
               float* x_draft, float* mu_q, int32_t* n_accept, float* log_ratio, float* mu_p) {
  if (check_ctx(c)) return FARD_EINVAL;
  RoundGraph& g = c->rgraph;
  auto eager = [&]() {
    return round_eager(c, x_pending, pending_id, eps, r, tau, log_sigma_factor, sigma_p, sigma_q, B, H, keep, n_keep, x_draft,
                       mu_q, n_accept, log_ratio, mu_p);
  };
  if (!g.on || c->prof.on || B <= 0) return eager();
  RoundKey key;
  memset(&key, 0, sizeof(key));
  const void* ptrs[13] = {x_pending, pending_id, eps, r, H, keep, n_keep, x_draft, mu_q, n_accept, log_ratio, mu_p, nullptr};
  memcpy(key.ptr, ptrs, sizeof(ptrs));
  key.f[0] = tau; key.f[1] = log_sigma_factor; key.f[2] = sigma_p; key.f[3] = sigma_q;
  key.B = B;
  const bool same = g.have_key && memcmp(&key, &g.key, sizeof(key)) == 0;
  const int K = c->cfg.K;
  if (same && g.exec) {
    // replay: the kernels read the cache lengths on the device; the host repeats its capacity rules and bounds
    int rc = round_capacity(c);
    if (rc) return rc;
    HIPCHK(c, hipGraphLaunch(g.exec, c->stream));
    c->mdl[FARD_DRAFT].len_hi += K;
    c->mdl[FARD_TARGET].len_hi += K + 1;
    c->mdl[FARD_DRAFT].written = c->mdl[FARD_TARGET].written = 0;
    return FARD_OK;
  }
  if (!same) {
    // first call with these arguments: launch as usual (this also validates them) and remember them
    g.drop();
    int rc = eager();
    if (rc == FARD_OK) {
      g.key = key;
      g.have_key = true;
    }
    return rc;
  }
  // second call in a row with the same arguments: record the launches into a graph, then launch the graph
  int rc = round_capacity(c);
  if (rc) return rc;
  const int hi0[2] = {c->mdl[0].len_hi, c->mdl[1].len_hi}, wr0[2] = {c->mdl[0].written, c->mdl[1].written};
  auto undo = [&]() {
    for (int w = 0; w < 2; ++w) { c->mdl[w].len_hi = hi0[w]; c->mdl[w].written = wr0[w]; }
    c->pend_n = 0;
    g.drop();
  };
  HIPCHK(c, hipStreamBeginCapture(c->stream, hipStreamCaptureModeRelaxed));
  rc = eager();
  hipGraph_t graph = nullptr;
  hipError_t e = hipStreamEndCapture(c->stream, &graph);
  if (rc != FARD_OK || e != hipSuccess || !graph) {
    if (graph) (void)hipGraphDestroy(graph);
    undo();
    if (rc != FARD_OK) return rc;
    return fail(c, FARD_EHIP, std::string("graph capture: ") + hipGetErrorString(e));
  }
  hipGraphExec_t exec = nullptr;
  e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
  if (e == hipSuccess) e = hipGraphLaunch(exec, c->stream);
  if (e != hipSuccess) {
    if (exec) (void)hipGraphExecDestroy(exec);
    (void)hipGraphDestroy(graph);
    undo();
    return fail(c, FARD_EHIP, std::string("graph launch: ") + hipGetErrorString(e));
  }
  g.graph = graph;
  g.exec = exec;
  return FARD_OK;
}

int spec_resample(fard_ctx* c, const float* mu_p, const float* mu_q, const float* eps, const int32_t* n_accept,
                  const int32_t* n_keep, const float* eps_res, const float* u_res, float log_sigma_factor, float sigma_p,
                  float sigma_q, int32_t B, int32_t J, float* x_next, int32_t* tries) {
  if (check_ctx(c)) return FARD_EINVAL;
  if (B < 0 || B > c->cfg.max_batch) return fail(c, FARD_ECAPACITY, "B > max_batch");
  if (J < 1) return fail(c, FARD_EINVAL, "J >= 1 required");
  if (!(sigma_p > 0.f) || !(sigma_q > 0.f)) return fail(c, FARD_EINVAL, "sigma_p, sigma_q > 0 required");
  if (B == 0) return FARD_OK;
  if (!mu_p || !mu_q || !eps || !n_accept || !n_keep || !eps_res || !u_res || !x_next || !tries)
    return fail(c, FARD_EINVAL, "null argument");
  const int K = c->cfg.K, D = c->cfg.target.d_latent, S = c->cfg.head.n_steps;
  const float* eps_last = eps + (size_t)S * B * (K + 1) * D;
  Bracket br(c, CLS_OTHER);
  HIPCHK(c, launch_round_finish(c->stream, mu_p, mu_q, eps_last, n_accept, n_keep, eps_res, u_res, nullptr, B, K, D, J,
                                log_sigma_factor, sigma_p, sigma_q, x_next, tries, nullptr, 0, nullptr));
  return FARD_OK;
}

// One round of generation on the staging buffers: round, closing token, draft catch-up.  The same launches for every
// round, so that a recording of one round replays for all of them.
static int generate_round_staged(fard_ctx* c, bool with_id, float tau, float lsf, float sp, float sq, int B, int J, float* tokens,
                                 int tok_cap, int* n_tokens) {
  const int K = c->cfg.K, D = c->cfg.target.d_latent, S = c->cfg.head.n_steps;
  hipStream_t s = c->stream;
  int rc = round_eager(c, c->g_next, with_id ? c->s_pid : nullptr, c->s_eps, c->s_r, tau, lsf, sp, sq, B, c->s_H, c->g_keep, c->s_nk,
                       c->g_x, c->g_mu_q, c->s_na, c->g_lr, c->g_mu_p);
  if (rc) return rc;
  { Bracket br(c, CLS_OTHER);
    HIPCHK(c, launch_round_finish(s, c->g_mu_p, c->g_mu_q, c->s_eps + (size_t)S * B * (K + 1) * D, c->s_na, c->s_nk, c->s_eres,
                                  c->s_ures, c->g_x, B, K, D, J, lsf, sp, sq, c->g_next, c->s_tr, tokens, tok_cap, n_tokens));
    HIPCHK(c, launch_catchup_pack(s, c->s_na, c->g_x, B, K, D, c->g_cu_nq, c->g_cu_x)); }
  return spec_forward(c, FARD_DRAFT, c->g_cu_x, nullptr, c->g_cu_nq, 1, B, B, 1, c->z, nullptr, nullptr);
}

static int generate_staged(fard_ctx* c, const float* x_first, const int32_t* first_id, const float* eps, const float* r,
                           const float* eps_res, const float* u_res, float tau, float lsf, float sp, float sq, int B, int R, int J,
                           float* tokens, int32_t* n_tokens, float* H, int32_t* n_keep, int32_t* n_accept, int32_t* tries) {
  const int K = c->cfg.K, D = c->cfg.target.d_latent, S = c->cfg.head.n_steps;
  hipStream_t s = c->stream;
  const size_t n_eps = (size_t)(S + 1) * B * (K + 1) * D, n_r = (size_t)B * K, n_eres = (size_t)B * J * D, n_ures = (size_t)B * J;
  const int tok_cap = R * (K + 1);
  RoundGraph& g = c->ggraph;
  RoundKey key;
  memset(&key, 0, sizeof(key));
  key.ptr[0] = tokens; key.ptr[1] = n_tokens; key.ptr[2] = first_id ? c->s_pid : nullptr;
  key.f[0] = tau; key.f[1] = lsf; key.f[2] = sp; key.f[3] = sq;
  key.B = B; key.pad = J * 65536 + R;
  if (!(g.have_key && memcmp(&key, &g.key, sizeof(key)) == 0)) {
    g.drop();
    g.key = key;
    g.have_key = true;
  }
  HIPCHK(c, hipMemcpyAsync(c->g_next, x_first, (size_t)B * D * 4, hipMemcpyDeviceToDevice, s));
  if (first_id) { copy_i32_kernel<<<(B + 255) / 256, 256, 0, s>>>(first_id, c->s_pid, B); HIPCHK(c, hipGetLastError()); }
  bool ran_eager = false;
  for (int t = 0; t < R; ++t) {
    { Bracket br(c, CLS_OTHER);
      const size_t total = n_eps + n_r + n_eres + n_ures;
      gen_stage_in_kernel<<<(unsigned)std::min<size_t>((total + 255) / 256, 1024), 256, 0, s>>>(
          eps + t * n_eps, r + t * n_r, eps_res + t * n_eres, u_res + t * n_ures, n_eps, n_r, n_eres, n_ures, c->s_eps, c->s_r,
          c->s_eres, c->s_ures);
      HIPCHK(c, hipGetLastError());
      if (t == 1 && first_id) HIPCHK(c, launch_fill_i32(s, c->s_pid, -1, B)); }   // later pending tokens are latents
    int rc = FARD_OK;
    if (g.exec) {
      HIPCHK(c, hipGraphLaunch(g.exec, s));
      c->mdl[FARD_DRAFT].len_hi += K + 1;
      c->mdl[FARD_TARGET].len_hi += K + 1;
      c->mdl[FARD_DRAFT].written = c->mdl[FARD_TARGET].written = 0;
    } else if (!ran_eager) {
      // the first round of a new argument set is launched kernel by kernel (it validates, and every kernel has run once)
      rc = generate_round_staged(c, first_id != nullptr, tau, lsf, sp, sq, B, J, tokens, tok_cap, n_tokens);
      ran_eager = true;
    } else {
      const int hi0[2] = {c->mdl[0].len_hi, c->mdl[1].len_hi}, wr0[2] = {c->mdl[0].written, c->mdl[1].written};
      HIPCHK(c, hipStreamBeginCapture(s, hipStreamCaptureModeRelaxed));
      rc = generate_round_staged(c, first_id != nullptr, tau, lsf, sp, sq, B, J, tokens, tok_cap, n_tokens);
      hipGraph_t graph = nullptr;
      hipError_t e = hipStreamEndCapture(s, &graph);
      hipGraphExec_t exec = nullptr;
      if (rc == FARD_OK && e == hipSuccess && graph) e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
      if (rc == FARD_OK && e == hipSuccess && exec) e = hipGraphLaunch(exec, s);
      if (rc != FARD_OK || e != hipSuccess || !exec) {
        if (exec) (void)hipGraphExecDestroy(exec);
        if (graph) (void)hipGraphDestroy(graph);
        for (int w = 0; w < 2; ++w) { c->mdl[w].len_hi = hi0[w]; c->mdl[w].written = wr0[w]; }
        c->pend_n = 0;
        g.drop();
        if (rc != FARD_OK) return rc;
        return fail(c, FARD_EHIP, std::string("graph of a generation round: ") + hipGetErrorString(e));
      }
      g.graph = graph;
      g.exec = exec;
    }
    if (rc) return rc;
    { Bracket br(c, CLS_OTHER);
      const int BK = B * K;
      gen_stage_out_kernel<<<(BK + 255) / 256, 256, 0, s>>>(c->s_H, c->s_nk, c->s_na, c->s_tr, BK, B, H + (size_t)t * BK,
                                                          n_keep + (size_t)t * B, n_accept + (size_t)t * B, tries + (size_t)t * B);
      HIPCHK(c, hipGetLastError()); }
  }
  return FARD_OK;
}

int spec_generate(fard_ctx* c, const float* x_first, const int32_t* first_id, const float* eps, const float* r,
                  const float* eps_res, const float* u_res, float tau, float log_sigma_factor, float sigma_p, float sigma_q,
                  int32_t B, int32_t R, int32_t J, float* tokens, int32_t* n_tokens, float* H, int32_t* n_keep,
                  int32_t* n_accept, int32_t* tries) {
  if (check_ctx(c)) return FARD_EINVAL;
  if (B < 0 || B > c->cfg.max_batch) return fail(c, FARD_ECAPACITY, "B > max_batch");
  if (R < 0 || J < 1) return fail(c, FARD_EINVAL, "R >= 0 and J >= 1 required");
  if (B == 0 || R == 0) return FARD_OK;
  if (!x_first || !eps || !r || !eps_res || !u_res || !tokens || !n_tokens || !H || !n_keep || !n_accept || !tries)
    return fail(c, FARD_EINVAL, "null argument");
  const int K = c->cfg.K, D = c->cfg.target.d_latent, S = c->cfg.head.n_steps;
  // the host only knows upper bounds of the cache lengths: every round may add K + 1 positions
  for (int w = 0; w < 2; ++w) {
    const Model& m = c->mdl[w];
    const long need = (long)m.len_hi + (long)R * (K + 1);
    if (need > c->cfg.max_ctx) return fail(c, FARD_ECAPACITY, "cache_len + R * (K + 1) exceeds max_ctx");
    if (m.c.pos == FARD_POS_LEARNED && need > m.c.max_pos) return fail(c, FARD_ECAPACITY, "positions beyond the learned table");
  }
  hipStream_t s = c->stream;
  const size_t eps_round = (size_t)(S + 1) * B * (K + 1) * D;
  const int tok_cap = R * (K + 1);
  HIPCHK(c, launch_fill_i32(s, n_tokens, 0, B));
  uint8_t* keep = c->g_keep;
  if (c->rgraph.on && !c->prof.on && J <= GEN_J_MAX)
    return generate_staged(c, x_first, first_id, eps, r, eps_res, u_res, tau, log_sigma_factor, sigma_p, sigma_q, B, R, J, tokens,
                           n_tokens, H, n_keep, n_accept, tries);
  for (int t = 0; t < R; ++t) {
    const float* eps_t = eps + (size_t)t * eps_round;
    int rc = round_eager(c, t == 0 ? x_first : c->g_next, t == 0 ? first_id : nullptr, eps_t, r + (size_t)t * B * K, tau,
                        log_sigma_factor, sigma_p, sigma_q, B, H + (size_t)t * B * K, keep, n_keep + (size_t)t * B, c->g_x,
                        c->g_mu_q, n_accept + (size_t)t * B, c->g_lr, c->g_mu_p);
    if (rc) return rc;
    { Bracket br(c, CLS_OTHER);
      HIPCHK(c, launch_round_finish(s, c->g_mu_p, c->g_mu_q, eps_t + (size_t)S * B * (K + 1) * D, n_accept + (size_t)t * B,
                                    n_keep + (size_t)t * B, eps_res + (size_t)t * B * J * D, u_res + (size_t)t * B * J, c->g_x,
                                    B, K, D, J, log_sigma_factor, sigma_p, sigma_q, c->g_next, tries + (size_t)t * B, tokens,
                                    tok_cap, n_tokens));
      // a draft that accepted all K drafts has not read draft K yet
      HIPCHK(c, launch_catchup_pack(s, n_accept + (size_t)t * B, c->g_x, B, K, D, c->g_cu_nq, c->g_cu_x)); }
    rc = spec_forward(c, FARD_DRAFT, c->g_cu_x, nullptr, c->g_cu_nq, 1, B, B, 1, c->z, nullptr, nullptr);
    if (rc) return rc;
  }
  return FARD_OK;
}

int spec_gemm(fard_ctx* c, const void* A, const void* W, const float* bias, int32_t M, int32_t K, int32_t N, int32_t act, void* out) {
  if (check_ctx(c)) return FARD_EINVAL;
  if (M < 0 || K < 1 || N < 1) return fail(c, FARD_ESHAPE, "M >= 0, K, N >= 1 required");
  if (M == 0) return FARD_OK;
  if (!A || !W || !out) return fail(c, FARD_EINVAL, "null argument");
  if (act < 0 || act > 2) return fail(c, FARD_EINVAL, "act");
  const void* Wk = W;
  if (c->bf16) {
    if (K % 64 != 0 || N % 32 != 0) return fail(c, FARD_ESHAPE, "bf16 GEMM needs K % 64 == 0 and N % 32 == 0");
    const size_t bytes = (size_t)K * N * 2;
    if (bytes > c->gemm_tmp_bytes) {
      HIPCHK(c, hipStreamSynchronize(c->stream));
      if (c->gemm_tmp) (void)hipFree(c->gemm_tmp);
      c->gemm_tmp = nullptr;
      c->gemm_tmp_bytes = 0;
      HIPCHK(c, hipMalloc(&c->gemm_tmp, bytes));
      c->gemm_tmp_bytes = bytes;
    }
    HIPCHK(c, launch_pack_weight(c->stream, W, 1, N, K, N, c->gemm_tmp, 0, 1));
    Wk = c->gemm_tmp;
  }
  HIPCHK(c, gemm(c, A, K, Wk, bias, out, N, M, N, K, nullptr, EPI_STORE, act));
  return FARD_OK;
}

int spec_gemm_narrow(fard_ctx* c, const void* A, const void* W, const float* bias, const float* gate, int32_t M,
                     int32_t K, int32_t N, int32_t epi, int32_t act, void* out, void* out_bf16) {
  if (check_ctx(c)) return FARD_EINVAL;
  if (!c->bf16) return fail(c, FARD_EINVAL, "spec_gemm_narrow needs a bf16 context");
  if (M < 0 || K < 1 || N < 1) return fail(c, FARD_ESHAPE, "M >= 0, K, N >= 1 required");
  if (M == 0) return FARD_OK;
  if (!A || !W || !out) return fail(c, FARD_EINVAL, "null argument");
  if (act < 0 || act > 2 || epi < 0 || epi > 3) return fail(c, FARD_EINVAL, "selector");
  if (epi == 3 && !gate) return fail(c, FARD_EINVAL, "epi 3 needs gate");
  if (out_bf16 && epi < 2) return fail(c, FARD_EINVAL, "out_bf16 goes with epi 2 or 3");
  GemmArgs a;
  a.A = A; a.lda = K; a.W = nullptr; a.bias = bias; a.out = out; a.ldo = N; a.gate = gate; a.ldg = N;
  a.M = M; a.N = N; a.K = K; a.m_dev = nullptr; a.act = act; a.epi = epi;
  a.copy_bf16 = out_bf16;
  if (!narrow_supported(a) || M > 1024) return fail(c, FARD_ESHAPE, "narrow GEMM needs M <= 1024, K % 64 == 0, N % 32 == 0");
  const size_t bytes = (size_t)K * N * 2;
  if (bytes > c->gemm_tmp_bytes) {
    HIPCHK(c, hipStreamSynchronize(c->stream));
    if (c->gemm_tmp) (void)hipFree(c->gemm_tmp);
    c->gemm_tmp = nullptr;
    c->gemm_tmp_bytes = 0;
    HIPCHK(c, hipMalloc(&c->gemm_tmp, bytes));
    c->gemm_tmp_bytes = bytes;
  }
  HIPCHK(c, launch_pack_weight(c->stream, W, 1, N, K, N, c->gemm_tmp, 0, 1));
  a.W = c->gemm_tmp;
  { Bracket br(c, CLS_GEMM_NARROW, 2.0 * M * (double)N * K, (double)K * N * 2);
    HIPCHK(c, launch_gemm_narrow(c->stream, a)); }
  return FARD_OK;
}

int spec_gemm_norm(fard_ctx* c, const void* x, const void* W, const float* g, const float* beta, const float* bias, int32_t M,
                   int32_t K, int32_t N, int32_t norm_type, float eps, int32_t act, void* out) {
  if (check_ctx(c)) return FARD_EINVAL;
  if (!c->bf16) return fail(c, FARD_EINVAL, "spec_gemm_norm needs a bf16 context");
  if (M < 0 || K < 1 || N < 1) return fail(c, FARD_ESHAPE, "M >= 0, K, N >= 1 required");
  if (M == 0) return FARD_OK;
  if (!x || !W || !g || !out) return fail(c, FARD_EINVAL, "null argument");
  if (act < 0 || act > 2 || (norm_type != FARD_NORM_LAYER && norm_type != FARD_NORM_RMS)) return fail(c, FARD_EINVAL, "selector");
  if (K % 64 != 0 || N % 32 != 0 || M > 1024) return fail(c, FARD_ESHAPE, "needs M <= 1024, K % 64 == 0, N % 32 == 0");
  // scratch: diag(g) W as bf16 [K, N], its packed form, column sums and folded bias
  const size_t wbytes = (size_t)K * N * 2, bytes = 2 * wbytes + (size_t)N * 8 + 256;
  if (bytes > c->gemm_tmp_bytes) {
    HIPCHK(c, hipStreamSynchronize(c->stream));
    if (c->gemm_tmp) (void)hipFree(c->gemm_tmp);
    c->gemm_tmp = nullptr;
    c->gemm_tmp_bytes = 0;
    HIPCHK(c, hipMalloc(&c->gemm_tmp, bytes));
    c->gemm_tmp_bytes = bytes;
  }
  char* base = (char*)c->gemm_tmp;
  bf16* scaled = (bf16*)base;
  void* packed = base + wbytes;
  float* cs = (float*)(base + 2 * wbytes);
  float* bf = cs + N;
  ln_fold_kernel<bf16><<<(N + 127) / 128, 128, 0, c->stream>>>((const bf16*)W, g, norm_type == FARD_NORM_LAYER ? beta : nullptr, bias,
                                                             K, N, scaled, cs, bf);
  HIPCHK(c, hipGetLastError());
  HIPCHK(c, launch_pack_weight(c->stream, scaled, 1, N, K, N, packed, 0, 1));
  GemmArgs a;
  a.A = x; a.lda = K; a.W = packed; a.bias = bf; a.out = out; a.ldo = N; a.gate = nullptr; a.ldg = 0;
  a.M = M; a.N = N; a.K = K; a.m_dev = nullptr; a.act = act; a.epi = EPI_STORE;
  a.ln_cs = cs; a.ln_eps = eps; a.ln_rms = norm_type == FARD_NORM_RMS;
  if (!narrow_supported(a)) return fail(c, FARD_ESHAPE, "unsupported shape");
  { Bracket br(c, CLS_GEMM_NARROW, 2.0 * M * (double)N * K, (double)K * N * 2);
    HIPCHK(c, launch_gemm_narrow(c->stream, a)); }
  return FARD_OK;
}

int spec_peak_probe(fard_ctx* c, int32_t kind, const void* buf, int64_t bytes, int32_t iters, int32_t reps, float* ms_per_launch,
                    double* units_per_launch) {
  if (check_ctx(c)) return FARD_EINVAL;
  if (kind != 0 && kind != 1) return fail(c, FARD_EINVAL, "kind must be 0 (read) or 1 (MFMA)");
  if (reps < 1 || reps > 1000) return fail(c, FARD_EINVAL, "1 <= reps <= 1000 required");
  if (!ms_per_launch || !units_per_launch) return fail(c, FARD_EINVAL, "null argument");
  if (kind == 0 && (!buf || bytes < 16 || bytes % 16 != 0 || ((uintptr_t)buf & 15))) return fail(c, FARD_ESHAPE, "buf: 16-byte aligned, bytes a positive multiple of 16");
  if (kind == 1 && (iters < 1 || iters > (1 << 20))) return fail(c, FARD_EINVAL, "1 <= iters <= 2^20 required");
  const int blocks = 2048;  // eight workgroups of four waves per compute unit
  int rc = loss_scratch(c, probe_sink_bytes(kind, blocks));
  if (rc) return rc;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  HIPCHK(c, hipEventCreate(&e0));
  if (hipEventCreate(&e1) != hipSuccess) {
    (void)hipEventDestroy(e0);
    return fail(c, FARD_EHIP, "hipEventCreate failed");
  }
  hipError_t err = hipSuccess;
  for (int r = -1; r < reps && err == hipSuccess; ++r) {  // launch -1 warms up
    if (r == 0) err = hipEventRecord(e0, c->stream);
    if (err == hipSuccess) err = kind == 0 ? launch_probe_read(c->stream, buf, (long)bytes, blocks, c->loss_tmp) : launch_probe_mfma(c->stream, iters, blocks, c->loss_tmp);
  }
  if (err == hipSuccess) err = hipEventRecord(e1, c->stream);
  if (err == hipSuccess) err = hipEventSynchronize(e1);
  float ms = 0.f;
  if (err == hipSuccess) err = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (err != hipSuccess) return fail(c, FARD_EHIP, hipGetErrorString(err));
  *ms_per_launch = ms / reps;
  // one 32x32x16 MFMA is 2*32*32*16 flop; four per iteration per wave, four waves per workgroup
  *units_per_launch = kind == 0 ? (double)bytes : (double)blocks * 4.0 * 4.0 * (double)iters * 32768.0;
  return FARD_OK;
}

int spec_profile_enable(fard_ctx* c, int32_t enable) {
  if (check_ctx(c)) return FARD_EINVAL;
  HIPCHK(c, hipStreamSynchronize(c->stream));
  c->prof.on = enable != 0;
  c->prof.used = 0;
  for (int i = 0; i < CLS_COUNT; ++i) c->prof.flops[i] = c->prof.bytes[i] = 0;
  return FARD_OK;
}

int spec_profile_read(fard_ctx* c, int32_t kernel_class, float* total_ms, int64_t* launches, double* flops, double* bytes) {
  if (check_ctx(c)) return FARD_EINVAL;
  if (kernel_class < 0 || kernel_class >= CLS_COUNT) return fail(c, FARD_EINVAL, "kernel_class");
  HIPCHK(c, hipStreamSynchronize(c->stream));
  float tot = 0.f;
  int64_t n = 0;
  for (size_t i = 0; i < c->prof.used; ++i) {
    if (c->prof.cls[i] != kernel_class) continue;
    float ms = 0.f;
    HIPCHK(c, hipEventElapsedTime(&ms, c->prof.pool[i].first, c->prof.pool[i].second));
    tot += ms;
    ++n;
  }
  if (total_ms) *total_ms = tot;
  if (launches) *launches = n;
  if (flops) *flops = c->prof.flops[kernel_class];
  if (bytes) *bytes = c->prof.bytes[kernel_class];
  return FARD_OK;
}

}  // extern "C"

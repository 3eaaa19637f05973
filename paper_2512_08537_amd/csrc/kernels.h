// Host-side launchers of the non-GEMM kernels.  T is the activation/weight storage type:
// `is_bf16` selects bf16 (MFMA path, fragment-packed KV cache) or fp32 (plain layouts).
#pragma once
#include "common.h"

namespace fard {

// ------------------------------------------------------------------ KV cache geometry
// bf16 path: per (layer, sample, kv head) the K region and the V region are each
// ctx_pad * d_head elements (ctx_pad a multiple of 32), stored in blocks of 32 positions laid
// out in MFMA operand order (see attn.hip).  fp32 path: plain [pos][d_head].
struct KvGeom {
  void* k;            // base of this layer's K storage
  void* v;
  int n_kv_heads, d_head, ctx_pad;
  int is_bf16;
};

// ------------------------------------------------------------------ row maps of a packed batch
struct RowMaps {
  int* row_start;     // [B+1] exclusive scan of n_q
  int* row_sample;    // [M]
  int* row_j;         // [M] index inside the sample's rows
  int* row_pos;       // [M] absolute position = cache_len[sample] + row_j
  int* m_total;       // [1] number of packed rows
};

// n_q = n_base[b] + add (n_base may be null -> n_q = add).  Also gathers the fp32 latent rows when
// x_first/x_rest are given: row j = 0 takes x_first[b, :], row j >= 1 takes x_rest[b, j-1, :]
// (x_rest is [B, K, D]); aux_row[r] = b * (K+1) + j indexes per-token side tensors.  n_q is clamped
// to nq_cap and rows beyond m_max are dropped, so downstream kernels never index out of bounds.
hipError_t launch_build_rows(hipStream_t s, const int* n_base, int add, int B, int K, int D,
                             const int* cache_len, RowMaps maps, const float* x_first,
                             const float* x_rest, float* x_out, int* aux_row, int m_max, int nq_cap);

// h[r, :] = x[r, :] W_in + b_in (+ pos[row_pos[r], :]) ; rows with cond_id[r] >= 0 take cond[id, :].
hipError_t launch_embed(hipStream_t s, int is_bf16, const float* x, int ldx, int D, const void* w_in,
                        const float* b_in, const void* pos_table, const int* row_pos,
                        const void* cond_table, const int* cond_id, float* h, int d, int M,
                        const int* m_dev);

// launch_embed followed by the norm of the same rows (gain g, bias b; norm_type 0 LayerNorm, 1 RMSNorm) into u, in
// one launch.
hipError_t launch_embed_norm(hipStream_t s, int is_bf16, const float* x, int ldx, int D, const void* w_in, const float* b_in,
                             const void* pos_table, const int* row_pos, const void* cond_table, const int* cond_id, float* h,
                             int d, int M, const int* m_dev, int norm_type, float eps, const float* g, const float* b, void* u,
                             int u_tiled = 0);

// out_T[r, :] = norm(h[r, :]) with optional affine (g, b) and optional AdaLN modulation
// (1 + scale[r, :]) / shift[r, :] read with row stride ldm.  norm_type 0 LayerNorm, 1 RMSNorm.
// in_map (optional) gathers: output row r is computed from input row in_map[r].
hipError_t launch_norm(hipStream_t s, int is_bf16, const float* h, int d, int M, const int* m_dev,
                       int norm_type, float eps, const float* g, const float* b, const float* shift,
                       const float* scale, int ldm, const int* in_map, void* out,
                       const float* parts = nullptr, int n_parts = 0, size_t part_stride = 0, float* h_wb = nullptr,
                       int out_tiled = 0);
// parts / n_parts / part_stride: K-slice partial sums [n_parts][M, d] that a preceding GEMM left for the
// residual stream; the norm adds them to its input row first and writes the completed row to h_wb (if given).
hipError_t launch_add_parts(hipStream_t s, float* h, const float* parts, int n_parts, size_t part_stride, int d,
                            int M, const int* m_dev);

// ---- KV cache addressing (device side)
// bf16 cache, blocks of 32 positions.  K block: [d/16][lane][8] with lane = (pos%32) + 32*((d%16)/8):
// the A operand of v_mfma_f32_32x32x16_bf16 with keys as rows.  V block: [d/32][half][lane][8] with
// lane = d%32 + 32*g, holding the 8 keys {16*half + 8*(i/4) + 4*g + i%4}: the A operand of the
// P*V product with dims as rows, keys ordered the way the score accumulators hold them.
__device__ __forceinline__ size_t k_offset_bf16(int pos, int d, int dh) {
  const int kb = pos >> 5, lr = pos & 31;
  const int dc = d >> 4, g = (d >> 3) & 1, i = d & 7;
  return (size_t)kb * 32 * dh + ((size_t)(dc * 64 + lr + 32 * g) << 3) + i;
}
__device__ __forceinline__ size_t v_offset_bf16(int pos, int d, int dh) {
  const int kb = pos >> 5, pk = pos & 31;
  const int hf = pk >> 4, rem = pk & 15;
  const int g = (rem >> 2) & 1, i = ((rem >> 3) << 2) | (rem & 3);
  const int db = d >> 5, lane = (d & 31) + 32 * g;
  return (size_t)kb * 32 * dh + ((size_t)((db * 2 + hf) * 64 + lane) << 3) + i;
}

// Splits qkv[M, (H+2Hkv) dh] rows: optional RoPE on q (in place) and k, then stores k, v at
// position row_pos[r] of sample row_sample[r] in the cache.
hipError_t launch_rope_append(hipStream_t s, void* qkv, int ld, int n_heads, KvGeom kv, int rope,
                              float rope_theta, const int* row_sample, const int* row_pos, int M,
                              const int* m_dev);

// The same with the rows still in the K-slice planes of the QKV product (fp32 [n_parts][M, ld], plane p at
// parts + p * part_stride): the planes are summed, q and k rotated in fp32; q goes to qkv as bf16 (the k and v columns of
// qkv are not written), k and v to the cache.  bf16 caches only.
hipError_t launch_rope_append_planes(hipStream_t s, const float* parts, int n_parts, size_t part_stride, void* qkv, int ld,
                                     int n_heads, KvGeom kv, int rope, float rope_theta, const int* row_sample,
                                     const int* row_pos, int M, const int* m_dev);

// Copies plain [B, Hkv, n, dh] tensors (storage type of the context) into the cache at positions 0..n-1.
hipError_t launch_kv_load(hipStream_t s, KvGeom kv, const void* k, const void* v, int B, int n);

// Cached causal attention.  q rows come from qkv (row r, head g at column g*dh); output
// out_T[r, g*dh + :].  ent_heads[r, g] (optional) receives the entropy of the attention row.
// append != 0 (bf16 caches, no RoPE): the kernel itself stores the new rows' K and V at positions
// cache_len[b] .. + n_q - 1 before it reads them, replacing a separate launch_rope_append.
// row_cnt (optional): sample b contributes row_cnt[b] rows starting at row_start[b] (a pass over part of a sample's
// rows; cache_len[b] is then the position of the first of them); without it the rows are row_start[b] .. row_start[b+1].
// n_pass > 1: that many passes in one launch; pass p reads entries [p * B, (p + 1) * B) of cache_len, row_start and
// row_cnt.  The K / V rows of all passes must be in the cache already (append == 0).
// split (optional, n > 1; bf16, append == 0, n_pass == 1): the 32-key blocks of every (sample, kv head) are dealt to n
// workgroups, each leaving its running softmax triple and unnormalised output rows in the planes of `split`, and a
// second launch folds them (few samples x kv heads against a long context would otherwise occupy a fraction of the
// chip).  M / m_dev: packed rows of the call (host bound / optional device count), needed by that second launch.
struct AttnSplit {
  int n;              // workgroups per (sample, kv head)
  int rows;           // row capacity of the planes
  float* o;           // [n][rows][n_heads][d_head] unnormalised outputs, relative to the split's own maximum
  float* mla;         // [n][rows][n_heads][4] running maximum, sum, entropy accumulator
};
hipError_t launch_attention(hipStream_t s, const void* qkv, int ld, int n_heads, KvGeom kv,
                            const int* cache_len, const int* row_start, int B, int nq_max,
                            void* out, int ldo, float* ent_heads, int append, const int* row_cnt = nullptr,
                            int n_pass = 1, const AttnSplit* split = nullptr, int M = 0, const int* m_dev = nullptr,
                            int out_tiled = 0);

// Shallow-feature entropy + threshold + prefix rule + compaction.  feat: [B, K, L] storage type.
// Up to ENT_SAMPLE_MODE_MIN_B samples: a wave per row, then one workgroup thresholds and compacts.  Above: a
// wave per sample applies the prefix rule itself and a second launch compacts in parallel through
// blk_cnt[ENT_MAX_BLOCKS].
constexpr int ENT_SAMPLE_MODE_MIN_B = 1024;
constexpr int ENT_MAX_BLOCKS = 2048;
hipError_t launch_entropy_prefilter(hipStream_t s, int is_bf16, const void* feat, int B, int K, int L,
                                    float tau, float* H, uint8_t* keep, int* n_keep, int* surv_idx,
                                    int* n_surv, int* blk_cnt);

// H[r] = softmax entropy of the fp32 row feat[r*ld .. r*ld+L) (one wave per row).
// parts (n_parts > 0): pending partial planes added to the rows on the fly; only when ent_rows_in_regs_f32 holds.
bool ent_rows_in_regs_f32(const float* feat, int ld, int L);
hipError_t launch_entropy_rows_f32(hipStream_t s, const float* feat, int ld, int rows, int L, float* H,
                                   const float* parts = nullptr, int n_parts = 0, size_t part_stride = 0);

// One draft step's threshold on per-row entropies already computed elsewhere (ATTN mode) or per
// head (mean over heads taken here): alive[b] &= (H >= tau); n_keep[b] += alive[b]; writes H and keep
// at column `step` of [B, K] arrays and compacts the alive sample indices into act_idx / n_act with the
// matching noise rows emap = b*(K+1)+step and output rows omap = b*K+step.
hipError_t launch_entropy_step(hipStream_t s, const float* ent_heads, int n_heads, const float* H_in,
                               int B, int K, int step, float tau, float* H, uint8_t* keep,
                               int* alive, int* n_keep, int* act_idx, int* n_act, int* emap, int* omap);

// Head pieces.
// hh[r, :] = x_t[r, :] W_in + b_in ; sc[k n + r, :] = T(silu(cz[r, :] + temb[k, :])) for the S sampler
// times k.  x_t comes from xsrc[xmap ? xmap[r] : r] * xscale.
hipError_t launch_head_prep(hipStream_t s, int is_bf16, const float* xsrc, const int* xmap, float xscale,
                            int D, const void* w_in, const float* b_in, const float* cz,
                            const float* temb, int S, float* hh, void* sc, float* xt_out, int w, int n,
                            const int* n_dev);

struct HeadStepArgs {
  const float* hh; int w;            // residual stream of the head [n, w]
  const float* shift; const float* scale; int ldm;   // final modulation
  const void* w_out; const float* b_out; int D;      // [w, D] storage type
  float* xt;                          // [n, D] current x_t (updated in place for the next step)
  const float* eps_next;              // noise of the next transition, row-mapped (may be null)
  const int* emap;                    // row -> row of eps (null = identity)
  const int* omap;                    // row -> row of mu / x (null = identity)
  float t, t_next;                    // current / next time
  int last;                           // 1: write mu, x ; 0: advance x_t
  int renoise;
  float sigma;                        // sigma_last * temperature (last step)
  float* mu; float* x;                // outputs of the last step, row-mapped
  const void* w_in; const float* b_in;   // input projection [D, w] of the next step (not last)
  float* hh_next;                     // [n, w] residual stream of the next step (may alias hh)
  int n; const int* n_dev;
};
hipError_t launch_head_out(hipStream_t s, int is_bf16, const HeadStepArgs& a);

// out[n] = act(sum_k in[k] W[k, n] + b[n]) for one fp32 vector (time embedding at init).
hipError_t launch_matvec(hipStream_t s, int is_bf16, const float* in, const void* W, const float* b,
                         int K, int N, int act, float* out);

// ln rho, acc flags and the length of the leading accepted run.
hipError_t launch_accept(hipStream_t s, const float* x, const float* mu_p, const float* mu_q,
                         const float* r, const int* n_keep, float log_sigma, float sigma_p,
                         float sigma_q, int B, int K, int D, int* n_accept, float* log_ratio,
                         uint8_t* acc);

// The token every sample's round ends with (Alg. 1 Step 5; bonus row when all kept drafts were accepted), one
// wave per sample; optionally appends accepted drafts + that token to tokens[b, n_tokens[b] ...] (capacity tok_cap).
hipError_t launch_round_finish(hipStream_t s, const float* mu_p, const float* mu_q, const float* eps_last,
                               const int* n_accept, const int* n_keep, const float* eps_res, const float* u_res,
                               const float* x_draft, int B, int K, int D, int J, float log_sigma, float sigma_p,
                               float sigma_q, float* x_next, int* tries, float* tokens, int tok_cap, int* n_tokens);
// nq[b] = (n_accept[b] == K); x_pack = draft K of those samples, packed in sample order.
hipError_t launch_catchup_pack(hipStream_t s, const int* n_accept, const float* x_draft, int B, int K, int D,
                               int* nq, float* x_pack);

// cache_len[b] += base + (n ? n[b] : 0)
// row_pos (optional, one row per sample): row b's position is refreshed to the new length
hipError_t launch_len_add(hipStream_t s, int* cache_len, const int* n, int base, int B, int* row_pos = nullptr);
hipError_t launch_fill_i32(hipStream_t s, int* p, int v, int n);
hipError_t launch_fill_f32(hipStream_t s, float* p, float v, size_t n);
// copy rows: dst[dmap ? dmap[r] : r, :] = src[r, :] for r < n (fp32 or storage type by elem_size)
hipError_t launch_scatter_rows(hipStream_t s, const void* src, void* dst, const int* dmap, int width,
                               int elem_size, int n, const int* n_dev);

// ---- training-side losses (losses.hip) -------------------------------------------------------------------
// Byte offsets of the scratch areas of launch_entropy_loss inside one buffer of `bytes` bytes (256-byte aligned base).
constexpr int ENT_LOSS_PARTS = 1024;      // partial sums of the loss reduction
struct EntLossScratch {
  size_t qT, kT, lse, hrow, partial, bytes;
};
EntLossScratch entropy_loss_scratch(int B, int H, int Hkv, int R, int dh);
// Attention-entropy loss of causal attention maps and its gradients.  q [B, H, R, dh], k [B, Hkv, R, dh] bf16;
// loss fp32 [1]; h_rows fp32 [B, H, R] or null; dq fp32 like q or null; dk fp32 like k or null.  dh in {32, 64, 128}.
hipError_t launch_entropy_loss(hipStream_t s, const void* q, const void* k, int B, int H, int Hkv, int R, int dh, void* scratch,
                               float* loss, float* h_rows, float* dq, float* dk);
// Smooth-L1 loss (mean over n elements) and its gradient; partial: n_part floats of scratch.
hipError_t launch_smooth_l1(hipStream_t s, int is_bf16, const void* pred, const void* target, long n, float beta, float* partial,
                            int n_part, float* loss, float* dpred);

// Peak probes (a streaming read, a register-only MFMA loop); sink: probe_sink_bytes(kind, blocks) bytes of scratch.
size_t probe_sink_bytes(int kind, int blocks);
hipError_t launch_probe_read(hipStream_t s, const void* buf, long bytes, int blocks, void* sink);
hipError_t launch_probe_mfma(hipStream_t s, int iters, int blocks, void* sink);

}  // namespace fard

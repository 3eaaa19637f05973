/* fastardiff.h - C ABI of the MI355X (gfx950) speculative-round library.
 *
 * One entropy-informed speculative decoding round for continuous-token AR + diffusion-head
 * generators, after Fast-ARDiff (Alg. 1 of the supplement; Sec. 4.3; Eq. 1; S2.1; S3):
 *   draft K latent tokens one by one with a small AR transformer and the shared diffusion head,
 *   stopping a sample at the first draft step whose shallow-layer entropy is below tau_ent;
 *   verify the surviving drafts in ONE KV-cached forward of the target transformer;
 *   decode the target-side means with the same per-step noise; accept the longest prefix that
 *   passes the continuous ratio test.
 *
 * Conventions
 *  - Every function returns FARD_OK (0) or a negative fard_status; none throws, aborts or exits.
 *    spec_last_error() gives the text of the last failure of a context.
 *  - Every array argument is CALLER-OWNED DEVICE memory unless the comment says "host".
 *    The context owns only what spec_round_init allocates (packed weights, KV caches, workspace).
 *  - All work is enqueued on the HIP stream given to spec_round_init and the calls return
 *    without synchronising (exceptions are marked "synchronises").  Outputs are valid once the
 *    caller has synchronised that stream.  Calls on one context must not overlap.
 *  - "storage type" = the context's dtype: FARD_F32 (float) or FARD_BF16 (bfloat16, arithmetic
 *    accumulates in fp32).  Latents, noise, means, entropies and uniforms are always fp32.
 *  - Row-major everywhere.  Shapes in brackets.
 *  - Token bookkeeping: the caches hold every accepted token except the newest, the PENDING
 *    token.  Draft step i reads token i-1 (the pending token for i = 1) and produces token i;
 *    verify row j reads token j and yields the target's distribution of token j+1.
 *    eps[:, b, j, :] is the noise trajectory of token j+1, shared by draft and target (S3 item 1).
 */
#ifndef FASTARDIFF_H
#define FASTARDIFF_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum fard_status {
  FARD_OK = 0,
  FARD_EINVAL = -1,     /* null pointer, bad enum value, missing weight */
  FARD_ESHAPE = -2,     /* sizes the kernels do not support or that disagree with the config */
  FARD_ECAPACITY = -3,  /* batch, rows or context beyond what init reserved */
  FARD_ENOMEM = -4,
  FARD_EHIP = -5,       /* a HIP call failed; text in spec_last_error */
  FARD_ESTATE = -6
};

enum { FARD_F32 = 0, FARD_BF16 = 1 };
enum { FARD_ACT_GELU = 0, FARD_ACT_SWIGLU = 1 };
enum { FARD_NORM_LAYER = 0, FARD_NORM_RMS = 1 };
enum { FARD_POS_LEARNED = 0, FARD_POS_ROPE = 1 };
enum { FARD_ENT_FEATURE = 0, FARD_ENT_ATTN = 1 };
enum { FARD_TARGET = 0, FARD_DRAFT = 1 };

typedef struct fard_ctx fard_ctx; /* opaque */

/* Pre-norm causal transformer (the AR module z = ART(x_{1:i-1}, c) of Sec. 3.2). */
typedef struct {
  int32_t n_layers, d_model, n_heads, n_kv_heads, d_head, d_ff;
  int32_t act;        /* FARD_ACT_*: erf-GELU MLP or SwiGLU MLP */
  int32_t norm;       /* FARD_NORM_*: LayerNorm (gain+bias) or RMSNorm (gain) */
  int32_t pos;        /* FARD_POS_*: learned absolute table or RoPE (rotate-half pairing) */
  int32_t has_bias;   /* biases on the QKV / O / MLP projections */
  float norm_eps, rope_theta;
  int32_t d_latent;   /* D: width of a latent token */
  int32_t n_cond_ids; /* rows of the class/text id table, 0 = none */
  int32_t d_out;      /* feature width after the optional up-projection, 0 = d_model */
  int32_t max_pos;    /* rows of the learned position table */
} fard_tf_cfg;

/* Few-step diffusion/flow head x_0 = Diff(x_t | t, z) (Sec. 3.2, Sec. 4.2): AdaLN residual MLP. */
typedef struct {
  int32_t n_blocks, width, d_cond, d_latent, n_steps, t_freq_dim;
  float t_scale, sigma_last, temperature;
  int32_t renoise; /* 1: re-noise with the shared eps_k between steps, 0: Euler step */
} fard_head_cfg;

typedef struct {
  fard_tf_cfg target, draft;
  fard_head_cfg head;
  int32_t K;             /* draft length gamma (Alg. 1 input), <= 64 */
  int32_t max_batch;     /* B <= max_batch in every call */
  int32_t max_ctx;       /* cache capacity per sample in tokens */
  int32_t entropy_layer; /* l_s: 1-indexed draft layer whose output feeds the entropy indicator */
  int32_t entropy_mode;  /* FARD_ENT_FEATURE: softmax over the d channels of the layer output;
                            FARD_ENT_ATTN: attention rows of that layer, mean over heads (S2.1) */
  int32_t prefix_rule;   /* must be 1: a failed draft drops itself and every later draft (Alg. 1) */
  int32_t dtype;         /* FARD_F32 or FARD_BF16 */
  float tau_ent;         /* default threshold; calls take their own */
} fard_round_cfg;

/* One named weight.  Matrices are [d_in, d_out] row-major (y = x W + b).  Names:
 *   <m> in {target, draft}:
 *     <m>.in.w [D,d]  <m>.in.b [d]  <m>.pos [max_pos,d] (learned)  <m>.cond [n_cond_ids,d]
 *     <m>.L<i>.n1.g/.n1.b/.n2.g/.n2.b [d] (.b only for LayerNorm)
 *     <m>.L<i>.wqkv [d,(H+2Hkv)dh] columns = q heads | k heads | v heads,  .bqkv
 *     <m>.L<i>.wo [H dh,d] .bo ;  GELU: .w1 [d,F] .b1 .w2 [F,d] .b2 ;  SwiGLU: .wg .wu [d,F] .wd [F,d]
 *     <m>.nf.g/.nf.b [d]   <m>.up.w [d,d_out] (only if d_out != d_model)
 *   head.in.w [D,w] .in.b  head.c.w [d_cond,w] .c.b  head.t1.w [t_freq,w] .t1.b  head.t2.w [w,w] .t2.b
 *   head.B<j>.mod.w [w,3w] columns = shift | scale | gate, .mod.b ; .w1 [w,w] .b1 .w2 [w,w] .b2
 *   head.f.mod.w [w,2w] columns = shift | scale, .f.mod.b ; head.out.w [w,D] .out.b
 * Biases and gains that are absent default to 0 and 1. */
typedef struct {
  const char* name;
  const void* data;   /* host or device pointer */
  int64_t numel;
  int32_t dtype;      /* FARD_F32 or FARD_BF16 (element type of `data`) */
  int32_t on_device;  /* 0: host memory, 1: device memory */
} fard_tensor;

/* Alg. 1 inputs (models, gamma, T, temperature, tau_ent): builds the context.  Copies and re-lays
 * every weight (the caller may free its buffers on return), allocates both KV caches (zeroed,
 * lengths 0) and the workspace for max_batch * (K+1) rows.  hip_stream: a hipStream_t or NULL for
 * the default stream.  Synchronises. */
int spec_round_init(const fard_round_cfg* cfg, const fard_tensor* weights, int32_t n_weights,
                    void* hip_stream, fard_ctx** out);
int spec_round_destroy(fard_ctx* ctx);

/* Sets the cached length of every sample of model `which` (FARD_TARGET / FARD_DRAFT).
 * cache_len: HOST int32 [B] or NULL (all 0).  Does not touch cache contents. */
int spec_kv_reset(fard_ctx* ctx, int32_t which, const int32_t* cache_len, int32_t B);
/* The same from DEVICE memory, without a host synchronisation (a serving loop that rewinds or re-seats its samples
 * between rounds of Alg. 1): cache_len[b] = clamp(cache_len_dev[b], 0, len_hi) for b < B.  len_hi (host) is the
 * caller's upper bound of those lengths; capacity is checked against it from then on.  cache_len_dev: device int32 [B]. */
int spec_kv_restore(fard_ctx* ctx, int32_t which, const int32_t* cache_len_dev, int32_t B, int32_t len_hi);
/* Writes positions 0..n-1 of one layer's cache from plain tensors k, v [B, H_kv, n, d_head] in
 * storage type (synthetic caches).  Lengths are set with spec_kv_reset. */
int spec_kv_load(fard_ctx* ctx, int32_t which, int32_t layer, const void* k, const void* v,
                 int32_t B, int32_t n);
/* Copies the current lengths to HOST int32 [B].  Synchronises.  Also resets the host-side upper bound that the
 * capacity checks use (it grows by K + 1 per round whatever was accepted) to the true maximum over all samples. */
int spec_kv_lengths(fard_ctx* ctx, int32_t which, int32_t* out_host, int32_t B);
/* cache_len[b] = base_len[b] + 1 + n_accept[b] for both models: the pending token and the accepted
 * drafts become context (Alg. 1 Step 4).  n_accept: device int32 [B]. `which`: FARD_TARGET,
 * FARD_DRAFT, or -1 for both.  Uses the lengths recorded at the start of the last
 * spec_draft / spec_verify of that model. */
int spec_kv_commit(fard_ctx* ctx, int32_t which, const int32_t* n_accept, int32_t B);

/* KV-cached forward of one model over packed rows (Alg. 1 Step 2 for the target, Step 1 for the
 * draft; causal structure of Sec. 3.1).  Sample b owns n_q[b] consecutive rows; row j of a sample
 * sits at position cache_len[b] + j and attends to the cache and to rows 0..j.
 *   x_in     fp32 [M, D] latent rows         cond_id  int32 [M] or NULL; >= 0: the row is an id row
 *   n_q      device int32 [B], sum <= M      M <= max(max_batch*(K+1), min(max_batch*max_ctx, 8192)) workspace rows
 *   nq_max   host upper bound of n_q[b]; device values are clamped to it.  One attention workgroup holds
 *            64 / (H/H_kv) rows of a sample (bf16); more rows per sample are taken in passes inside every layer.
 *            Capacity (cache_len + nq_max <= max_ctx) is checked against it on the host.
 *   commit   1: cache_len[b] += n_q[b]
 *   z_out    storage type [M, d_out]         shallow_out  fp32 [M, d] residual stream after layer
 *   h_attn_out fp32 [M] head-mean attention-row entropy of layer entropy_layer (either may be NULL) */
int spec_forward(fard_ctx* ctx, int32_t which, const float* x_in, const int32_t* cond_id,
                 const int32_t* n_q, int32_t nq_max, int32_t B, int32_t M, int32_t commit, void* z_out,
                 float* shallow_out, float* h_attn_out);

/* Prefill: builds the KV cache of one model from a prefix of known tokens instead of loading it (the prefix that
 * Alg. 1 starts from; causal structure of Sec. 3.1).  Sample b's rows x[b, 0 .. n[b]-1, :] are appended at
 * positions cache_len[b] .. cache_len[b] + n[b] - 1; row j attends to the cache and to rows 0..j.  Whole prefixes go
 * through the layers at once while B of them fit into the workspace (8192 rows), else in passes of workspace / B rows
 * per sample; inside a layer the attention takes 64 / (n_heads / n_kv_heads) rows of a sample at a time (what one
 * attention workgroup holds).  The result is that of one causal forward over all rows.
 *   x        device fp32 [B, n_max, D] latent rows (rows at or beyond n[b] are not read)
 *   first_id device int32 [B] or NULL: >= 0 makes row 0 of the prefix an id row (class token); needs an id table
 *   n        HOST int32 [B], 0 <= n[b] <= n_max (copied before return)
 *   z_last   storage type [B, d_out] or NULL: the feature of each sample's last prefix row (what the head decodes
 *            into the first token); rows of samples with n[b] = 0 are left untouched
 * Errors: FARD_ECAPACITY if cache_len + max n exceeds max_ctx or the learned position table; FARD_EINVAL for
 * n[b] outside [0, n_max].  Synchronises once at the start (for the copy of n). */
int spec_prefill(fard_ctx* ctx, int32_t which, const float* x, const int32_t* first_id, const int32_t* n,
                 int32_t n_max, int32_t B, void* z_last);

/* Shallow-layer entropy indicator + pre-filter (abstract; Eq. 1; Sec. 4.3; Alg. 1 Step 1):
 * H[b,i] = -sum_c p_c ln p_c, p = softmax(feat[b,i,:]); keep[b,i] = all_{j<=i}(H[b,j] >= tau);
 * n_keep[b] = sum_i keep; surv_idx = ascending flat indices b*K+i of kept drafts; n_surv = count.
 *   feat storage type [B, K, L]; H fp32 [B,K]; keep uint8 [B,K]; n_keep int32 [B];
 *   surv_idx int32 [B*K] (first n_surv valid); n_surv int32 [1].  B*K = 0 gives n_surv = 0. */
int entropy_prefilter(fard_ctx* ctx, const void* feat, int32_t B, int32_t K, int32_t L, float tau,
                      float* H, uint8_t* keep, int32_t* n_keep, int32_t* surv_idx, int32_t* n_surv);
/* entropy_prefilter for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): needs no context and calls no allocating routine.  Same operation, same
 * kernels and the same outputs as entropy_prefilter; the per-workgroup survivor counts that the large-batch path
 * (B > 1024) passes from its first launch to its second live in an 8 KiB device array inside the library, one copy
 * per GPU, held until the process ends.
 *   dtype       FARD_F32 / FARD_BF16: element type of feat
 *   hip_stream  hipStream_t to enqueue on (NULL: default stream) on the CURRENT device; does not synchronise
 * Limits: B <= 2^21 samples and B * K <= 2^24 rows, else FARD_ECAPACITY.  All calls on one GPU share that array: calls
 * that overlap on one GPU (different streams, different threads) race; calls in stream order do not (nothing in the
 * array has to survive between calls or start at zero).  Errors are returned as codes only (no context, no text). */
int entropy_prefilter_static(const void* feat, int32_t dtype, int32_t B, int32_t K, int32_t L, float tau, float* H,
                             uint8_t* keep, int32_t* n_keep, int32_t* surv_idx, int32_t* n_surv, void* hip_stream);
/* tau = 0.3 * mean_H - 0.1 * std_H (Sec. 4.3). Host-only helper. */
float entropy_threshold(float mean_H, float std_H);

/* Few-step head on n rows (Sec. 3.2 head, Sec. 4.2 few steps): S = n_steps sampler steps from
 * x_{t_0} = temperature * eps[0]; mu = last x_0 estimate; x = mu + sigma_last * temperature * eps[S].
 *   z storage type [n_max, d_cond]; n_rows device int32 [1] or NULL (= n_max): rows >= *n_rows are
 *   skipped (so a survivor count can be passed without a host round trip);
 *   eps fp32 [S+1, n_max, D]; mu, x fp32 [n_max, D]. */
int diffhead_decode(fard_ctx* ctx, const void* z, const int32_t* n_rows, int32_t n_max,
                    const float* eps, float* mu, float* x);

/* Alg. 1 Step 1 for a batch: K sequential draft steps with the entropy early stop.
 *   x_pending fp32 [B, D]; pending_id int32 [B] or NULL (>= 0: the pending token is an id row);
 *   eps fp32 [S+1, B, K+1, D]; tau: threshold for this call.
 * Outputs: H fp32 [B,K] (0 after a sample stopped); keep uint8 [B,K]; n_keep int32 [B];
 *   x_draft, mu_q fp32 [B, K, D] (rows of dropped drafts are left untouched).
 * The draft cache advances by one token per executed step; spec_kv_commit rolls it back. */
int spec_draft(fard_ctx* ctx, const float* x_pending, const int32_t* pending_id, const float* eps,
               float tau, int32_t B, float* H, uint8_t* keep, int32_t* n_keep, float* x_draft,
               float* mu_q);

/* Alg. 1 Step 1, one draft step per call (a serving loop that interleaves other work, or that supplies the token
 * a step reads): step i = 0 starts a draft stage like spec_draft does, steps must follow in order, and after the last
 * one the state is that of spec_draft (spec_verify / spec_kv_commit as usual).  Same kernels and launches as spec_draft.
 *   x_prev fp32 [B, D]: the token step i reads (token i-1; the pending token for i = 0), or NULL for i > 0: the
 *   library's own draft x_draft[:, i-1, :].  prev_id int32 [B] or NULL (>= 0: that token is an id row).
 *   The other arguments are those of spec_draft; a step writes column i of H / keep and row i of x_draft / mu_q.
 * Errors: FARD_ESTATE for steps out of order, FARD_EINVAL for i outside [0, K) or a NULL x_prev at i = 0. */
int spec_draft_step(fard_ctx* ctx, int32_t i, const float* x_prev, const int32_t* prev_id, const float* eps,
                    float tau, int32_t B, float* H, uint8_t* keep, int32_t* n_keep, float* x_draft, float* mu_q);

/* Alg. 1 Steps 2-4: target forward over [pending, x_1..x_K'] per sample (K' = n_keep[b]), head on
 * all K'+1 rows with the shared noise, ratio and accept test.
 *   log_sigma_factor = ln Sigma of S3 item 2; sigma_p, sigma_q: std of the last transition.
 *   ln rho[b,i] = ln Sigma + D ln(sigma_q/sigma_p) - |x_i - mu_p,i|^2/(2 sigma_p^2) + |x_i - mu_q,i|^2/(2 sigma_q^2)
 *   acc[b,i] = (ln r[b,i] <= ln rho[b,i]); n_accept[b] = leading run of acc within the first K'.
 * Outputs: n_accept int32 [B]; log_ratio fp32 [B,K]; mu_p fp32 [B,K+1,D] (row K' is the bonus
 *   distribution's mean; rows beyond are zero); z_p storage type [B,K+1,d_out] or NULL.
 * The target cache is written for all K'+1 rows; lengths change only in spec_kv_commit. */
int spec_verify(fard_ctx* ctx, const float* x_pending, const int32_t* pending_id,
                const float* x_draft, const float* mu_q, const int32_t* n_keep, const float* r,
                const float* eps, float log_sigma_factor, float sigma_p, float sigma_q, int32_t B,
                int32_t* n_accept, float* log_ratio, float* mu_p, void* z_p);

/* The accept test alone (Alg. 1 Steps 3-4) on caller-provided means.  acc uint8 [B,K]. */
int spec_accept(fard_ctx* ctx, const float* x_draft, const float* mu_p, const float* mu_q,
                const float* r, const int32_t* n_keep, float log_sigma_factor, float sigma_p,
                float sigma_q, int32_t B, int32_t* n_accept, float* log_ratio, uint8_t* acc);

/* spec_draft + spec_verify + spec_kv_commit(both) in one call (one round of Alg. 1, Steps 1-4). */
int spec_round(fard_ctx* ctx, const float* x_pending, const int32_t* pending_id, const float* eps,
               const float* r, float tau, float log_sigma_factor, float sigma_p, float sigma_q,
               int32_t B, float* H, uint8_t* keep, int32_t* n_keep, float* x_draft, float* mu_q,
               int32_t* n_accept, float* log_ratio, float* mu_p);

/* Launch-bound rounds as one HIP graph (a round of Alg. 1 at a few tens of samples is several hundred short
 * dependent kernels).  enable = 1: spec_round called with exactly the arguments of the call before it
 * (same pointers, scalars and B) records its launches into a graph on the second such call and replays that
 * graph on every later one; a call with other arguments launches kernel by kernel again and starts over.
 * Replays read the cache lengths on the device, so spec_kv_reset / spec_kv_load between calls are fine; the
 * host-side capacity rules (FARD_ECAPACITY) are checked on every call as usual.  The buffers the arguments
 * name must stay allocated while the graph is in use; their contents may change freely.
 * spec_generate uses the same switch: the noise of each round is first copied to staging buffers inside the context
 * (one small launch), so every round is the same set of launches; the first round of a new argument set (tokens,
 * n_tokens, the scalars, B, R, J <= 64) is launched kernel by kernel, the second is recorded, all later rounds, also
 * of later calls with the same arguments, are replays; the per-round records are copied out after each round.
 * enable = 0 drops the graphs.  Per-kernel timing (spec_profile_enable) switches replay off while it is on.
 * Errors: FARD_ESTATE if the context runs on the default stream (it cannot be captured). */
int spec_graph_enable(fard_ctx* ctx, int32_t enable);

/* Alg. 1 Step 5 (S3 item 3) and the token a round ends with, for every sample (device memory throughout):
 *   n_accept[b] < n_keep[b]: draft n_accept[b]+1 was rejected; the token is drawn from the residual
 *     max(0, Sigma p - q) by acceptance-rejection: proposal j = mu_p[b, n] + sigma_p * eps_res[b, j, :] is taken
 *     when u_res[b, j] <= max(0, 1 - q(x_j) / (Sigma p(x_j))); J proposals at most, the last one is taken
 *     if none passes (tries[b] = J);
 *   otherwise: the target's own sample of row n_keep[b] under the shared noise,
 *     mu_p[b, n_keep] + sigma_p * eps[S, b, n_keep, :] (tries[b] = 0).
 *   mu_p fp32 [B,K+1,D], mu_q fp32 [B,K,D], eps fp32 [S+1,B,K+1,D] (the round's shared noise), eps_res fp32
 *   [B,J,D], u_res fp32 [B,J]; x_next fp32 [B,D], tries int32 [B]. */
int spec_resample(fard_ctx* ctx, const float* mu_p, const float* mu_q, const float* eps,
                  const int32_t* n_accept, const int32_t* n_keep, const float* eps_res, const float* u_res,
                  float log_sigma_factor, float sigma_p, float sigma_q, int32_t B, int32_t J, float* x_next,
                  int32_t* tries);

/* R rounds of Alg. 1 in a row (Steps 1-5) without a host synchronisation: spec_round, spec_resample, cache
 * commit, and one single-row draft forward for the samples that accepted all K drafts (their draft model has
 * not read draft K yet); the closing token of a round is the pending token of the next.
 *   x_first fp32 [B,D] / first_id int32 [B] or NULL: the pending row of the first round (as in spec_draft)
 *   eps fp32 [R][S+1,B,K+1,D], r fp32 [R][B,K], eps_res fp32 [R][B,J,D], u_res fp32 [R][B,J]: pre-drawn
 *   tokens fp32 [B, R*(K+1), D]: per sample the accepted drafts and the closing token of every round, in
 *     order; n_tokens int32 [B] their count.  H fp32 [R,B,K], n_keep, n_accept, tries int32 [R,B]: per round.
 * All samples stay active for all R rounds.  Errors: FARD_ECAPACITY unless cache_len + R*(K+1) <= max_ctx
 * (and the learned position table) for both models: the host tracks only upper bounds of the lengths. */
int spec_generate(fard_ctx* ctx, const float* x_first, const int32_t* first_id, const float* eps,
                  const float* r, const float* eps_res, const float* u_res, float tau, float log_sigma_factor,
                  float sigma_p, float sigma_q, int32_t B, int32_t R, int32_t J, float* tokens,
                  int32_t* n_tokens, float* H, int32_t* n_keep, int32_t* n_accept, int32_t* tries);

/* out = act(A W + b) through the library's GEMM kernel, for tests and kernel timing.
 *   A storage type [M,K]; W storage type [K,N] row-major (re-laid on every call); bias fp32 [N] or
 *   NULL; act: 0 none, 1 erf-GELU, 2 SiLU; out storage type [M,N].  bf16: K % 64 == 0, N % 32 == 0. */
int spec_gemm(fard_ctx* ctx, const void* A, const void* W, const float* bias, int32_t M, int32_t K,
              int32_t N, int32_t act, void* out);

/* One small-batch GEMM through the narrow-tile kernel (bf16 contexts), for tests and kernel timing: the
 * draft steps and head decodes of a round (Alg. 1 Steps 1-2) run their GEMMs through it.  All pointers
 * are device memory.  A storage type [M,K]; W storage type [K,N] row-major (re-laid on every call);
 * bias fp32 [N] or NULL; M <= 1024, K % 64 == 0, N % 32 == 0.
 *   epi 0  out storage type [M,N] = act(A W + bias);   1: the same, out fp32
 *   epi 2  out fp32 [M,N] += A W + bias;   3: out fp32 [M,N] += gate[m,n] * (A W + bias), gate fp32 [M,N]
 *   out_bf16 (epi 2, 3 only; or NULL): the updated out is also stored as bf16 [M,N] there.
 * K is never split: no atomics, results are deterministic.
 * Errors: FARD_ESHAPE for sizes outside the limits above, FARD_EINVAL for bad selectors or NULLs. */
int spec_gemm_narrow(fard_ctx* ctx, const void* A, const void* W, const float* bias, const float* gate,
                     int32_t M, int32_t K, int32_t N, int32_t epi, int32_t act, void* out, void* out_bf16);

/* The norm of Sec. 3.1's transformer blocks folded into the GEMM that follows it (how the round runs the second norm
 * of a block without a launch of its own): out = act(norm(x) W + bias), norm(x)_k = g_k (x_k - mean) rstd + beta_k
 * (LayerNorm, norm_type 0; beta NULL = 0) or g_k x_k rstd (RMSNorm, norm_type 1), statistics over the K entries of a
 * row.  Computed as rstd (x W' - mean colsum(W')) + (bias + beta W) with W' = diag(g) W rounded to bf16: the row
 * statistics are summed from the bf16 activation fragments on their way into the matrix cores.
 *   x bf16 [M, K] (the raw rows); W bf16 [K, N] row-major; g, beta fp32 [K]; bias fp32 [N] or NULL; out bf16 [M, N].
 *   M <= 1024, K % 64 == 0, N % 32 == 0; act 0 none, 1 GELU, 2 SiLU.  bf16 contexts only. */
int spec_gemm_norm(fard_ctx* ctx, const void* x, const void* W, const float* g, const float* beta,
                   const float* bias, int32_t M, int32_t K, int32_t N, int32_t norm_type, float eps, int32_t act,
                   void* out);

/* Training side of the draft model (Sec. 3, "Add feature-level entropy loss"; S2.1): the attention-entropy loss
 *   L_entropy = (1 / (B N R)) sum_{b, heads, rows r, columns c} Omega_{r,c} ln Omega_{r,c}      (<= 0)
 * of the causal attention maps Omega = softmax(q k^T / sqrt(d_head)) (row r sees columns 0..r; query head h reads kv
 * head h / (H / H_kv)), and its gradients with respect to q and k.  Nothing of size R x R is written to memory.
 *   q   storage type [B, H, R, d_head]        k   storage type [B, H_kv, R, d_head]   (bf16 contexts only; 16-byte aligned)
 *   loss fp32 [1]      h_rows fp32 [B, H, R] row entropies H_r = -sum_c Omega ln Omega, or NULL
 *   dq  fp32 like q, or NULL                  dk  fp32 like k, or NULL   (written, not accumulated)
 * d_head in {32, 64, 128}.  Scratch grows inside the context (hipMalloc on first use or growth: not for capture).
 * Errors: FARD_ESTATE in an fp32 context, FARD_ESHAPE for unsupported sizes, FARD_ENOMEM. */
int spec_entropy_loss(fard_ctx* ctx, const void* q, const void* k, int32_t B, int32_t H, int32_t H_kv, int32_t R,
                      int32_t d_head, float* loss, float* h_rows, float* dq, float* dk);

/* The feature regression loss that the method keeps from EAGLE (Sec. 2, L_reg; Sec. 3 "Retain feature-level
 * regression loss"): mean over n elements of 0.5 d^2 / beta (|d| < beta) or |d| - 0.5 beta, d = pred - target.
 *   pred, target storage type [n]; loss fp32 [1]; dpred fp32 [n] = dloss/dpred, or NULL.  beta > 0. */
int spec_smooth_l1(fard_ctx* ctx, const void* pred, const void* target, int64_t n, float beta, float* loss,
                   float* dpred);

/* Peak probes for the roofline of Sec. 3's round (no operation of the method; measurement only): what this GPU
 * sustains on the two resources the kernels are priced against, timed with HIP events on the context's stream.
 *   kind 0: streaming read of buf (device, 16-byte aligned, bytes a positive multiple of 16; read only), 16 B per
 *           lane per load over 2048 workgroups; units_per_launch = bytes.
 *   kind 1: register-only loop of bf16 32x32x16 MFMAs, 4 * iters per wave over 2048 workgroups of four waves;
 *           units_per_launch = flop.  buf and bytes are ignored.
 * One warm-up launch, then reps timed launches; *ms_per_launch (host) is their average, *units_per_launch (host)
 * the bytes or flop of one launch.  Blocks the host until done; allocates a few KB inside the context on first
 * use (not for capture). */
int spec_peak_probe(fard_ctx* ctx, int32_t kind, const void* buf, int64_t bytes, int32_t iters, int32_t reps,
                    float* ms_per_launch, double* units_per_launch);

/* Per-kernel timing with HIP events on the context's stream.  enable = 1 brackets every launch of
 * the named kernel class between two events; spec_profile_read synchronises and returns the
 * accumulated time (ms) and launch count since enable, then clears them.
 * class: 0 GEMMs of the streaming kernels (every GEMM above a few hundred rows, the weight stream of the 72-row verify
 * stage), 1 attention, 2 entropy, 3 everything else, 4 GEMMs of the narrow-tile kernel (draft steps, head decodes). */
int spec_profile_enable(fard_ctx* ctx, int32_t enable);
int spec_profile_read(fard_ctx* ctx, int32_t kernel_class, float* total_ms, int64_t* launches,
                      double* flops, double* bytes);

const char* spec_last_error(const fard_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* FASTARDIFF_H */

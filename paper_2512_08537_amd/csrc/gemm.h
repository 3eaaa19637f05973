// Host-side interface of the GEMM kernels (bf16 MFMA path and fp32 path).
#pragma once
#include "common.h"

namespace fard {

// What the epilogue does with acc[m, n] = sum_k A[m, k] W[k, n].
enum Epi {
  EPI_STORE = 0,       // out_T[m, n]   = act(acc + bias[n])                (activation storage type)
  EPI_STORE_F32 = 1,   // out_f32[m, n] = act(acc + bias[n])
  EPI_RESID = 2,       // out_f32[m, n] += acc + bias[n]                    (residual stream update)
  EPI_GATE_RESID = 3,  // out_f32[m, n] += gate[m, n] * (acc + bias[n])
  EPI_SWIGLU = 4,      // out_T[m, j]   = silu(acc[m, gate col j]) * acc[m, up col j]  (interleaved columns)
  EPI_PARTIAL = 5,     // out_f32[z][m, n] = partial sum of K slice z (+ bias[n] in slice 0); narrow kernel, or the streaming
                       // kernel through launch_gemm_bf16_planes:
                       // the consumer (the next norm) adds the k_slices planes to the residual stream
};

struct GemmArgs {
  const void* A;       // [M, K] row-major, leading dimension lda (elements); bf16 or fp32 per path
  int lda;
  const void* W;       // bf16 path: fragment-packed weights; fp32 path: [K, N] row-major
  const float* bias;   // [N] or nullptr
  void* out;
  int ldo;
  const float* gate;   // [M, ldg] fp32, EPI_GATE_RESID only
  int ldg;
  int M, N, K;         // N counts weight columns (2F for EPI_SWIGLU)
  const int* m_dev;    // optional device-side row count (rows >= *m_dev are skipped)
  int act;
  int epi;
  int k_slices = 1;    // EPI_PARTIAL: K slices (blockIdx.z), plane z at out + z * part_stride
  size_t part_stride = 0;
  // narrow kernel only:
  void* copy_bf16 = nullptr;       // EPI_RESID / EPI_GATE_RESID: the updated values are also stored as bf16 [M, ldo] here
  const float* ln_cs = nullptr;    // non-null: A holds the raw rows x and W = diag(g) W0; the epilogue applies the norm
                                   // of the rows, rstd_r (acc - mean_r ln_cs[n]) + bias[n], with ln_cs[n] = sum_k W[k, n]
                                   // and bias = b0 + beta W0 folded by the caller; statistics come from the A fragments
  float ln_eps = 0.f;
  int ln_rms = 0;                  // 1: RMS norm (no mean)
  // A modulated LayerNorm between two GEMMs without a launch of its own (the head's AdaLN blocks, Sec. 3.2):
  // the GEMM that updates the rows h (EPI_RESID / EPI_GATE_RESID) also writes v = bf16(h (1 + copy_scale)) to
  // copy_bf16 and, per row and 16-column tile, the tile's mean and centred sum of squares to mom_out;
  const float* copy_scale = nullptr;   // [M, copy_ld] fp32: scale of the norm that follows
  int copy_ld = 0;
  float* mom_out = nullptr;            // [M][mom_ld >= N / 16] pairs (mean, sum of squares about it), a row's tiles side by side
  int mom_ld = 0;
  // the next GEMM multiplies v and finishes, with the rows' mean_r and rstd_r merged from the tile moments,
  //   out[r, n] = act(rstd_r (acc[r, n] - mean_r c1[r, n]) + c0[r, n] + bias[n]),
  // c1[r, :] = (1 + scale_r) W and c0[r, :] = shift_r W supplied by the caller:
  //   LN(h)(1 + scale) + shift times W, with the row-wise factors taken out of the sum over k.
  const float* ada_mom = nullptr;      // [M][ada_mom_ld >= K / 16] pairs, as written through mom_out
  int ada_mom_ld = 0;
  const float* ada_c1 = nullptr;       // [M, ada_ld] fp32
  const float* ada_c0 = nullptr;
  int ada_ld = 0;
  float ada_eps = 0.f;
  // Tile order for bf16 activations that pass from one narrow-kernel GEMM to the next (a_tiled: the A operand;
  // out_tiled: what EPI_STORE stores and copy_bf16 receives): element (r, k) of a [rows, K] matrix at
  //   ((((r / 16) (K / 32) + k / 32) 4 + k / 8 % 4) 16 + r % 16) 8 + k % 8,
  // i.e. the 16-byte pieces a lane of the 16 x 16 x 32 MFMA reads, rows innermost, so that a wave's operand load
  // reads 1 KiB of consecutive memory (lanes whose pieces lie a row apart are served one by one: measured 0.4 us of
  // a 3.9 us launch at 8-16 rows, 0.8 us at 32).  Whole 16-row tiles must be allocated.
  int a_tiled = 0, out_tiled = 0;
};

// Packed bf16 weight size in elements for a [K, N] matrix (K % 16 == 0, N % 32 == 0).
inline size_t packed_elems(int K, int N) { return (size_t)K * (size_t)N; }

// Returns hipSuccess or the launch error.  K % 64 == 0 and N % 32 == 0 are required (bf16 path).
hipError_t launch_gemm_bf16(hipStream_t s, const GemmArgs& a);
hipError_t launch_gemm_f32(hipStream_t s, const GemmArgs& a);

// K split over workgroups of the streaming kernel, every split writing its partial sums to its own fp32 plane
// (a.epi == EPI_PARTIAL, plane z at out + z * part_stride, bias in plane 0; no atomics): for GEMMs of up to 128 rows
// against tens of MB of weights, where the column tiles alone are too few workgroups to stream the weights and wider
// tiles are needed so that the activation panel is not re-read once per 32 columns.  a.k_slices must be
// gemm_plane_count(K, wanted): the number of planes actually written for a wanted split count.
int gemm_plane_count(int K, int splits);
hipError_t launch_gemm_bf16_planes(hipStream_t s, const GemmArgs& a);

// Narrow-tile GEMM: one workgroup per 16 columns and 16-64 rows, no K split (no atomics; EPI_RESID and
// EPI_GATE_RESID read-modify-write their tile), bf16 A.  Meant for M <= 64, or a few hundred rows when K
// and N are about 1024.
bool narrow_supported(const GemmArgs& a);
hipError_t launch_gemm_narrow(hipStream_t s, const GemmArgs& a);

// Re-lay a row-major [K, N] matrix (src_is_bf16: bf16 else fp32; leading dimension ld) into MFMA
// fragment order.  Destination n-block index = nb_offset + nb * nb_stride (lets two matrices be
// interleaved block by block for the SwiGLU epilogue).
hipError_t launch_pack_weight(hipStream_t s, const void* src, int src_is_bf16, int ld, int K, int N,
                              void* dst, int nb_offset, int nb_stride);

}  // namespace fard

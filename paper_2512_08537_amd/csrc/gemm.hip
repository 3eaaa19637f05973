// GEMM kernels: out = epilogue(A[M,K] * W[K,N]).
//
// bf16 path (gfx950 MFMA).  The GEMMs of a speculative round are skinny (M = a few hundred rows at
// most) and small (2-50 MB of weights each), so one launch lives or dies by how many weight bytes
// it keeps in flight, not by MFMA issue rate.  Design:
//  * weights are pre-laid in v_mfma_f32_32x32x16_bf16 B-fragment order, so every wave streams them
//    from HBM straight into registers as fully contiguous 1 KiB loads, through a register ring that
//    keeps P k-steps (8-16 KiB per wave) in flight; they never touch LDS;
//  * the activation panel of a workgroup (BM rows x KC = 256 k) is staged in LDS once per chunk and
//    shared by the 4 waves, each of which owns its own 32*WN output columns; the next chunk is
//    prefetched into registers while the current one is consumed, so the inner loop has no barrier;
//  * K is split across workgroups when the tile grid alone cannot cover the chip (residual-stream
//    epilogues add their partial sums with fp32 atomics);
//  * workgroups are numbered so that all M-tiles of one weight panel land on the same XCD (ids are
//    dealt to the 8 XCDs round-robin): the panel is fetched from HBM once per L2.
//
// fp32 path: a plain LDS-tiled FMA kernel, used by the small all-fp32 configuration.
#include "gemm.h"

namespace fard {

namespace {

// KC: k per staged activation chunk (template parameter, 256 or 512).  LDS rows are KC + 8 bf16 long
// (528 / 1040 B): the 16-byte reads of 32 consecutive rows spread over all banks.

// Register e of a 32x32 accumulator holds row 8*(e/4) + 4*(lane/32) + e%4, column lane%32.

// Direct epilogue: every wave stores its own accumulator blocks, no barrier.  For tiles of many-row products, where a
// compute unit runs workgroup after workgroup and the waves' stores overlap the next tiles' MFMAs.
template <int KIND, bool FULL, int WM, int WN>
__device__ __forceinline__ void epilogue(const GemmArgs& a, f32x16 (&acc)[WM][WN], int m0, int M, int nb0, int nblocks,
                                         int cl, int rhalf, bool add_bias, bool atomic, int sp) {
  if constexpr (KIND == EPI_SWIGLU) {
    if constexpr (WN == 2) {
      if (nb0 + 1 >= nblocks) return;
      const int col = (nb0 >> 1) * 32 + cl;
      bf16* out = (bf16*)a.out;
#pragma unroll
      for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int row = m0 + 32 * i + 8 * (e >> 2) + rhalf + (e & 3);
          if (FULL || row < M) out[(size_t)row * a.ldo + col] = (bf16)(silu(acc[i][0][e]) * acc[i][1][e]);
        }
    }
    return;
  } else {
#pragma unroll
    for (int j = 0; j < WN; ++j) {
      if (nb0 + j >= nblocks) continue;
      const int col = (nb0 + j) * 32 + cl;
      const float bv = (a.bias != nullptr && add_bias) ? a.bias[col] : 0.f;
#pragma unroll
      for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int row = m0 + 32 * i + 8 * (e >> 2) + rhalf + (e & 3);
          if (!FULL && row >= M) continue;
          float v = acc[i][j][e] + bv;
          const size_t o = (size_t)row * a.ldo + col;
          if constexpr (KIND == EPI_STORE) {
            ((bf16*)a.out)[o] = (bf16)apply_act(v, a.act);
          } else if constexpr (KIND == EPI_STORE_F32) {
            ((float*)a.out)[o] = apply_act(v, a.act);
          } else if constexpr (KIND == EPI_PARTIAL) {
            ((float*)a.out)[(size_t)sp * a.part_stride + o] = v;   // the K split's own plane: no atomics
          } else {
            if constexpr (KIND == EPI_GATE_RESID) v *= a.gate[(size_t)row * a.ldg + col];
            float* dst = (float*)a.out + o;
            if (atomic) atomicAdd(dst, v);       // partial sums of a split K range meet in memory
            else *dst += v;
          }
        }
    }
  }
}

// Staged epilogue, for products of one row tile (M <= 128), whose launch is one workgroup per compute unit.
// The tile leaves through LDS, 32 rows at a time: the waves that hold the sums write
// their accumulator block, then all 256 threads read it back row-contiguous and store 16 bytes per lane (whole cache
// lines), in a loop of a few dozen instructions.  The direct epilogue, unrolled over the 16 WM WN accumulator registers, with
// its row and kind tests per element, runs to several thousand instructions per kernel; here every workgroup executes
// it once, cold, and its instruction fetches queue behind the weight stream (measured at 72 rows: 4.3 us of a
// 16 us launch between the last MFMA and the last store).  lds: 32 x (BN + 4) floats.
template <int WM, int WN, int NWN>
__device__ __forceinline__ void staged_epilogue(const GemmArgs& a, f32x16 (&acc)[WM][WN], float* lds, int m0, int M,
                                                int n0, bool holds_sums, int nw, bool add_bias, bool atomic, int sp) {
  constexpr int BNW = 32 * WN, BN = BNW * NWN, LDT = BN + 4;
  constexpr int GPR = BN / 4;                              // groups of 4 columns per row
  constexpr int RSTEP = 256 / GPR;                         // rows covered by one pass of the 256 threads
  static_assert(256 % GPR == 0 && 32 % RSTEP == 0, "a thread keeps its column group over all rows");
  const int lane = threadIdx.x & 63;
  const int col = (threadIdx.x % GPR) * 4, r0 = threadIdx.x / GPR;
  const int gc = n0 + col;
  const int N = a.N, epi = a.epi;
  f32x4 bias4 = {0.f, 0.f, 0.f, 0.f};
  if (epi != EPI_SWIGLU && a.bias != nullptr && add_bias && gc < N) bias4 = *(const f32x4*)(a.bias + gc);
#pragma unroll
  for (int i = 0; i < WM; ++i) {
    const int mb = m0 + 32 * i;
    if (mb >= M) break;                                    // uniform over the workgroup
    __syncthreads();                                       // the staging area is free
    if (holds_sums) {
#pragma unroll
      for (int j = 0; j < WN; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e)
          lds[(8 * (e >> 2) + 4 * (lane >> 5) + (e & 3)) * LDT + nw * BNW + 32 * j + (lane & 31)] = acc[i][j][e];
    }
    __syncthreads();
    if (epi == EPI_SWIGLU) {
      // packed column blocks alternate gate / up (32 columns each): output column = packed / 2
      constexpr int OGPR = BN / 8;                         // groups of 4 output columns per row
      bf16* out = (bf16*)a.out;
      for (int idx = threadIdx.x; idx < 32 * OGPR; idx += 256) {
        const int row = idx / OGPR, oc = (idx - row * OGPR) * 4;
        const int pc = (oc >> 5) * 64 + (oc & 31);         // packed column of the gate value
        const int gr = mb + row;
        if (gr >= M || n0 + pc + 32 >= N) continue;        // gate and up blocks both inside N
        const f32x4 g = *(const f32x4*)(&lds[row * LDT + pc]), u = *(const f32x4*)(&lds[row * LDT + pc + 32]);
        bf16x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = (bf16)(silu(g[e]) * u[e]);
        *(bf16x4*)(out + (size_t)gr * a.ldo + (n0 >> 1) + oc) = o;
      }
      continue;
    }
    if (atomic) {
      // partial sums of a split K range meet in memory: one column per lane, so that an atomic instruction of a wave
      // covers whole 128-byte segments
      for (int idx = threadIdx.x; idx < 32 * BN; idx += 256) {
        const int row = idx / BN, c = idx - row * BN;
        const int gr = mb + row, gn = n0 + c;
        if (gr >= M || gn >= N) continue;
        float v = lds[row * LDT + c];
        if (a.bias != nullptr && add_bias) v += a.bias[gn];
        if (epi == EPI_GATE_RESID) v *= a.gate[(size_t)gr * a.ldg + gn];
        atomicAdd((float*)a.out + (size_t)gr * a.ldo + gn, v);
      }
      continue;
    }
    if (gc >= N) continue;                                 // N % 32 == 0: a group is all in or all out
    for (int row = r0; row < 32; row += RSTEP) {
      const int gr = mb + row;
      if (gr >= M) break;
      f32x4 v = *(const f32x4*)(&lds[row * LDT + col]) + bias4;
      const size_t o = (size_t)gr * a.ldo + gc;
      if (epi == EPI_STORE) {
        bf16x4 t;
#pragma unroll
        for (int e = 0; e < 4; ++e) t[e] = (bf16)apply_act(v[e], a.act);
        *(bf16x4*)((bf16*)a.out + o) = t;
      } else if (epi == EPI_STORE_F32) {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = apply_act(v[e], a.act);
        *(f32x4*)((float*)a.out + o) = v;
      } else if (epi == EPI_PARTIAL) {
        *(f32x4*)((float*)a.out + (size_t)sp * a.part_stride + o) = v;   // the K split's own plane: no atomics
      } else {
        if (epi == EPI_GATE_RESID) v *= *(const f32x4*)(a.gate + (size_t)gr * a.ldg + gc);
        float* dst = (float*)a.out + o;
        *(f32x4*)dst = *(const f32x4*)dst + v;
      }
    }
  }
}

// WM x WN: 32x32 accumulator blocks per wave.  KW: waves of the workgroup that share the same output
// columns and split every chunk's 16 k-steps between them (their partial sums meet in LDS at the end);
// the other 4/KW waves sit side by side along N.  P: ring depth in k-steps of one wave.
template <int WM, int WN, int KW, int P, int KC, bool STAGED>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmArgs a, int n_tiles, int m_tiles, int splits,
                                                        int chunks_per_split, int xm) {
  constexpr int KSTEPS = KC / 16;                          // MFMA k-steps per chunk
  constexpr int LDS_STRIDE = KC + 8;
  constexpr int RPP = KC / 8;                              // 16-byte pieces per row of a chunk
  constexpr int NWN = 4 / KW;                              // waves along N
  constexpr int SPW = KSTEPS / KW;                         // k-steps per wave per chunk
  constexpr int G = (P > SPW) ? P : SPW;                   // k-steps per unrolled group (both powers of two)
  constexpr int BM = 32 * WM;
  constexpr int PIECES = BM * (KC / 8);                    // 16-byte pieces in one A chunk
  constexpr int PPT = PIECES / 256;                        // pieces per thread (BM multiple of 32 -> exact)
  constexpr int RED_FLOATS = (KW > 1) ? NWN * WM * WN * 16 * 64 : 0;
  constexpr int STAGE_BYTES = STAGED ? 32 * (32 * WN * NWN + 4) * 4 : 0;   // one 32-row block of the tile on its way out
  constexpr int LDS_AR = (BM * LDS_STRIDE * 2 > RED_FLOATS * 4) ? BM * LDS_STRIDE * 2 : RED_FLOATS * 4;
  constexpr int LDS_BYTES = LDS_AR > STAGE_BYTES ? LDS_AR : STAGE_BYTES;
  static_assert(G % P == 0 && G % SPW == 0, "ring depth and steps per wave must be powers of two");
  extern __shared__ __attribute__((aligned(16))) char lds_raw[];   // LDS_BYTES, passed at launch
  bf16* lds = (bf16*)lds_raw;
  (void)LDS_BYTES;

  // blockIdx -> (weight panel, m tile): workgroup id % 8 is the XCD; the XCDs form xm groups along M times 8 / xm
  // groups along the panels, a group's panels are dealt round-robin, and the m tiles of a panel are consecutive
  // slots of its XCD.
  const int id = blockIdx.x;
  const int xcd = id & 7, slot = id >> 3;
  const int xn = 8 / xm;                                   // XCD groups along the panels; xm of them along M
  const int xmi = xcd % xm, xni = xcd / xm;
  const int mt_per = (m_tiles + xm - 1) / xm;              // m tiles of one group along M
  const int pq = slot / mt_per, mt = xmi * mt_per + (slot - pq * mt_per);
  const int panel = pq * xn + xni;
  if (panel >= n_tiles * splits || mt >= m_tiles) return;
  const int nt = panel % n_tiles, sp = panel / n_tiles;

  const int M = eff_rows(a.M, a.m_dev);
  const int m0 = mt * BM;
  if (m0 >= M) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kw = wave % KW, nw = wave / KW;
  const int nblocks = a.N >> 5;
  const int kb16 = a.K >> 4;                               // k-steps in the whole K
  const int nb0 = (nt * NWN + nw) * WN;
  const int total_chunks = (a.K + KC - 1) / KC;
  const int c_begin = sp * chunks_per_split;
  int n_chunks = total_chunks - c_begin;
  if (n_chunks > chunks_per_split) n_chunks = chunks_per_split;
  const int s_begin = c_begin * KSTEPS;                    // first global k-step of this workgroup
  int n_steps = kb16 - s_begin;                            // valid k-steps of this workgroup
  if (n_steps > n_chunks * KSTEPS) n_steps = n_chunks * KSTEPS;

  const bf16* __restrict__ A = (const bf16*)a.A;
  const bf16x8* __restrict__ Wp = (const bf16x8*)a.W;

  f32x16 acc[WM][WN];
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  bf16x8 zero8;
#pragma unroll
  for (int e = 0; e < 8; ++e) zero8[e] = (bf16)0.f;

  bf16x8 areg[PPT];
  auto load_a = [&](int chunk) {                           // chunk: index inside this workgroup
    // unconditional loads from clamped (always valid) addresses keep the loop free of branches, so the
    // loads stay in flight; rows >= M are never stored, columns past this workgroup's K range are zeroed
    const int k0 = (c_begin + chunk) * KC;
    const bool live = chunk < n_chunks;
#pragma unroll
    for (int i = 0; i < PPT; ++i) {
      const int c = tid + i * 256;
      const int row = c / RPP, kc = c % RPP;
      const int gr = (m0 + row < M) ? m0 + row : M - 1;
      const int k = k0 + kc * 8;
      const bool ok = live && k < a.K;
      const bf16x8 v = *(const bf16x8*)(A + (size_t)gr * a.lda + (ok ? k : 0));
      areg[i] = ok ? v : zero8;
    }
  };
  auto store_a = [&]() {
#pragma unroll
    for (int i = 0; i < PPT; ++i) {
      const int c = tid + i * 256;
      const int row = c / RPP, kc = c % RPP;
      *(bf16x8*)(&lds[row * LDS_STRIDE + kc * 8]) = areg[i];
    }
  };

  // B ring: this wave's k-steps, in order q = chunk * SPW + j, live in slot q % P
  bf16x8 breg[P][WN];
  const bf16x8* bbase[WN];
#pragma unroll
  for (int j = 0; j < WN; ++j) {
    const int nb = (nb0 + j < nblocks) ? nb0 + j : 0;      // columns past N: valid reads, never stored
    bbase[j] = Wp + ((size_t)nb * kb16 + s_begin) * 64 + lane;
  }
  auto load_b = [&](int q, int p) {
    // past the end the last fragment is re-read: it only ever meets zeroed activation columns
    int s = (q / SPW) * KSTEPS + kw * SPW + (q % SPW);
    s = s < n_steps ? s : n_steps - 1;
#pragma unroll
    for (int j = 0; j < WN; ++j) breg[p][j] = bbase[j][(size_t)s * 64];
  };

  load_a(0);
#pragma unroll
  for (int p = 0; p < P; ++p) load_b(p, p);

  const int q_total = n_chunks * SPW;
  // The activation fragments of step g + 1 are read from LDS while the MFMAs of step g run (two sets of registers), and
  // every step ends with a scheduling barrier: without it the compiler gathers the ring's refills of a whole group of
  // steps at the group's start and waits for all of them at its end, so that the memory pipe runs empty once per group.
  bf16x8 af[2][WM];
  auto read_af = [&](int ks, int slot) {
#pragma unroll
    for (int i = 0; i < WM; ++i)
      af[slot][i] = *(const bf16x8*)(&lds[(32 * i + (lane & 31)) * LDS_STRIDE + ks * 16 + (lane >> 5) * 8]);
  };
  static_assert(SPW % 2 == 0 && G % 2 == 0, "fragment sets alternate by step parity");
  for (int q0 = 0; q0 < q_total; q0 += G) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const int q = q0 + g;
      const int ks = kw * SPW + (g % SPW);                 // k-step inside the chunk
      if (g % SPW == 0) {                                  // chunk boundary (static position)
        const int c = q / SPW;
        if (c > 0) __syncthreads();                        // every wave is done reading the previous chunk
        store_a();
        __syncthreads();
        load_a(c + 1);                                     // prefetch; zeros past the last chunk
        read_af(ks, g & 1);
      }
      if ((g + 1) % SPW != 0) read_af(ks + 1, (g + 1) & 1);
#pragma unroll
      for (int j = 0; j < WN; ++j)
#pragma unroll
        for (int i = 0; i < WM; ++i)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[g & 1][i], breg[g % P][j], acc[i][j], 0, 0, 0);
      load_b(q + P, g % P);
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  // partial sums of the KW waves that share columns: waves kw > 0 hand theirs over through LDS, one at a time
  if constexpr (KW > 1) {
    float* red = (float*)lds_raw + (size_t)nw * WM * WN * 16 * 64;
    for (int r = 1; r < KW; ++r) {
      __syncthreads();
      if (kw == r) {
#pragma unroll
        for (int i = 0; i < WM; ++i)
#pragma unroll
          for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) red[((i * WN + j) * 16 + e) * 64 + lane] = acc[i][j][e];
      }
      __syncthreads();
      if (kw == 0) {
#pragma unroll
        for (int i = 0; i < WM; ++i)
#pragma unroll
          for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] += red[((i * WN + j) * 16 + e) * 64 + lane];
      }
    }
  }

  // waves kw == 0 hold the tile's sums
  if constexpr (STAGED) {
    staged_epilogue<WM, WN, NWN>(a, acc, (float*)lds_raw, m0, M, nt * NWN * WN * 32, kw == 0, nw, sp == 0,
                                 splits > 1 && a.epi != EPI_PARTIAL, sp);
    return;
  }
  if (kw != 0) return;
  // epilogue, specialised on (kind, whole tile inside M) so that the executed path is straight-line
  const bool full = (m0 + BM <= M);
  const bool atomic = splits > 1 && a.epi != EPI_PARTIAL;
  const int cl = lane & 31, rhalf = (lane >> 5) * 4;
#define FARD_EPI(KIND)                                                                              \
  do {                                                                                              \
    if (full) epilogue<KIND, true, WM, WN>(a, acc, m0, M, nb0, nblocks, cl, rhalf, sp == 0, atomic, sp); \
    else epilogue<KIND, false, WM, WN>(a, acc, m0, M, nb0, nblocks, cl, rhalf, sp == 0, atomic, sp);     \
  } while (0)
  switch (a.epi) {
    case EPI_STORE: FARD_EPI(EPI_STORE); break;
    case EPI_STORE_F32: FARD_EPI(EPI_STORE_F32); break;
    case EPI_RESID: FARD_EPI(EPI_RESID); break;
    case EPI_GATE_RESID: FARD_EPI(EPI_GATE_RESID); break;
    case EPI_SWIGLU: FARD_EPI(EPI_SWIGLU); break;
    case EPI_PARTIAL: FARD_EPI(EPI_PARTIAL); break;
    default: break;
  }
#undef FARD_EPI
}

template <int WM, int WN, int KW, int P, int KC>
hipError_t launch_cfg(hipStream_t s, const GemmArgs& a, int splits) {
  constexpr int BN = 32 * WN * (4 / KW), BM = 32 * WM;
  const int n_tiles = (a.N + BN - 1) / BN;
  const int m_tiles = (a.M + BM - 1) / BM;
  const int total_chunks = (a.K + KC - 1) / KC;
  if (splits > total_chunks) splits = total_chunks;
  if (splits < 1) splits = 1;
  const int cps = (total_chunks + splits - 1) / splits;
  splits = (total_chunks + cps - 1) / cps;
  const int panels = n_tiles * splits;
  // XCD groups: every XCD has its own L2 and fetches what its workgroups read.  With xm groups along M and 8 / xm
  // along the panels an XCD reads 1 / xm of the activations and xm / 8 of the weights; take the split with the least
  // bytes fetched over all eight (measured: a 2304 x 5120 x 1280 product fetches 224 MB with xm = 1 and runs in
  // 82 us, 55 us with xm = 4).
  int xm = 1;
  {
    const double a_bytes = 2.0 * a.M * a.K, b_bytes = 2.0 * a.K * a.N;
    double best = 8.0 * a_bytes + b_bytes;
    for (int c = 2; c <= 8 && c <= m_tiles; c *= 2) {
      const double cost = (8.0 / c) * a_bytes + c * b_bytes;
      if (cost < 0.98 * best) { best = cost; xm = c; }
    }
  }
  const int xn = 8 / xm;
  const int grid = 8 * ((m_tiles + xm - 1) / xm) * ((panels + xn - 1) / xn);
  // same formula as in the kernel: the activation chunk or the partial sums of the KW wave groups
  constexpr int LDS_STRIDE = KC + 8;
  constexpr int RED_FLOATS = (KW > 1) ? (4 / KW) * WM * WN * 16 * 64 : 0;
  constexpr int STAGE_BYTES = 32 * (BN + 4) * 4;            // staged epilogue only; one size for both instances
  constexpr int LDS_AR = (BM * LDS_STRIDE * 2 > RED_FLOATS * 4) ? BM * LDS_STRIDE * 2 : RED_FLOATS * 4;
  constexpr int LDS_BYTES = LDS_AR > STAGE_BYTES ? LDS_AR : STAGE_BYTES;
  // one row tile: one workgroup per compute unit, each through its epilogue once -> the staged, compact one
  const bool staged = m_tiles == 1;
  if constexpr (LDS_BYTES > 64 * 1024) {
    static bool attr_set = false;                          // per template instance
    if (!attr_set) {
      hipError_t e = hipFuncSetAttribute((const void*)gemm_bf16_kernel<WM, WN, KW, P, KC, true>,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
      if (e == hipSuccess)
        e = hipFuncSetAttribute((const void*)gemm_bf16_kernel<WM, WN, KW, P, KC, false>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
      if (e != hipSuccess) return e;
      attr_set = true;
    }
  }
  if (staged) gemm_bf16_kernel<WM, WN, KW, P, KC, true><<<grid, 256, LDS_BYTES, s>>>(a, n_tiles, m_tiles, splits, cps, xm);
  else gemm_bf16_kernel<WM, WN, KW, P, KC, false><<<grid, 256, LDS_BYTES, s>>>(a, n_tiles, m_tiles, splits, cps, xm);
  return hipGetLastError();
}

// ------------------------------------------------------------------------ skinny variants (M <= a few hundred)
// For the GEMMs of a few hundred rows (2-50 MB of weights each) a launch is one memory round trip long
// if, and only if, every load it needs is in flight from the first cycle:
// gemm_bf16_res_kernel (64 < M): the whole activation panel of the workgroup (64 rows x its K range,
// in passes of up to ~1100 k) goes HBM/L2 -> LDS by the direct-to-LDS loads of gfx950
// (global_load_lds_dwordx4: no registers, 1 KiB per wave instruction) while the first P k-steps of every
// wave's weight stream are requested; one wait, one barrier, then an MFMA loop without barriers whose
// LDS fragment reads run two steps ahead of the MFMAs.
// It finishes through lds_epilogue: partial tiles meet in LDS, then all 256 threads read them back
// row-contiguous and write 8-16 bytes per lane (full cache lines) instead of 2-byte scattered stores.
constexpr int RU = 1056;              // bytes between activation units in LDS (1 KiB unit + 32 B: conflict-free reads)

// Tile of the workgroup: BM x BN, partial sums of KW wave groups.  lds holds KW * BM * (BN + 4) floats.
template <int WM, int WN, int KW, int NWN>
__device__ __forceinline__ void lds_epilogue(const GemmArgs& a, f32x16 (&acc)[WM][WN], float* lds, int m0, int M,
                                             int n0, int kw, int nw, bool add_bias, bool atomic) {
  constexpr int BM = 32 * WM, BNW = 32 * WN, BN = BNW * NWN, LDT = BN + 4;
  const int lane = threadIdx.x & 63;
  // a thread keeps its 4 columns over all rows of the tile: its bias is requested before the barriers
  constexpr int GPR = BN / 4;                              // groups of 4 columns per row
  static_assert(256 % GPR == 0, "a thread keeps its column group over all rows");
  const int col = (threadIdx.x % GPR) * 4;
  const int gc = n0 + col;
  f32x4 bias4 = {0.f, 0.f, 0.f, 0.f};
  if (a.epi != EPI_SWIGLU && a.bias != nullptr && add_bias && gc < a.N) bias4 = *(const f32x4*)(a.bias + gc);
  __syncthreads();                                         // the staging area is free
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int row = 32 * i + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
        lds[(kw * BM + row) * LDT + nw * BNW + 32 * j + (lane & 31)] = acc[i][j][e];
      }
  __syncthreads();
  const int N = a.N;
  if (a.epi == EPI_SWIGLU) {
    // packed column blocks alternate gate / up (32 columns each): output column = packed / 2
    constexpr int OGPR = BN / 8;                           // groups of 4 output columns per row
    bf16* out = (bf16*)a.out;
    for (int idx = threadIdx.x; idx < BM * OGPR; idx += 256) {
      const int row = idx / OGPR, og = idx - row * OGPR;
      const int oc = og * 4;                               // output column inside the tile's output half
      const int pc = (oc >> 5) * 64 + (oc & 31);           // packed column of the gate value
      const int gr = m0 + row;
      if (gr >= M || n0 + pc + 32 >= N) continue;         // gate and up blocks both inside N
      f32x4 g = {0.f, 0.f, 0.f, 0.f}, u = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int k = 0; k < KW; ++k) {
        g += *(const f32x4*)(&lds[(k * BM + row) * LDT + pc]);
        u += *(const f32x4*)(&lds[(k * BM + row) * LDT + pc + 32]);
      }
      bf16x4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = (bf16)(silu(g[e]) * u[e]);
      *(bf16x4*)(out + (size_t)gr * a.ldo + (n0 >> 1) + oc) = o;
    }
    return;
  }
  if (gc >= N) return;                                     // N % 32 == 0: a group is all in or all out
  for (int row = threadIdx.x / GPR; row < BM; row += 256 / GPR) {
    const int gr = m0 + row;
    if (gr >= M) break;
    f32x4 v = bias4;
#pragma unroll
    for (int k = 0; k < KW; ++k) v += *(const f32x4*)(&lds[(k * BM + row) * LDT + col]);
    const size_t o = (size_t)gr * a.ldo + gc;
    if (a.epi == EPI_STORE) {
      bf16x4 t;
#pragma unroll
      for (int e = 0; e < 4; ++e) t[e] = (bf16)apply_act(v[e], a.act);
      *(bf16x4*)((bf16*)a.out + o) = t;
    } else if (a.epi == EPI_STORE_F32) {
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = apply_act(v[e], a.act);
      *(f32x4*)((float*)a.out + o) = v;
    } else {
      if (a.epi == EPI_GATE_RESID) v *= *(const f32x4*)(a.gate + (size_t)gr * a.ldg + gc);
      float* dst = (float*)a.out + o;
      if (atomic) {
#pragma unroll
        for (int e = 0; e < 4; ++e) atomicAdd(dst + e, v[e]);   // partial sums of a split K range meet in memory
      } else {
        *(f32x4*)dst = *(const f32x4*)dst + v;
      }
    }
  }
}

template <int WM, int WN, int KW, int P>
__global__ __launch_bounds__(256) void gemm_bf16_res_kernel(GemmArgs a, int n_tiles, int m_tiles, int splits,
                                                            int chunks_per_split, int chunks_per_pass) {
  constexpr int NWN = 4 / KW;
  constexpr int SPW = 16 / KW;                             // k-steps per wave per 256-k chunk
  constexpr int BM = 32 * WM;
  constexpr int UPC = BM / 2;                              // units per chunk
  constexpr int AD = 3;                                    // LDS fragment reads run AD steps ahead (ring of AD+1 divides P)
  static_assert(P % (AD + 1) == 0, "fragment ring must divide the weight ring");
  extern __shared__ __attribute__((aligned(16))) char lds_raw[];

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
  const int kw = wave % KW, nw = wave / KW;
  const int nblocks = a.N >> 5;
  const int kb16 = a.K >> 4;
  const int nb0 = (nt * NWN + nw) * WN;
  const int total_chunks = a.K >> 8;                       // K % 256 == 0 (host check)
  const int c_begin = sp * chunks_per_split;
  int n_chunks = total_chunks - c_begin;
  if (n_chunks > chunks_per_split) n_chunks = chunks_per_split;
  const int n_steps = n_chunks * 16;                       // k-steps of this workgroup
  const int s_begin = c_begin * 16;

  const bf16* __restrict__ A = (const bf16*)a.A;
  const bf16x8* __restrict__ Wp = (const bf16x8*)a.W;

  f32x16 acc[WM][WN];
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  bf16x8 zero8;
#pragma unroll
  for (int e = 0; e < 8; ++e) zero8[e] = (bf16)0.f;

  // weight ring: this wave's k-steps in order q = chunk * SPW + j live in slot q % P
  bf16x8 breg[P][WN];
  const bf16x8* bbase[WN];
#pragma unroll
  for (int j = 0; j < WN; ++j) {
    const int nb = (nb0 + j < nblocks) ? nb0 + j : 0;      // columns past N: valid reads, never stored
    bbase[j] = Wp + ((size_t)nb * kb16 + s_begin) * 64 + lane;
  }
  auto load_b = [&](int q, int p) {
    int s = (q / SPW) * 16 + kw * SPW + (q % SPW);
    s = s < n_steps ? s : n_steps - 1;                     // past the end: a re-read that only meets zeros
#pragma unroll
    for (int j = 0; j < WN; ++j) breg[p][j] = bbase[j][(size_t)s * 64];
  };
#pragma unroll
  for (int p = 0; p < P; ++p) load_b(p, p);

  const int urow = lane & 1, ukp = lane >> 1;              // lane -> (row parity, k-piece) inside a unit
  const int q_total = n_chunks * SPW;
  const int wave_steps_per_pass = chunks_per_pass * SPW;
  // byte offset of this lane's fragment inside a unit pair, for row block i: rows 32 i + lane % 32
  int frag_off[WM];
#pragma unroll
  for (int i = 0; i < WM; ++i) {
    const int r = 32 * i + (lane & 31);
    frag_off[i] = (r >> 1) * RU + ((((lane >> 5) * 2) + (r & 1)) << 4);
  }

  for (int pass0 = 0; pass0 < n_chunks; pass0 += chunks_per_pass) {
    int pc = n_chunks - pass0;
    if (pc > chunks_per_pass) pc = chunks_per_pass;
    if (pass0 > 0) __syncthreads();                        // previous panel fully consumed
    for (int u = wave; u < pc * UPC; u += 4) {             // activation panel: units dealt to the waves
      const int c = u / UPC, pr = u - c * UPC;
      int row = m0 + 2 * pr + urow;
      row = row < M ? row : M - 1;                         // rows past M: valid reads, never stored
      const bf16* g = A + (size_t)row * a.lda + (size_t)(c_begin + pass0 + c) * 256 + ukp * 8;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                       (__attribute__((address_space(3))) void*)(lds_raw + (size_t)u * RU), 16, 0, 0);
    }
    __builtin_amdgcn_s_waitcnt(0);                         // every outstanding load of this wave, LDS writes included
    __syncthreads();

    const int q_begin = pass0 * SPW;
    int q_end = q_begin + wave_steps_per_pass;
    if (q_end > q_total) q_end = q_total;
    // fragment of step q (clamped to the panel; steps past its end are zeroed at use)
    auto frag = [&](int q, bf16x8 (&f)[WM]) {
      const int qc = q < q_end ? q : q_end - 1;
      const int c = qc / SPW - pass0;
      const int ks = kw * SPW + (qc % SPW);
      const int base = c * UPC * RU + ks * 64;             // a k-step is 2 pieces x 2 rows x 16 B = 64 B further
#pragma unroll
      for (int i = 0; i < WM; ++i) f[i] = *(const bf16x8*)(lds_raw + base + frag_off[i]);
    };
    bf16x8 af[AD + 1][WM];
#pragma unroll
    for (int d = 0; d < AD; ++d) frag(q_begin + d, af[d]);
    for (int q0 = q_begin; q0 < q_end; q0 += P) {
#pragma unroll
      for (int g = 0; g < P; ++g) {
        const int q = q0 + g;
        frag(q + AD, af[(g + AD) % (AD + 1)]);
        const bool live = q < q_end;                       // select, not a branch: branches would drain the ring
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
          for (int i = 0; i < WM; ++i)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(live ? af[g % (AD + 1)][i] : zero8, breg[g][j],
                                                                acc[i][j], 0, 0, 0);
        load_b(q + P, g);
        __builtin_amdgcn_sched_barrier(0);                 // the refill stays P steps ahead of its use
      }
    }
  }
  lds_epilogue<WM, WN, KW, NWN>(a, acc, (float*)lds_raw, m0, M, nt * NWN * WN * 32, kw, nw, sp == 0, splits > 1);
}

constexpr int RES_LDS_BUDGET = 150 * 1024;

template <int WM, int WN, int KW, int P>
hipError_t launch_res(hipStream_t s, const GemmArgs& a, int splits) {
  const int BN = 32 * WN * (4 / KW), BM = 32 * WM;
  const int n_tiles = (a.N + BN - 1) / BN;
  const int m_tiles = (a.M + BM - 1) / BM;
  const int total_chunks = a.K / 256;
  if (splits > total_chunks) splits = total_chunks;
  if (splits < 1) splits = 1;
  const int cps = (total_chunks + splits - 1) / splits;
  splits = (total_chunks + cps - 1) / cps;
  const int chunk_bytes = (BM / 2) * RU;
  int cpp = RES_LDS_BUDGET / chunk_bytes;                  // chunks resident per pass
  if (cpp > cps) cpp = cps;
  size_t lds = (size_t)cpp * chunk_bytes;
  const size_t epi = (size_t)KW * BM * (BN + 4) * 4;
  if (lds < epi) lds = epi;
  static bool attr_set = false;                            // per template instance
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)gemm_bf16_res_kernel<WM, WN, KW, P>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, RES_LDS_BUDGET + 8192);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int panels = n_tiles * splits;
  const int grid = ((panels + 7) / 8) * 8 * m_tiles;
  gemm_bf16_res_kernel<WM, WN, KW, P><<<grid, 256, lds, s>>>(a, n_tiles, m_tiles, splits, cps, cpp);
  return hipGetLastError();
}

// Tile choice.  The chip has 256 CUs; these GEMMs rarely have that many 128-column tiles, so narrow
// tiles (waves splitting K inside the workgroup) and K splits across workgroups are used until the
// grid covers it.  EPI_SWIGLU needs both column blocks of a pair in one wave (WN = 2).
template <int WM>
hipError_t launch_wm(hipStream_t s, const GemmArgs& a) {
  const bool resid = (a.epi == EPI_RESID || a.epi == EPI_GATE_RESID);
  if constexpr (WM == 3) {
    // a few hundred rows, full-K store epilogue: 64-row streaming tiles when they waste fewer rows than 96-row ones
    // (measured over whole rounds against the resident-activation kernel: 29.4 -> 29.0 ms with 256-row draft steps)
    if (!resid && a.epi != EPI_SWIGLU && a.M > 96 && a.M <= 640) {
      const int m64 = (a.M + 63) / 64, m96 = (a.M + 95) / 96;
      if (m64 * 64 < m96 * 96) return launch_cfg<2, 1, 1, 8, 256>(s, a, 1);
    }
    // 65-96 rows with a SwiGLU epilogue: one 96-row tile of the streaming kernel, two waves per 64 packed columns sharing
    // the k-steps (measured at 72 x 27648 x 5120: 62 us against 78 us for two 64-row tiles of the resident-activation
    // kernel, which stream every weight panel twice)
    if (a.epi == EPI_SWIGLU && a.M > 64 && a.M <= 96) return launch_cfg<3, 2, 2, 16, 256>(s, a, 1);
    // up to 96 rows, or a SwiGLU epilogue: the resident-activation kernel on 64-row tiles, sized so that the
    // grid stays within one workgroup per CU
    if (!resid && (a.M <= 96 || a.epi == EPI_SWIGLU) && a.M <= 640 && a.K % 256 == 0) {
      const int mt64 = (a.M + 63) / 64;
      if (a.epi == EPI_SWIGLU || ((a.N + 63) / 64) * mt64 > 256) {
        if (((a.N + 127) / 128) * mt64 <= 288) return launch_res<2, 2, 2, 16>(s, a, 1);
      } else {
        return launch_res<2, 1, 2, 16>(s, a, 1);
      }
    }
  }
  const int m_tiles = (a.M + 32 * WM - 1) / (32 * WM);
  constexpr int KC = 256;
  const int total_chunks = (a.K + KC - 1) / KC;
  auto tiles = [&](int bn) { return ((a.N + bn - 1) / bn) * m_tiles; };
  auto splits_for = [&](int t) { return (resid && t < 256) ? (256 + t - 1) / t : 1; };
  if constexpr (WM >= 3) {
    // Hundreds to thousands of rows: MFMA-bound tiles, many per compute unit.  An 8-step weight ring (not 16) keeps
    // 64x256, 64x128 and 96x128 tiles within 256 registers, so two workgroups share a compute unit and one's epilogue
    // and ramp overlap the other's MFMA loop; measured over the verify and prefill shapes (TFLOP/s, 16-step ring of
    // the same or the previously routed tile -> 8-step): 6144 x 7168 x 5120 966 -> 1184 and 6144 x 5120 x 5120
    // 804 -> 1062 (64x256), 6144 x 5120 x 13824 953 -> 1064 (128x128), SwiGLU 6144 x 27648 x 5120 1176 -> 1255
    // (128x256), 8256 x 5120 x 1280 624 -> 890, 4128 x 3072 x 1024 447 -> 761 and 2304 x 5120 x 1280 685 -> 807
    // (64x128), 576 x 5120 x 1280 442 -> 540 (96x128).
    auto t = [&](int bm, int bn) { return ((a.N + bn - 1) / bn) * ((a.M + bm - 1) / bm); };
    // A few hundred rows against a matrix whose 96-row tiles would leave half the chip idle: 32 x 128 tiles (136
    // registers: three workgroups per compute unit), for residual epilogues with K split over enough workgroups to
    // cover the chip (measured: 288 x 3072 x 1024 11.9 -> 7.4 us, 576 x 1280 x 1280 15.8 -> 8.9 us with 2 splits,
    // 288 x 1024 x 4096 13.9 -> 10.8-11.1 us, 576 x 1280 x 5120 22.3 -> 18.8 us)
    if (a.epi != EPI_SWIGLU && a.M > 96 && t(96, 128) < 128 && t(32, 128) >= 64) {
      int sp = 1;
      if (resid) sp = std::min(std::max((256 + t(32, 128) - 1) / t(32, 128), 1), std::min(total_chunks, 4));
      return launch_cfg<1, 1, 1, 8, 256>(s, a, sp);
    }
    if (a.epi == EPI_SWIGLU) {
      if (tiles(256) >= 512) return launch_cfg<4, 2, 1, 8, 256>(s, a, 1);
    } else if (!resid || t(64, 128) >= 512 || (t(64, 128) >= 256 && a.K <= 2048)) {
      // (a residual epilogue with few tiles or a long K keeps the K split over workgroups below)
      if (a.K > 8192 && t(128, 128) >= 512) return launch_cfg<4, 1, 1, 8, 256>(s, a, 1);
      if (t(64, 256) >= 900) return launch_cfg<2, 2, 1, 8, 256>(s, a, 1);
      if (t(64, 128) >= 400) return launch_cfg<2, 1, 1, 8, 256>(s, a, 1);
      if (!resid) return launch_cfg<3, 1, 1, 8, 256>(s, a, 1);
    }
  }
  if (tiles(256) >= 512) return launch_cfg<WM, 2, 1, 16, 256>(s, a, 1);
  if (a.epi != EPI_SWIGLU && tiles(128) * (resid ? total_chunks : 1) >= 256)
    return launch_cfg<WM, 1, 1, WM >= 3 ? 8 : 16, 256>(s, a, splits_for(tiles(128)));
  if (WM > 1 && a.epi != EPI_SWIGLU) return launch_cfg<WM, 1, 1, WM >= 3 ? 8 : 16, 256>(s, a, splits_for(tiles(128)));
  if (a.epi == EPI_SWIGLU || tiles(64) >= 192) return launch_cfg<WM, 2, 4, 8, 256>(s, a, splits_for(tiles(64)));
  return launch_cfg<WM, 1, 4, 8, 256>(s, a, splits_for(tiles(32)));
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
  if (a.K % 64 != 0 || a.N % 32 != 0 || a.lda % 8 != 0) return hipErrorInvalidValue;
  if (a.epi == EPI_SWIGLU && a.N % 64 != 0) return hipErrorInvalidValue;
  if (a.M <= 32) return launch_wm<1>(s, a);
  if (a.M <= 64) return launch_wm<2>(s, a);
  // thousands of rows: 128-row tiles reuse every weight fragment a third more often than 96-row tiles and win once
  // they still make several rounds of 256-column workgroups over the chip (measured: + 5-15 % from about 900
  // workgroups on, - 13-37 % below)
  if ((long)((a.N + 255) / 256) * ((a.M + 127) / 128) >= 900) return launch_wm<4>(s, a);
  return launch_wm<3>(s, a);
}

int gemm_plane_count(int K, int splits) {
  const int total_chunks = (K + 255) / 256;
  if (splits > total_chunks) splits = total_chunks;
  if (splits < 1) splits = 1;
  const int cps = (total_chunks + splits - 1) / splits;
  return (total_chunks + cps - 1) / cps;
}

hipError_t launch_gemm_bf16_planes(hipStream_t s, const GemmArgs& a) {
  if (a.M <= 0) return hipSuccess;
  if (a.epi != EPI_PARTIAL || a.K % 64 != 0 || a.N % 32 != 0 || a.lda % 8 != 0) return hipErrorInvalidValue;
  if (a.k_slices != gemm_plane_count(a.K, a.k_slices) || a.part_stride < (size_t)a.M * a.ldo) return hipErrorInvalidValue;
  // 128-column workgroups, one 32-column block per wave, a 16-step weight ring (measured at 72 rows against 50-280 MB of
  // weights: ahead of 256- and 64-column workgroups and of an 8-step ring at every split count)
  if (a.M <= 32) return launch_cfg<1, 1, 1, 16, 256>(s, a, a.k_slices);
  if (a.M <= 64) return launch_cfg<2, 1, 1, 16, 256>(s, a, a.k_slices);
  if (a.M <= 96) return launch_cfg<3, 1, 1, 16, 256>(s, a, a.k_slices);
  if (a.M <= 128) return launch_cfg<4, 1, 1, 16, 256>(s, a, a.k_slices);
  return hipErrorInvalidValue;
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

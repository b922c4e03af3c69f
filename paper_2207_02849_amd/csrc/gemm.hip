// Grouped MFMA GEMM with fused epilogues for gfx950.
//
//   C (fp32 accumulators) = sum_p A_p * B_p^T  over one or two operand pairs, then an epilogue.
//
// Every dense contraction of the hypergradient path (forward, backward, and the forward-
// over-reverse passes of the Hessian-vector product; paper Sec. 3.2) has this shape because each
// operand is kept in the workspace with its reduction index contiguous ("K-major") and zero-
// padded to a multiple of 128 in both extents.  The two-pair form is the concatenated-K product
// of the R-op passes, e.g. Rz = Ra W + a V as [Ra | a] [W ; V].
//
// Launch = a batch of up to MAX_PROBLEMS independent problems plus optional bias-row jobs,
// flattened on blockIdx.x.  Skinny problems (few output tiles, long K) are split along K *inside*
// the workgroup: KG groups (of 4 wavefronts, or of one) each take a contiguous range of k-tiles with their own
// LDS operand buffers, and the groups' accumulators are summed through LDS in group order, so the
// result is bit-reproducible and no inter-workgroup synchronisation exists.  (Splitting K across
// workgroups was measured first: the agent-scope fences it needs write back the L2 of every XCD
// and cost 10-80 us per launch on this chip.)
//
// Tiling: 4 wavefronts (2 x 2), or 8 (4 x 2) on the 128 x 64 tiles, own a BM x BN tile; a wavefront
// owns TM x TN MFMA blocks of 32 x 32.  K is consumed in tiles of NCH 16-byte chunks per row: global -> registers
// -> LDS with the next tile's global loads in flight during the multiplies.  LDS rows are padded
// by one chunk so the 16-byte fragment reads of 8 consecutive rows hit distinct banks.
//
// Fragments: lane l supplies row (l % 32) of the A block and of the B block; lanes 0-31 take the
// even chunks of the k-tile, lanes 32-63 the odd ones.  A chunk is 8 bf16 (one
// v_mfma_f32_32x32x16_bf16) or 4 floats (four v_mfma_f32_32x32x2_f32); A and B share the chunk
// assignment, so the order of k inside the product does not matter.  Register r of lane l holds
// C[8*(r/4) + 4*(l/32) + r%4][l%32]: four consecutive rows of one column per register quad, which
// is what the epilogues consume (one 4-element vector store into the transposed output).
#include "internal.h"

namespace betty {

// ------------------------------------------------------------------------------------------
// epilogue helpers
// ------------------------------------------------------------------------------------------

__device__ __forceinline__ void act_eval(int act, float z, float& a, float& d1, float& d2) {
  if (act == BETTY_ACT_RELU) {
    const bool pos = z > 0.f;
    a = pos ? z : 0.f; d1 = pos ? 1.f : 0.f; d2 = 0.f;
  } else if (act == BETTY_ACT_GELU_ERF) {
    const float Phi = 0.5f * (1.f + erff(z * 0.70710678118654752f));
    const float pdf = 0.39894228040143268f * expf(-0.5f * z * z);
    a = z * Phi; d1 = Phi + z * pdf; d2 = pdf * (2.f - z * z);
  } else {
    a = z; d1 = 1.f; d2 = 0.f;
  }
}

template <typename T> __device__ __forceinline__ void store1(T* p, float x);
template <> __device__ __forceinline__ void store1<float>(float* p, float x) { *p = x; }
template <> __device__ __forceinline__ void store1<__bf16>(__bf16* p, float x) { *p = (__bf16)x; }

// four consecutive elements, p aligned to 4 elements
template <typename T> __device__ __forceinline__ void store4(T* p, const float (&x)[4]);
template <> __device__ __forceinline__ void store4<float>(float* p, const float (&x)[4]) {
  *(float4*)p = make_float4(x[0], x[1], x[2], x[3]);
}
template <> __device__ __forceinline__ void store4<__bf16>(__bf16* p, const float (&x)[4]) {
  typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
  bf16x4 v = {(__bf16)x[0], (__bf16)x[1], (__bf16)x[2], (__bf16)x[3]};
  *(bf16x4*)p = v;
}

// One 32x32 MFMA block as seen by one lane: 16 accumulators = rows rb + 8*(k/4) + k%4 (k = 0..15)
// of column col, with rb = block row + 4*(lane/32).  M, N = valid extent.
//
// The epilogue is split in two so that its memory latency hides behind the k loop: epi_prefetch
// (before the loop) issues every load the mode needs for the block's 16 elements into EpiRegs;
// epi_finish (after the loop) computes and stores.  Nothing the prefetch reads is written by the
// same launch before epi_finish of the same element.
// NR = 16: a whole block;  NR = 4: one register quad (four consecutive rows), rb already at its first row.
template <int NR> struct EpiRegs { float a[NR], b[NR], c[NR], d[NR]; float colv; };

template <int NR> __device__ __forceinline__ int epi_row(int rb, int k) { return NR == 16 ? rb + 8 * (k >> 2) + (k & 3) : rb + k; }

template <int NR>
__device__ __forceinline__ int epi_offset(int rb, int k, long long ld, int col) {
  return (int)((long long)epi_row<NR>(rb, k) * ld + col);   // layer slices are < 2^31 elements
}

template <int MODE, int NR>
__device__ __forceinline__ void epi_prefetch(const Epilogue& e, int M, int N, int rb, int col, EpiRegs<NR>& R) {
  if constexpr (MODE == EPI_RFWD_LAST_HESS) {
    // every lane of the block takes part in the row sums later: lanes outside the valid extent hold zeros
    const bool colok = col < N;
    R.colv = (colok && e.colvec) ? e.colvec[col] : 0.f;
#pragma unroll
    for (int k = 0; k < NR; ++k) {
      const int row = epi_row<NR>(rb, k);
      const bool ok = colok && row < M;
      R.a[k] = (ok && e.dphi) ? e.dphi[epi_offset<NR>(rb, k, e.ldf, col)] : 0.f;
      R.b[k] = ok ? e.e[row] : 0.f;
    }
    return;
  }
  if (col >= N || rb >= M) return;
  const long long ldx = MODE >= EPI_WGRAD ? e.ldc : e.ldf;
  if constexpr (MODE == EPI_FWD || MODE == EPI_FWD_LAST || MODE == EPI_RFWD || MODE == EPI_RFWD_LAST)
    R.colv = e.colvec ? e.colvec[col] : 0.f;
#pragma unroll
  for (int k = 0; k < NR; ++k) {
    const bool ok = epi_row<NR>(rb, k) < M;
    const int o = epi_offset<NR>(rb, k, ldx, col);
    if constexpr (MODE == EPI_BWD) {
      R.a[k] = ok ? e.dphi[o] : 0.f;
      R.b[k] = (ok && e.e_io) ? e.e_io[o] : 0.f;
    } else if constexpr (MODE == EPI_RFWD) {
      R.a[k] = ok ? e.dphi[o] : 0.f;
    } else if constexpr (MODE == EPI_RBWD) {
      R.a[k] = ok ? e.dphi[o] : 0.f;
      R.b[k] = (ok && e.e) ? e.e[o] : 0.f;
      R.c[k] = (ok && e.e) ? e.Rz[o] : 0.f;
    } else if constexpr (MODE == EPI_WGRAD) {
      R.a[k] = (ok && e.lam) ? e.lam[o] : 0.f;
      R.b[k] = (ok && e.lam) ? e.x[o] : 0.f;
    } else if constexpr (MODE == EPI_WGRAD_NEUMANN) {
      R.a[k] = ok ? e.x[o] : 0.f;                         // s: the partial sum so far
      R.b[k] = ok ? e.v[o] : 0.f;                         // g: the vector the series is applied to
      R.c[k] = (ok && e.lam) ? e.lam[o] : 0.f;
    } else if constexpr (MODE == EPI_WGRAD_NEUMANN_L2) {
      R.a[k] = ok ? e.p[o] : 0.f;                         // s
      R.b[k] = ok ? e.v[o] : 0.f;                         // g
      R.c[k] = ok ? e.lam[o] : 0.f;
      R.d[k] = ok ? e.x[o] : 0.f;                         // w
    } else if constexpr (MODE == EPI_WGRAD_SGD) {
      R.a[k] = ok ? e.v[o] : 0.f;
      R.b[k] = ok ? e.p[o] : 0.f;
      R.c[k] = (ok && e.lam) ? e.lam[o] : 0.f;
      R.d[k] = (ok && e.x) ? e.x[o] : 0.f;
    }
  }
}

template <typename T, int MODE, int NR>
__device__ __forceinline__ void epi_finish(const Epilogue& e, int M, int N, int rb, int col,
                                           const float (&acc)[NR], const EpiRegs<NR>& R) {
  float val[NR];
  if constexpr (MODE == EPI_RFWD_LAST_HESS) {
    // rows live across the 32 lanes of a half-wavefront (lane % 32 = column): butterfly sums
    const bool colok = col < N;
    float rz[NR], dot[NR];
#pragma unroll
    for (int k = 0; k < NR; ++k) {
      rz[k] = colok ? acc[k] + R.colv : 0.f;
      dot[k] = R.a[k] * rz[k];
    }
    if (e.act == BETTY_LOSS_SOFTMAX_CE) {
#pragma unroll
      for (int o = 16; o > 0; o >>= 1)
#pragma unroll
        for (int k = 0; k < NR; ++k) dot[k] += __shfl_xor(dot[k], o, 64);
#pragma unroll
      for (int k = 0; k < NR; ++k) val[k] = R.b[k] * (R.a[k] * rz[k] - R.a[k] * dot[k]);
    } else {
#pragma unroll
      for (int k = 0; k < NR; ++k) val[k] = R.b[k] * 2.f * rz[k];
    }
  }
  if (col >= N || rb >= M) return;
  const long long ldx = MODE >= EPI_WGRAD ? e.ldc : e.ldf;
  bool ok[NR];
  int of[NR];
#pragma unroll
  for (int k = 0; k < NR; ++k) {
    ok[k] = epi_row<NR>(rb, k) < M;
    of[k] = epi_offset<NR>(rb, k, ldx, col);
  }
  if constexpr (MODE == EPI_RFWD_LAST_HESS) {
    // val is set; fall through to the operand copies
  } else if constexpr (MODE == EPI_FWD) {
    float d1[NR], d2[NR];
#pragma unroll
    for (int k = 0; k < NR; ++k) act_eval(e.act, acc[k] + R.colv, val[k], d1[k], d2[k]);
#pragma unroll
    for (int k = 0; k < NR; ++k)
      if (ok[k]) e.dphi_out[of[k]] = d1[k];
    if (e.d2_out) {
#pragma unroll
      for (int k = 0; k < NR; ++k)
        if (ok[k]) e.d2_out[of[k]] = d2[k];
    }
  } else if constexpr (MODE == EPI_FWD_LAST || MODE == EPI_RFWD_LAST) {
#pragma unroll
    for (int k = 0; k < NR; ++k)
      if (ok[k]) e.f0[of[k]] = acc[k] + R.colv;
    return;
  } else if constexpr (MODE == EPI_BWD) {
    if (e.e_io) {
#pragma unroll
      for (int k = 0; k < NR; ++k)
        if (ok[k]) e.e_io[of[k]] = acc[k] * R.b[k];
    }
#pragma unroll
    for (int k = 0; k < NR; ++k) val[k] = acc[k] * R.a[k];
  } else if constexpr (MODE == EPI_RFWD) {
#pragma unroll
    for (int k = 0; k < NR; ++k)
      if (ok[k]) e.f0[of[k]] = acc[k] + R.colv;
#pragma unroll
    for (int k = 0; k < NR; ++k) val[k] = R.a[k] * (acc[k] + R.colv);
  } else if constexpr (MODE == EPI_RBWD) {
#pragma unroll
    for (int k = 0; k < NR; ++k) val[k] = acc[k] * R.a[k] + R.b[k] * R.c[k];
  } else if constexpr (MODE == EPI_WGRAD) {            // C = acc (+ 2 e^lam x)
    if (e.lam) {
#pragma unroll
      for (int k = 0; k < NR; ++k)
        if (ok[k]) e.C[of[k]] = acc[k] + 2.f * expf(R.a[k]) * R.b[k];
    } else {
#pragma unroll
      for (int k = 0; k < NR; ++k)
        if (ok[k]) e.C[of[k]] = acc[k];
    }
    return;
  } else if constexpr (MODE == EPI_WGRAD_INIT) {       // v = acc (and p = acc if asked); operand copies
#pragma unroll
    for (int k = 0; k < NR; ++k) {
      val[k] = acc[k];
      if (ok[k]) { e.v[of[k]] = acc[k]; if (e.p) e.p[of[k]] = acc[k]; }
    }
  } else if constexpr (MODE == EPI_WGRAD_NEUMANN) {    // Hs = acc (+ 2 e^lam s); s <- g + s - alpha Hs
#pragma unroll
    for (int k = 0; k < NR; ++k) {
      float hs = acc[k];
      if (e.lam) hs += 2.f * expf(R.c[k]) * R.a[k];
      val[k] = R.b[k] + (R.a[k] - e.alpha * hs);
    }
#pragma unroll
    for (int k = 0; k < NR; ++k)
      if (ok[k]) e.p[of[k]] = val[k];
  } else if constexpr (MODE == EPI_WGRAD_SGD) {          // lower optimiser step: momentum SGD in place
#pragma unroll
    for (int k = 0; k < NR; ++k) {
      float gk = acc[k] + e.gamma * R.b[k];
      if (e.lam) gk += 2.f * expf(R.c[k]) * (R.b[k] - R.d[k]);     // x: anchor of a proximal term
      const float mk = e.beta * R.a[k] + gk;
      if (ok[k]) { e.v[of[k]] = mk; e.p[of[k]] = R.b[k] - e.alpha * mk; }
    }
    return;
  } else if constexpr (MODE == EPI_WGRAD_NEUMANN_L2) {  // final step: only d(lambda) leaves the kernel
#pragma unroll
    for (int k = 0; k < NR; ++k) {
      const float el = 2.f * expf(R.c[k]);
      const float sn = R.b[k] + (R.a[k] - e.alpha * (acc[k] + el * R.a[k]));
      if (ok[k]) e.C[of[k]] = -el * R.d[k] * (e.alpha * sn);
    }
    return;
  } else {
    return;
  }
  // operand-typed copies: row-major element by element, transposed as 4-element vectors; rows
  // beyond M are written as zeros (they are padding of the transposed operand)
#pragma unroll
  for (int k = 0; k < NR; ++k)
    if (!ok[k]) val[k] = 0.f;
  if (e.out) {
    T* o = (T*)e.out;
#pragma unroll
    for (int k = 0; k < NR; ++k)
      if (ok[k]) store1<T>(o + (long long)epi_row<NR>(rb, k) * e.ld + col, val[k]);
  }
  if (e.outT) {
    T* o = (T*)e.outT + (long long)col * e.ldT + rb;
#pragma unroll
    for (int q = 0; q < NR / 4; ++q) {
      const float quad[4] = {val[4 * q], val[4 * q + 1], val[4 * q + 2], val[4 * q + 3]};
      if (rb + 8 * q < M) store4<T>(o + 8 * q, quad);
    }
  }
  if constexpr (MODE == EPI_FWD && sizeof(T) == 4) {
    // fp32 forward of a bf16 problem: the bf16 operand copies of the activation leave from here too
    if (e.out2) {
      __bf16* o = (__bf16*)e.out2;
#pragma unroll
      for (int k = 0; k < NR; ++k)
        if (ok[k]) store1<__bf16>(o + (long long)epi_row<NR>(rb, k) * e.ld + col, val[k]);
    }
    if (e.outT2) {
      __bf16* o = (__bf16*)e.outT2 + (long long)col * e.ldT + rb;
#pragma unroll
      for (int q = 0; q < NR / 4; ++q) {
        const float quad[4] = {val[4 * q], val[4 * q + 1], val[4 * q + 2], val[4 * q + 3]};
        if (rb + 8 * q < M) store4<__bf16>(o + 8 * q, quad);
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// the kernel
// ------------------------------------------------------------------------------------------

__device__ __forceinline__ float wave_sum_f(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}

// bias-shaped outputs: one wavefront per row of a K-major matrix, same update rules as the tiles
template <typename T, int MODE>
__device__ void bias_rows(const BiasJob& j, int row) {
  const int lane = threadIdx.x & 63;
  if (row >= j.rows) return;
  const T* p = (const T*)j.Mt + (long long)row * j.ld;
  float acc = 0.f;
  for (int c = lane; c < j.k; c += 64) acc += (float)p[c];
  acc = wave_sum_f(acc);
  if (lane != 0) return;
  switch (MODE) {
    case EPI_WGRAD: {
      float g = acc;
      if (j.lam) g += 2.f * expf(j.lam[row]) * j.x[row];
      j.C[row] = g;
      break;
    }
    case EPI_WGRAD_INIT:
      j.v[row] = acc;
      if (j.p) j.p[row] = acc;
      break;
    case EPI_WGRAD_NEUMANN: {
      const float so = j.x[row];
      float hs = acc;
      if (j.lam) hs += 2.f * expf(j.lam[row]) * so;
      j.p[row] = j.v[row] + (so - j.alpha * hs);
      break;
    }
    case EPI_WGRAD_SGD: {
      const float wo = j.p[row];
      float gk = acc + j.gamma * wo;
      if (j.lam) gk += 2.f * expf(j.lam[row]) * (wo - (j.x ? j.x[row] : 0.f));
      const float mk = j.beta * j.v[row] + gk;
      j.v[row] = mk;
      j.p[row] = wo - j.alpha * mk;
      break;
    }
    case EPI_WGRAD_NEUMANN_L2: {
      const float so = j.p[row], el = 2.f * expf(j.lam[row]);
      const float sn = j.v[row] + (so - j.alpha * (acc + el * so));
      j.C[row] = -el * j.x[row] * (j.alpha * sn);
      break;
    }
    default: break;
  }
}

// (128-tiles are compiled for two resident workgroups per compute unit, so that one workgroup's
// epilogue traffic overlaps the other's k loop)
template <typename T, int BM, int BN, int NCH, int WPG, int KG, int MODE>
__global__ __launch_bounds__(64 * WPG * KG, (BM == 128 && KG == 1) ? 2 : 1) void gemm_fused_kernel(GemmBatch batch) {
  constexpr int GT = 64 * WPG;                     // threads of one K group
  constexpr int WM = WPG == 8 ? 4 : WPG == 4 ? 2 : 1, WN = WPG >= 4 ? 2 : 1;   // wavefronts of a group over the tile
  constexpr int ROW = NCH + 1;                     // LDS row pitch in 16-byte chunks
  constexpr int EPC = 16 / (int)sizeof(T);         // elements per chunk
  constexpr int KT = NCH * EPC;                    // elements per k-tile
  constexpr int TM = BM / (32 * WM), TN = BN / (32 * WN);   // 32x32 blocks per wavefront
  constexpr int LA = BM * NCH / GT, LB = BN * NCH / GT;
  static_assert(WPG == 1 || WPG == 4 || WPG == 8, "a K group is one wavefront, 2 x 2 or 4 x 2 wavefronts");
  static_assert(BM % (32 * WM) == 0 && BN % (32 * WN) == 0 && (BM * NCH) % GT == 0 && (BN * NCH) % GT == 0, "tile");
  extern __shared__ u32x4 smem[];

  // KG groups share the tile; group kg owns a contiguous range of k-tiles and its own LDS
  // operand buffers.  (Wavefront-uniform values are forced into scalar registers.)
  const int kg = __builtin_amdgcn_readfirstlane(threadIdx.x / GT);
  const int tid = threadIdx.x % GT, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = WPG >= 4 ? wave >> 1 : 0, wn = WPG >= 4 ? wave & 1 : 0;
  // Unsplit launches keep two LDS operand buffers and alternate between them, so the stores of
  // one k-tile overlap the multiplication of the previous one and a k-tile costs one barrier.
  constexpr bool DB = KG == 1;
  constexpr int LBUF = (BM + BN) * ROW;            // one operand buffer, in chunks
  u32x4* sA = smem + kg * LBUF;
  u32x4* sB = sA + BM * ROW;
  // a one-wavefront group owns its LDS region alone: no workgroup barrier inside the k loop
#define BETTY_GROUP_SYNC() do { if constexpr (WPG == 1) __builtin_amdgcn_wave_barrier(); else __syncthreads(); } while (0)

  // ---- which job is this workgroup?
  int bid = blockIdx.x;
  if (bid >= batch.gemm_blocks) {
    bid -= batch.gemm_blocks;
    int j = 0;
    while (j + 1 < batch.n_bias && bid >= batch.bias_begin[j + 1]) ++j;
    bias_rows<T, MODE>(batch.bias[j], (bid - batch.bias_begin[j]) * (WPG * KG) + (threadIdx.x >> 6));
    return;
  }
  int pi = 0;
  while (pi + 1 < batch.n && bid >= batch.block_begin[pi + 1]) ++pi;
  const GemmArgs& g = batch.p[pi].g;
  const int tile = bid - batch.block_begin[pi];
  const int tiles_n = g.Np / BN;
  int tm = tile / tiles_n, tn = tile % tiles_n;
  if (g.xgm > 0) {                                 // XCD-compact order (see GemmArgs)
    const int x = tile & 7, q = tile >> 3;
    const int rm = (g.Mp / BM) / g.xgm, rn = tiles_n / g.xgn;
    tm = (x / g.xgn) * rm + q / rn;
    tn = (x % g.xgn) * rn + q % rn;
  }
  const int m0 = tm * BM, n0 = tn * BN;

  const int T0 = g.Kp[0] / KT, T1 = g.Kp[1] / KT, TT = T0 + T1;
  const int NI = (TT + KG - 1) / KG;               // iterations of every group (same barrier count)
  const int tb = kg * NI;
  const int te = tb + NI < TT ? tb + NI : TT;

  f32x16 acc[TM * TN];
#pragma unroll
  for (int i = 0; i < TM * TN; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;

  // epilogue inputs of this wavefront's blocks: requested now, consumed after the k loop.  Only
  // group 0 finishes the tile.  (With several blocks per wavefront the prefetch is kept for the
  // parameter-shaped modes, whose epilogue moves far more bytes than their k loop.)
  constexpr bool PREFETCH = TM * TN == 1 || (MODE >= EPI_WGRAD && BM == 64);
  // One-wavefront K groups: the tile is a single MFMA block, and once the groups' partial sums are
  // in LDS the first four wavefronts each finish one register quad of it (four consecutive rows
  // per lane), so the epilogue's arithmetic and stores run on four wavefronts instead of one.
  constexpr bool SPLIT_EPI = WPG == 1 && KG >= 4;
  const Epilogue& e = batch.p[pi].e;
  EpiRegs<16> pre[SPLIT_EPI ? 1 : TM * TN];
  EpiRegs<4> pre4;
  // A wavefront's loads return in the order issued, so a workgroup that requests its epilogue
  // inputs first starts its k loop only once they are there, and one that requests them last waits
  // for them after it: either way it streams and multiplies one after the other, and workgroups
  // that start together do so in step (the memory side idles while every k loop waits on operand
  // latency).  Parameter-shaped launches therefore alternate the two schedules between
  // neighbouring workgroups: one half streams while the other half multiplies (measured on the
  // Neumann weight-gradient launch of the 5M-parameter model: 28.3 -> 25.0 us).
  constexpr bool STAGGER = MODE >= EPI_WGRAD && BM == 64 && KG == 1;
  const bool early = !STAGGER || ((blockIdx.x >> 3) & 1) == 0;
  if constexpr (SPLIT_EPI) {
    if (kg < 4) epi_prefetch<MODE, 4>(e, g.M, g.N, m0 + 8 * kg + 4 * (lane >> 5), n0 + (lane & 31), pre4);
  } else if constexpr (PREFETCH) {
    if (kg == 0 && early) {
#pragma unroll
      for (int ij = 0; ij < TM * TN; ++ij)
        epi_prefetch<MODE, 16>(e, g.M, g.N, m0 + wm * TM * 32 + (ij / TN) * 32 + 4 * (lane >> 5),
                               n0 + wn * TN * 32 + (ij % TN) * 32 + (lane & 31), pre[ij]);
    }
  }

  // Two register sets hold the global loads of the next two k-tiles, so two tiles' worth of
  // loads are in flight while a third is multiplied out of LDS (four sets in the long-loop form
  // of the unsplit activation-shaped launches, see below).
  constexpr bool LONG_LOOP = KG == 1 && MODE < EPI_WGRAD;
  u32x4 ra0[LA], rb0[LB], ra1[LA], rb1[LB];
  u32x4 ra2[LONG_LOOP ? LA : 1], rb2[LONG_LOOP ? LB : 1], ra3[LONG_LOOP ? LA : 1], rb3[LONG_LOOP ? LB : 1];
  // operand bases of both pairs are read from the kernel arguments once, not per k-tile
  const long long lda0 = g.lda[0], lda1 = g.lda[1], ldb0 = g.ldb[0], ldb1 = g.ldb[1];
  const T* const Abase0 = (const T*)g.A[0] + (long long)m0 * lda0 + (long long)(tid / NCH) * lda0 + (tid % NCH) * EPC;
  const T* const Abase1 = (const T*)g.A[1] + (long long)m0 * lda1 + (long long)(tid / NCH) * lda1 + (tid % NCH) * EPC;
  const T* const Bbase0 = (const T*)g.B[0] + (long long)n0 * ldb0 + (long long)(tid / NCH) * ldb0 + (tid % NCH) * EPC;
  const T* const Bbase1 = (const T*)g.B[1] + (long long)n0 * ldb1 + (long long)(tid / NCH) * ldb1 + (tid % NCH) * EPC;
#define BETTY_GLOAD(RA_, RB_, t_)                                                                    \
  {                                                                                                  \
    const bool second_ = (t_) >= T0;                                                                 \
    const int tt_ = second_ ? (t_) - T0 : (t_);                                                      \
    const T* Ab_ = (second_ ? Abase1 : Abase0) + (long long)tt_ * KT;                                \
    const T* Bb_ = (second_ ? Bbase1 : Bbase0) + (long long)tt_ * KT;                                \
    const long long lda_ = (second_ ? lda1 : lda0) * (GT / NCH);                                    \
    const long long ldb_ = (second_ ? ldb1 : ldb0) * (GT / NCH);                                    \
    _Pragma("unroll") for (int i_ = 0; i_ < LA; ++i_) RA_[i_] = *(const u32x4*)(Ab_ + i_ * lda_);    \
    _Pragma("unroll") for (int i_ = 0; i_ < LB; ++i_) RB_[i_] = *(const u32x4*)(Bb_ + i_ * ldb_);    \
  }
  // one k-tile: registers -> LDS, refill the registers dist_ tiles ahead (always_, or if that tile
  // exists), multiply.  Every thread of the workgroup passes both barriers whether or not its group
  // still has a tile (t_ < te).
#define BETTY_STAGE(RA_, RB_, t_, first_, always_, dist_, buf_)                                      \
  {                                                                                                  \
    const bool live_ = KG == 1 || (t_) < te;                                                         \
    u32x4* const sA_ = sA + (DB ? (buf_) * LBUF : 0);                                                \
    u32x4* const sB_ = sB + (DB ? (buf_) * LBUF : 0);                                                \
    if (!DB && !(first_)) BETTY_GROUP_SYNC();                                                        \
    if (live_) {                                                                                     \
      _Pragma("unroll") for (int i_ = 0; i_ < LA; ++i_) {                                            \
        const int idx_ = tid + i_ * GT;                                                              \
        sA_[(idx_ / NCH) * ROW + idx_ % NCH] = RA_[i_];                                              \
      }                                                                                              \
      _Pragma("unroll") for (int i_ = 0; i_ < LB; ++i_) {                                            \
        const int idx_ = tid + i_ * GT;                                                              \
        sB_[(idx_ / NCH) * ROW + idx_ % NCH] = RB_[i_];                                              \
      }                                                                                              \
    }                                                                                                \
    BETTY_GROUP_SYNC();                                                                              \
    if ((always_) || (t_) + (dist_) < te) BETTY_GLOAD(RA_, RB_, (t_) + (dist_))                      \
    if (live_) {                                                                                     \
      _Pragma("unroll") for (int j_ = 0; j_ < NCH / 2; ++j_) {                                       \
        const int c_ = 2 * j_ + (lane >> 5);                                                         \
        u32x4 af_[TM], bf_[TN];                                                                      \
        _Pragma("unroll") for (int i_ = 0; i_ < TM; ++i_)                                            \
          af_[i_] = sA_[(wm * TM * 32 + i_ * 32 + (lane & 31)) * ROW + c_];                          \
        _Pragma("unroll") for (int i_ = 0; i_ < TN; ++i_)                                            \
          bf_[i_] = sB_[(wn * TN * 32 + i_ * 32 + (lane & 31)) * ROW + c_];                          \
        _Pragma("unroll") for (int i_ = 0; i_ < TM; ++i_)                                            \
          _Pragma("unroll") for (int jn_ = 0; jn_ < TN; ++jn_)                                       \
            MfmaChunk<T>::run(af_[i_], bf_[jn_], acc[i_ * TN + jn_]);                                \
      }                                                                                              \
    }                                                                                                \
  }

  const int n_full = te - tb;                       // tiles this group really has (<= NI)
  // Long-loop form, for unsplit activation-shaped launches with at least eight k-tiles.  What
  // counts for them is how many k-tiles are really in flight.  The compiler decides how long a
  // wavefront waits before it stores a register set to LDS from what it can prove about the loads
  // in flight, and where control flow merges it assumes the worst of the incoming paths: a refill
  // inside a branch, or a loop that can be entered with other loads in flight than its back edge
  // carries, makes every stage wait for all outstanding loads, i.e. for the tile requested one
  // stage ago, the full memory latency every other stage (512 x 4096 x 8192: 74 us).  Here the loop
  // is entered through straight-line code that leaves exactly the loop's own state, refills
  // unconditionally, and keeps four register sets, so a stage waits for the oldest set only while
  // three k-tiles stay in flight (66 us; 39 us for half the rows, which took 70 us before;
  // 8192 x 8192 x 4096 on 128-tiles 803 -> 695 us).
  bool done = false;
  if constexpr (LONG_LOOP) {
    if (n_full >= 8) {
      BETTY_GLOAD(ra0, rb0, tb)
      BETTY_GLOAD(ra1, rb1, tb + 1)
      BETTY_GLOAD(ra2, rb2, tb + 2)
      BETTY_GLOAD(ra3, rb3, tb + 3)
      int it = 0;
      for (; it + 7 < n_full; it += 4) {
        BETTY_STAGE(ra0, rb0, tb + it, false, true, 4, 0)
        BETTY_STAGE(ra1, rb1, tb + it + 1, false, true, 4, 1)
        BETTY_STAGE(ra2, rb2, tb + it + 2, false, true, 4, 0)
        BETTY_STAGE(ra3, rb3, tb + it + 3, false, true, 4, 1)
      }
      for (; it < n_full; it += 4) {                // the last four to seven tiles
        BETTY_STAGE(ra0, rb0, tb + it, false, false, 4, 0)
        if (it + 1 < n_full) BETTY_STAGE(ra1, rb1, tb + it + 1, false, false, 4, 1)
        if (it + 2 < n_full) BETTY_STAGE(ra2, rb2, tb + it + 2, false, false, 4, 0)
        if (it + 3 < n_full) BETTY_STAGE(ra3, rb3, tb + it + 3, false, false, 4, 1)
      }
      done = true;
    }
  }
  if (!done) {
    if (tb < te) BETTY_GLOAD(ra0, rb0, tb)
    if (tb + 1 < te) BETTY_GLOAD(ra1, rb1, tb + 1)
    // Unsplit launches (KG == 1) have long k loops: steady state while both refills of an iteration
    // stay inside the k-range, then a short tail.  K-split launches run a handful of tiles per
    // group; they keep the compact loop (less code to fetch for a kernel that lives a few us).
    int it = 0;
    if constexpr (KG == 1) {
      if (n_full > 3) {                               // first pair peeled: no barrier before the first store
        BETTY_STAGE(ra0, rb0, tb, true, true, 2, 0)
        BETTY_STAGE(ra1, rb1, tb + 1, false, true, 2, 1)
        it = 2;
      }
      for (; it + 3 < n_full; it += 2) {
        BETTY_STAGE(ra0, rb0, tb + it, false, true, 2, 0)
        BETTY_STAGE(ra1, rb1, tb + it + 1, false, true, 2, 1)
      }
    }
    for (; it < NI; it += 2) {
      BETTY_STAGE(ra0, rb0, tb + it, it == 0, false, 2, 0)
      if (it + 1 < NI) BETTY_STAGE(ra1, rb1, tb + it + 1, false, false, 2, 1)
    }
  }
#undef BETTY_STAGE
#undef BETTY_GLOAD
#undef BETTY_GROUP_SYNC

  // ---- combine the K groups through LDS in group order (bit-reproducible); group 0 finishes
  if constexpr (SPLIT_EPI) {
    __syncthreads();                                // all groups are done with the operand tiles
    float* red = (float*)smem;
#pragma unroll
    for (int r = 0; r < 16; ++r) red[(kg * 16 + r) * 64 + lane] = acc[0][r];
    __syncthreads();
    if (kg >= 4) return;
    float q4[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) q4[r] = red[(4 * kg + r) * 64 + lane];
#pragma unroll 1
    for (int g2 = 1; g2 < KG; ++g2) {
#pragma unroll
      for (int r = 0; r < 4; ++r) q4[r] += red[((g2 * 16) + 4 * kg + r) * 64 + lane];
    }
    epi_finish<T, MODE, 4>(e, g.M, g.N, m0 + 8 * kg + 4 * (lane >> 5), n0 + (lane & 31), q4, pre4);
    return;
  } else if constexpr (KG > 1) {
    __syncthreads();                                // all groups are done with the operand tiles
    float* red = (float*)smem;
    if (kg > 0) {
#pragma unroll
      for (int i = 0; i < TM * TN; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) red[(((kg - 1) * TM * TN + i) * 16 + r) * GT + tid] = acc[i][r];
    }
    __syncthreads();
    if (kg > 0) return;
#pragma unroll 1
    for (int g2 = 1; g2 < KG; ++g2) {
#pragma unroll
      for (int i = 0; i < TM * TN; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] += red[(((g2 - 1) * TM * TN + i) * 16 + r) * GT + tid];
    }
  }

  // ---- epilogue from registers, one MFMA block at a time
#pragma unroll
  for (int ij = 0; ij < TM * TN; ++ij) {
    const int rb = m0 + wm * TM * 32 + (ij / TN) * 32 + 4 * (lane >> 5);
    const int col = n0 + wn * TN * 32 + (ij % TN) * 32 + (lane & 31);
    if (!PREFETCH || !early) epi_prefetch<MODE, 16>(e, g.M, g.N, rb, col, pre[ij]);
    float accf[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) accf[r] = acc[ij][r];
    epi_finish<T, MODE, 16>(e, g.M, g.N, rb, col, accf, pre[ij]);
  }
}

// ------------------------------------------------------------------------------------------
// weight-gradient launches of large layers (bf16 operands): 128 x 128 tiles, epilogue through LDS
// ------------------------------------------------------------------------------------------
//
// For a layer with millions of parameters the parameter-shaped epilogue (two or more fp32 vectors
// in, one out, two operand copies out) moves more bytes than the k loop, and with 64-tiles the
// operand panels cross the L2 -> L1 path twice as often.  This kernel keeps the k loop of
// gemm_fused_kernel at 128 x 128 but finishes the tile differently: the accumulators go to LDS once,
// then the tile is worked off in four passes of 32 rows in which a thread owns a 4 x 4 patch, so
// that every access to the flat fp32 vectors is a 16-byte access and eight neighbouring lanes
// cover a whole 128-byte line.  The inputs of pass p + 1 are requested before pass p is computed
// (those of pass 0 before the last two k-tiles are multiplied), and the transposed operand copy
// leaves through a small LDS staging tile as 16-byte rows.  Two workgroups fit a compute unit, so
// one streams its epilogue while the other multiplies.

template <int MODE, bool LAM> constexpr int wg_narr() {
  return MODE == EPI_WGRAD ? (LAM ? 2 : 0) : MODE == EPI_WGRAD_INIT ? 0 : MODE == EPI_WGRAD_NEUMANN ? (LAM ? 3 : 2)
       : MODE == EPI_WGRAD_SGD ? (LAM ? 4 : 2) : 4;
}
template <int MODE, bool LAM> constexpr int wg_nreg() { return wg_narr<MODE, LAM>() > 0 ? wg_narr<MODE, LAM>() : 1; }

constexpr int WG_BT = 128;                 // tile extent
constexpr int WG_HP = WG_BT + 8;           // pitch of the fp32 accumulator tile in LDS (floats)
constexpr int WG_PASS = 32;                // rows per epilogue pass
constexpr int WG_TP = WG_PASS + 8;         // pitch of the transposed staging tile (elements)
constexpr size_t WG_LDS_OPERANDS = (size_t)2 * 2 * WG_BT * (GEMM_NCH + 1) * 16;
constexpr size_t WG_LDS_EPILOGUE = (size_t)WG_BT * WG_HP * 4 + (size_t)WG_BT * WG_TP * 2;
constexpr size_t WG_LDS = WG_LDS_OPERANDS > WG_LDS_EPILOGUE ? WG_LDS_OPERANDS : WG_LDS_EPILOGUE;

// what a workgroup needs of its problem's epilogue, read from the kernel arguments once
struct WgTile {
  const float* src[4];                     // fp32 inputs in the order the mode consumes them
  float* C; float* v; float* p;
  __bf16* out; __bf16* outT;
  long long ldc; int ld, ldT;
  int M, N, m0, n0;
  float alpha, beta, gamma;
  bool has_x;
};

// The flat fp32 vectors of a layer this large are streamed once per launch and come round again
// only after gigabytes of other traffic: their 16-byte accesses carry the non-temporal hint
// (121M-parameter model +3 %; the same hint on the operand copies, which the next launches read,
// loses 0.3 %).
typedef float f32x4v __attribute__((ext_vector_type(4)));

// Rows and columns are clamped into the valid extent instead of being predicated, so the loads of
// all arrays of a patch are in flight together (a load inside control flow makes the compiler wait
// for the earlier ones first).  VEC: 16-byte accesses, whole patch inside the column extent.
template <bool VEC>
__device__ __forceinline__ void load_patch(const float* __restrict__ p, long long ld, int row0, int col0, int M, int N,
                                           float (&r)[4][4]) {
  if constexpr (VEC) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const f32x4v t = __builtin_nontemporal_load((const f32x4v*)(p + (long long)min(row0 + i, M - 1) * ld + col0));
      r[i][0] = t.x; r[i][1] = t.y; r[i][2] = t.z; r[i][3] = t.w;
    }
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) r[i][j] = p[(long long)min(row0 + i, M - 1) * ld + min(col0 + j, N - 1)];
  }
}

template <bool VEC>
__device__ __forceinline__ void store_patch(float* __restrict__ p, long long ld, int row0, int col0, int M, int N,
                                            const float (&r)[4][4]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (row0 + i >= M) continue;
    float* q = p + (long long)(row0 + i) * ld + col0;
    if constexpr (VEC) {
      const f32x4v o4 = {r[i][0], r[i][1], r[i][2], r[i][3]};
      __builtin_nontemporal_store(o4, (f32x4v*)q);
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (col0 + j < N) q[j] = r[i][j];
    }
  }
}

template <int MODE, bool LAM, bool VEC>
__device__ __forceinline__ void wg_request(const WgTile& w, int pass, int pr, int pc, float (&in)[wg_nreg<MODE, LAM>()][4][4]) {
  constexpr int NARR = wg_narr<MODE, LAM>();
  const int row0 = w.m0 + WG_PASS * pass + 4 * pr, col0 = w.n0 + 4 * pc;
#pragma unroll
  for (int k = 0; k < NARR; ++k) load_patch<VEC>(w.src[k], w.ldc, row0, col0, w.M, w.N, in[k]);
}

// one pass of 32 rows: accumulators from LDS, the mode's update rule, stores.  Every thread of the
// workgroup calls it (it contains barriers when the transposed copy is asked for).
template <int MODE, bool LAM, bool VEC>
__device__ __forceinline__ void wg_finish(const WgTile& w, int pass, int pr, int pc, int tid, const float* hs, __bf16* sT,
                                          const float (&in)[wg_nreg<MODE, LAM>()][4][4]) {
  constexpr int NR = wg_nreg<MODE, LAM>();
  const int row0 = w.m0 + WG_PASS * pass + 4 * pr, col0 = w.n0 + 4 * pc;
  float acc[4][4], val[4][4], val2[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float4 h4 = *(const float4*)(hs + (WG_PASS * pass + 4 * pr + i) * WG_HP + 4 * pc);
    acc[i][0] = h4.x; acc[i][1] = h4.y; acc[i][2] = h4.z; acc[i][3] = h4.w;
  }
  const float (&I0)[4][4] = in[0];
  const float (&I1)[4][4] = in[NR > 1 ? 1 : 0];
  const float (&I2)[4][4] = in[NR > 2 ? 2 : 0];
  const float (&I3)[4][4] = in[NR > 3 ? 3 : 0];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float a = acc[i][j];
      if constexpr (MODE == EPI_WGRAD) {                   // I0 = lam, I1 = x
        val[i][j] = LAM ? a + 2.f * expf(I0[i][j]) * I1[i][j] : a;
      } else if constexpr (MODE == EPI_WGRAD_INIT) {
        val[i][j] = a;
      } else if constexpr (MODE == EPI_WGRAD_NEUMANN) {    // I0 = s, I1 = g, I2 = lam
        float h = a;
        if constexpr (LAM) h += 2.f * expf(I2[i][j]) * I0[i][j];
        val[i][j] = I1[i][j] + (I0[i][j] - w.alpha * h);
      } else if constexpr (MODE == EPI_WGRAD_NEUMANN_L2) { // I0 = s, I1 = g, I2 = lam, I3 = w
        const float el = 2.f * expf(I2[i][j]);
        const float sn = I1[i][j] + (I0[i][j] - w.alpha * (a + el * I0[i][j]));
        val[i][j] = -el * I3[i][j] * (w.alpha * sn);
      } else {                                             // SGD: I0 = momentum, I1 = w, I2 = lam, I3 = anchor
        float gk = a + w.gamma * I1[i][j];
        if constexpr (LAM) gk += 2.f * expf(I2[i][j]) * (I1[i][j] - (w.has_x ? I3[i][j] : 0.f));
        const float mk = w.beta * I0[i][j] + gk;
        val[i][j] = mk;
        val2[i][j] = I1[i][j] - w.alpha * mk;
      }
    }
  if constexpr (MODE == EPI_WGRAD || MODE == EPI_WGRAD_NEUMANN_L2) {
    store_patch<VEC>(w.C, w.ldc, row0, col0, w.M, w.N, val);
    return;
  } else if constexpr (MODE == EPI_WGRAD_SGD) {
    store_patch<VEC>(w.v, w.ldc, row0, col0, w.M, w.N, val);
    store_patch<VEC>(w.p, w.ldc, row0, col0, w.M, w.N, val2);
    return;
  } else {
    if constexpr (MODE == EPI_WGRAD_INIT) {
      store_patch<VEC>(w.v, w.ldc, row0, col0, w.M, w.N, val);
      if (w.p) store_patch<VEC>(w.p, w.ldc, row0, col0, w.M, w.N, val);
    } else {
      store_patch<VEC>(w.p, w.ldc, row0, col0, w.M, w.N, val);
    }
    // operand copies of the new vector: row-major [row][col] and transposed [col][row]; rows beyond
    // M inside a stored group are padding of the operand and are written as zeros
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (row0 + i >= w.M) {
#pragma unroll
        for (int j = 0; j < 4; ++j) val[i][j] = 0.f;
      }
    if (w.out) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (row0 + i >= w.M) continue;
        __bf16* o = w.out + (long long)(row0 + i) * w.ld + col0;
        if constexpr (VEC) {
          store4<__bf16>(o, val[i]);
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j)
            if (col0 + j < w.N) o[j] = (__bf16)val[i][j];
        }
      }
    }
    if (w.outT) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float quad[4] = {val[0][j], val[1][j], val[2][j], val[3][j]};
        store4<__bf16>(sT + (4 * pc + j) * WG_TP + 4 * pr, quad);
      }
      __syncthreads();
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int q = tid + 256 * u, c = q >> 2, k = q & 3;
        const int row = w.m0 + WG_PASS * pass + 8 * k;
        if (w.n0 + c < w.N && row < w.M)
          *(u32x4*)(w.outT + (long long)(w.n0 + c) * w.ldT + row) = *(const u32x4*)(sT + c * WG_TP + 8 * k);
      }
      __syncthreads();
    }
  }
}

// How many passes ahead the epilogue inputs are requested (the ring of register sets below holds
// one more).  Requesting the whole tile ahead (3, affordable with two input arrays) was measured
// slower than one pass ahead on the 121M-parameter model: 620 against 576 us per launch.  The final
// step of the series (four input arrays, once per hypergradient) requests each pass as it gets
// to it: a second register set would not fit beside the tile walk's state.
template <int MODE, bool LAM> constexpr int wg_depth() { return MODE == EPI_WGRAD_NEUMANN_L2 ? 0 : 1; }
constexpr int WG_NPASS = WG_BT / WG_PASS;

template <int MODE, bool LAM, bool VEC>
__device__ __forceinline__ void wg_epilogue(const WgTile& w, int pr, int pc, int tid, const float* hs, __bf16* sT,
                                            float (&in)[wg_depth<MODE, LAM>() + 1][wg_nreg<MODE, LAM>()][4][4]) {
  constexpr int DEPTH = wg_depth<MODE, LAM>(), EARLY = DEPTH < 2 ? DEPTH : 2;
  // (with 16-byte accesses the first EARLY passes were requested inside the k loop)
#pragma unroll
  for (int q = VEC ? EARLY : 0; q < DEPTH; ++q) wg_request<MODE, LAM, VEC>(w, q, pr, pc, in[q]);
#pragma unroll
  for (int pass = 0; pass < WG_NPASS; ++pass) {
    if (pass + DEPTH < WG_NPASS) wg_request<MODE, LAM, VEC>(w, pass + DEPTH, pr, pc, in[(pass + DEPTH) % (DEPTH + 1)]);
    wg_finish<MODE, LAM, VEC>(w, pass, pr, pc, tid, hs, sT, in[pass % (DEPTH + 1)]);
  }
}

template <int MODE, bool LAM>
__global__ __launch_bounds__(256, 2) void wgrad128_kernel(GemmBatch batch) {
  typedef __bf16 T;
  constexpr int BT = WG_BT, NCH = GEMM_NCH, ROW = NCH + 1, EPC = 8, KT = NCH * EPC, GT = 256;
  constexpr int LA = BT * NCH / GT;
  constexpr int LBUF = 2 * BT * ROW;
  extern __shared__ u32x4 smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;

  // The first batch.walkers workgroups (two per compute unit) walk the tiles (tile = blockIdx.x,
  // then + walkers, ...) instead of one workgroup starting per tile, and where registers allow
  // request the first two k-tiles of their next tile before they finish the current one
  // (121M-parameter model: first weight-gradient launch 389 -> 370 us, Neumann launches 547 -> 536 us).
  // The bias rows follow in workgroups of their own.
  const int P = batch.walkers;
  if ((int)blockIdx.x >= P) {
    const int bid = blockIdx.x - P;
    int j = 0;
    while (j + 1 < batch.n_bias && bid >= batch.bias_begin[j + 1]) ++j;
    bias_rows<T, MODE>(batch.bias[j], (bid - batch.bias_begin[j]) * 4 + (threadIdx.x >> 6));
    return;
  }
  // patch of this thread inside an epilogue pass: eight lanes side by side cover 32 columns of four rows
  const int pc = 8 * wave + (lane & 7), pr = lane >> 3;

  // position and operands of a tile
  int pi, m0, n0, T0, TT;
  long long lda0, lda1, ldb0, ldb1;
  const T *Abase0, *Abase1, *Bbase0, *Bbase1;
#define BETTY_WG_LOCATE(tile_)                                                                       \
  {                                                                                                  \
    pi = 0;                                                                                          \
    while (pi + 1 < batch.n && (tile_) >= batch.block_begin[pi + 1]) ++pi;                           \
    const GemmArgs& g_ = batch.p[pi].g;                                                              \
    const int t_ = (tile_) - batch.block_begin[pi];                                                  \
    const int tiles_n_ = g_.Np / BT;                                                                 \
    int tm_ = t_ / tiles_n_, tn_ = t_ % tiles_n_;                                                    \
    if (g_.xgm > 0) {                                 /* XCD-compact order (see GemmArgs) */         \
      const int x_ = t_ & 7, q_ = t_ >> 3;                                                           \
      const int rm_ = (g_.Mp / BT) / g_.xgm, rn_ = tiles_n_ / g_.xgn;                                \
      tm_ = (x_ / g_.xgn) * rm_ + q_ / rn_;                                                          \
      tn_ = (x_ % g_.xgn) * rn_ + q_ % rn_;                                                          \
    }                                                                                                \
    m0 = tm_ * BT; n0 = tn_ * BT;                                                                    \
    T0 = g_.Kp[0] / KT; TT = T0 + g_.Kp[1] / KT;     /* an even number of k-tiles (operands are padded to 128) */ \
    lda0 = g_.lda[0]; lda1 = g_.lda[1]; ldb0 = g_.ldb[0]; ldb1 = g_.ldb[1];                          \
    Abase0 = (const T*)g_.A[0] + (long long)(m0 + tid / NCH) * lda0 + (tid % NCH) * EPC;             \
    Abase1 = (const T*)g_.A[1] + (long long)(m0 + tid / NCH) * lda1 + (tid % NCH) * EPC;             \
    Bbase0 = (const T*)g_.B[0] + (long long)(n0 + tid / NCH) * ldb0 + (tid % NCH) * EPC;             \
    Bbase1 = (const T*)g_.B[1] + (long long)(n0 + tid / NCH) * ldb1 + (tid % NCH) * EPC;             \
  }
  u32x4 ra0[LA], rb0[LA], ra1[LA], rb1[LA];
#define BETTY_WG_GLOAD(RA_, RB_, t_)                                                                 \
  {                                                                                                  \
    const bool second_ = (t_) >= T0;                                                                 \
    const int tt_ = second_ ? (t_) - T0 : (t_);                                                      \
    const T* Ab_ = (second_ ? Abase1 : Abase0) + (long long)tt_ * KT;                                \
    const T* Bb_ = (second_ ? Bbase1 : Bbase0) + (long long)tt_ * KT;                                \
    const long long lda_ = (second_ ? lda1 : lda0) * (GT / NCH);                                    \
    const long long ldb_ = (second_ ? ldb1 : ldb0) * (GT / NCH);                                    \
    _Pragma("unroll") for (int i_ = 0; i_ < LA; ++i_) RA_[i_] = *(const u32x4*)(Ab_ + i_ * lda_);    \
    _Pragma("unroll") for (int i_ = 0; i_ < LA; ++i_) RB_[i_] = *(const u32x4*)(Bb_ + i_ * ldb_);    \
  }
  // one k-tile: registers -> LDS buffer buf_, (refill the registers two tiles ahead), multiply.
  // Two buffers alternate, so a k-tile costs one barrier.
#define BETTY_WG_STAGE(RA_, RB_, t_, refill_, buf_)                                                  \
  {                                                                                                  \
    u32x4* const sA_ = smem + (buf_) * LBUF;                                                         \
    u32x4* const sB_ = sA_ + BT * ROW;                                                               \
    _Pragma("unroll") for (int i_ = 0; i_ < LA; ++i_) {                                              \
      const int idx_ = tid + i_ * GT;                                                                \
      sA_[(idx_ / NCH) * ROW + idx_ % NCH] = RA_[i_];                                                \
      sB_[(idx_ / NCH) * ROW + idx_ % NCH] = RB_[i_];                                                \
    }                                                                                                \
    __syncthreads();                                                                                 \
    if (refill_) BETTY_WG_GLOAD(RA_, RB_, (t_) + 2)                                                  \
    _Pragma("unroll") for (int j_ = 0; j_ < NCH / 2; ++j_) {                                         \
      const int c_ = 2 * j_ + (lane >> 5);                                                           \
      u32x4 af_[2], bf_[2];                                                                          \
      _Pragma("unroll") for (int i_ = 0; i_ < 2; ++i_) {                                             \
        af_[i_] = sA_[(wm * 64 + i_ * 32 + (lane & 31)) * ROW + c_];                                 \
        bf_[i_] = sB_[(wn * 64 + i_ * 32 + (lane & 31)) * ROW + c_];                                 \
      }                                                                                              \
      _Pragma("unroll") for (int i_ = 0; i_ < 2; ++i_)                                               \
        _Pragma("unroll") for (int jn_ = 0; jn_ < 2; ++jn_)                                          \
          MfmaChunk<T>::run(af_[i_], bf_[jn_], acc[i_ * 2 + jn_]);                                   \
    }                                                                                                \
  }

  float* const hs = (float*)smem;
  __bf16* const sT = (__bf16*)(hs + BT * WG_HP);
  int tile = blockIdx.x;
  BETTY_WG_LOCATE(tile)
  BETTY_WG_GLOAD(ra0, rb0, 0)
  BETTY_WG_GLOAD(ra1, rb1, 1)
  for (;;) {
    // here the first two k-tiles of `tile` are in flight and pi, m0, n0, TT, the bases describe it
    const Epilogue& e = batch.p[pi].e;
    WgTile w;
    w.C = e.C; w.v = e.v; w.p = e.p; w.out = (T*)e.out; w.outT = (T*)e.outT;
    w.ldc = e.ldc; w.ld = e.ld; w.ldT = e.ldT;
    w.M = batch.p[pi].g.M; w.N = batch.p[pi].g.N; w.m0 = m0; w.n0 = n0;
    w.alpha = e.alpha; w.beta = e.beta; w.gamma = e.gamma;
    w.has_x = e.x != nullptr;
    if constexpr (MODE == EPI_WGRAD) { w.src[0] = e.lam; w.src[1] = e.x; w.src[2] = e.lam; w.src[3] = e.lam; }
    else if constexpr (MODE == EPI_WGRAD_NEUMANN) { w.src[0] = e.x; w.src[1] = e.v; w.src[2] = e.lam; w.src[3] = e.x; }
    else if constexpr (MODE == EPI_WGRAD_NEUMANN_L2) { w.src[0] = e.p; w.src[1] = e.v; w.src[2] = e.lam; w.src[3] = e.x; }
    else if constexpr (MODE == EPI_WGRAD_SGD) { w.src[0] = e.v; w.src[1] = e.p; w.src[2] = e.lam; w.src[3] = e.x ? e.x : e.p; }
    else { w.src[0] = w.src[1] = w.src[2] = w.src[3] = nullptr; }
    // 16-byte accesses need every flat vector of the tile aligned and the tile inside the columns
    unsigned long long bits = (unsigned long long)w.C | (unsigned long long)w.v | (unsigned long long)w.p;
#pragma unroll
    for (int k = 0; k < wg_narr<MODE, LAM>(); ++k) bits |= (unsigned long long)w.src[k];
    const bool vec = (bits & 15) == 0 && (w.ldc & 3) == 0 && n0 + BT <= w.N;

    f32x16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;

    int it = 0;
    for (; it + 2 < TT; it += 2) {
      BETTY_WG_STAGE(ra0, rb0, it, true, 0)
      BETTY_WG_STAGE(ra1, rb1, it + 1, true, 1)
    }
    // every operand load is issued: request the inputs of the first epilogue pass behind them
    float in[wg_depth<MODE, LAM>() + 1][wg_nreg<MODE, LAM>()][4][4];
    if (vec) {
#pragma unroll
      for (int q = 0; q < (wg_depth<MODE, LAM>() < 2 ? wg_depth<MODE, LAM>() : 2); ++q) wg_request<MODE, LAM, true>(w, q, pr, pc, in[q]);
    }
    BETTY_WG_STAGE(ra0, rb0, it, false, 0)
    BETTY_WG_STAGE(ra1, rb1, it + 1, false, 1)

    // accumulators -> LDS (the operand buffers are dead): register r of lane l of block (i, j) is
    // element [64 wm + 32 i + 8 (r / 4) + 4 (l / 32) + r % 4][64 wn + 32 j + l % 32]
    __syncthreads();
#pragma unroll
    for (int ij = 0; ij < 4; ++ij)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        hs[(wm * 64 + (ij >> 1) * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3)) * WG_HP + wn * 64 + (ij & 1) * 32 + (lane & 31)] = acc[ij][r];
    __syncthreads();

    // the next tile's first two k-tiles, requested ahead of this tile's epilogue (after the last
    // tile the same tile once more: no branch around the loads, see gemm_fused_kernel's long loop)
    // (only in the modes whose epilogue reads nothing: with epilogue inputs in flight as well the
    // request ahead gains nothing measurable, and with three or four input arrays there are no
    // registers for it)
    constexpr bool AHEAD = wg_narr<MODE, LAM>() == 0;
    const int next = tile + P;
    const bool more = next < batch.gemm_blocks;
    if constexpr (AHEAD) {
      BETTY_WG_LOCATE(more ? next : tile)
      BETTY_WG_GLOAD(ra0, rb0, 0)
      BETTY_WG_GLOAD(ra1, rb1, 1)
    }
    if (vec) wg_epilogue<MODE, LAM, true>(w, pr, pc, tid, hs, sT, in);
    else wg_epilogue<MODE, LAM, false>(w, pr, pc, tid, hs, sT, in);
    if (!more) break;
    __syncthreads();                                // the next k loop writes where this epilogue read
    tile = next;
    if constexpr (!AHEAD) {
      BETTY_WG_LOCATE(tile)
      BETTY_WG_GLOAD(ra0, rb0, 0)
      BETTY_WG_GLOAD(ra1, rb1, 1)
    }
  }
#undef BETTY_WG_STAGE
#undef BETTY_WG_GLOAD
#undef BETTY_WG_LOCATE
}

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------

template <typename T, int BT, int WPG, int KG>
constexpr size_t lds_bytes() {
  constexpr size_t operands = (size_t)(KG == 1 ? 2 : KG) * 2 * BT * (GEMM_NCH + 1) * 16;
  constexpr size_t reduce = (size_t)(WPG == 1 ? KG : KG - 1) * BT * BT * 4;
  return operands > reduce ? operands : reduce;
}

template <typename T, int BT, int WPG, int KG, int MODE>
static void launch_one(int total, hipStream_t st, const GemmBatch& b, hipError_t& err) {
  constexpr size_t lds = lds_bytes<T, BT, WPG, KG>();
  static bool configured = false;
  if (!configured) {
    if (lds > 48 * 1024) {
      hipError_t e = hipFuncSetAttribute((const void*)gemm_fused_kernel<T, BT, BT, GEMM_NCH, WPG, KG, MODE>,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (e != hipSuccess) { err = e; return; }
    }
    configured = true;
  }
  gemm_fused_kernel<T, BT, BT, GEMM_NCH, WPG, KG, MODE><<<total, 64 * WPG * KG, lds, st>>>(b);
}

// 128 x 64 tiles, unsplit, eight wavefronts with one MFMA block each (a launch of these tiles puts
// one workgroup on a compute unit, and two wavefronts per SIMD hide each other's barrier and LDS
// waits: 121M-parameter model +2.3 % over four wavefronts of two blocks): the activation-shaped
// products of a grid that would otherwise leave one to four 64-tiles per compute unit
template <typename T, int MODE>
static void launch_rect(int total, hipStream_t st, const GemmBatch& b, hipError_t& err) {
  constexpr size_t lds = (size_t)2 * (128 + 64) * (GEMM_NCH + 1) * 16;
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void*)gemm_fused_kernel<T, 128, 64, GEMM_NCH, 8, 1, MODE>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) { err = e; return; }
    configured = true;
  }
  gemm_fused_kernel<T, 128, 64, GEMM_NCH, 8, 1, MODE><<<total, 512, lds, st>>>(b);
}

template <typename T>
static void launch_rect_mode(int mode, int total, hipStream_t st, const GemmBatch& b, hipError_t& err) {
  switch (mode) {
#define BETTY_CASE_R(M_) case M_: launch_rect<T, M_>(total, st, b, err); break;
    BETTY_CASE_R(EPI_FWD) BETTY_CASE_R(EPI_FWD_LAST) BETTY_CASE_R(EPI_BWD) BETTY_CASE_R(EPI_RFWD)
    BETTY_CASE_R(EPI_RFWD_LAST) BETTY_CASE_R(EPI_RBWD) BETTY_CASE_R(EPI_RFWD_LAST_HESS)
#undef BETTY_CASE_R
    default: err = hipErrorInvalidValue; break;
  }
}

template <typename T, int BT, int WPG, int KG>
static void launch_chain_mode(int mode, int total, hipStream_t st, const GemmBatch& b, hipError_t& err) {
  switch (mode) {
#define BETTY_CASE(M_) case M_: launch_one<T, BT, WPG, KG, M_>(total, st, b, err); break;
    BETTY_CASE(EPI_FWD) BETTY_CASE(EPI_FWD_LAST) BETTY_CASE(EPI_BWD) BETTY_CASE(EPI_RFWD)
    BETTY_CASE(EPI_RFWD_LAST) BETTY_CASE(EPI_RBWD) BETTY_CASE(EPI_RFWD_LAST_HESS)
    default: err = hipErrorInvalidValue; break;
  }
}

template <typename T, int BT>
static void launch_wgrad_mode(int mode, int total, hipStream_t st, const GemmBatch& b, hipError_t& err) {
  switch (mode) {
#define BETTY_CASE_W(M_) case M_: launch_one<T, BT, 4, 1, M_>(total, st, b, err); break;
    BETTY_CASE_W(EPI_WGRAD) BETTY_CASE_W(EPI_WGRAD_INIT) BETTY_CASE_W(EPI_WGRAD_NEUMANN)
    BETTY_CASE_W(EPI_WGRAD_NEUMANN_L2) BETTY_CASE_W(EPI_WGRAD_SGD)
#undef BETTY_CASE_W
    default: err = hipErrorInvalidValue; break;
  }
}
#undef BETTY_CASE

template <int MODE, bool LAM>
static void launch_wgrad128_one(int total, hipStream_t st, const GemmBatch& b, hipError_t& err) {
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void*)wgrad128_kernel<MODE, LAM>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)WG_LDS);
    if (e != hipSuccess) { err = e; return; }
    configured = true;
  }
  wgrad128_kernel<MODE, LAM><<<total - b.gemm_blocks + b.walkers, 256, WG_LDS, st>>>(b);
}

// bf16 weight-gradient launches on 128-tiles; the L2-decay term (lam) is the same for every problem of a batch
static void launch_wgrad128(int mode, int total, hipStream_t st, const GemmBatch& b, hipError_t& err) {
  const bool lam = b.p[0].e.lam != nullptr;
  switch (mode) {
#define BETTY_CASE_W(M_) case M_: if (lam) launch_wgrad128_one<M_, true>(total, st, b, err); else launch_wgrad128_one<M_, false>(total, st, b, err); break;
    BETTY_CASE_W(EPI_WGRAD) BETTY_CASE_W(EPI_WGRAD_NEUMANN) BETTY_CASE_W(EPI_WGRAD_SGD)
#undef BETTY_CASE_W
    case EPI_WGRAD_INIT: launch_wgrad128_one<EPI_WGRAD_INIT, false>(total, st, b, err); break;
    case EPI_WGRAD_NEUMANN_L2: launch_wgrad128_one<EPI_WGRAD_NEUMANN_L2, true>(total, st, b, err); break;
    default: err = hipErrorInvalidValue; break;
  }
}

template <typename T>
static void launch_elem(int cfg, int mode, int total, hipStream_t st, const GemmBatch& b, hipError_t& err) {
  if (mode >= EPI_WGRAD) {
    if (cfg == GEMM_128x1 && sizeof(T) == 2) launch_wgrad128(mode, total, st, b, err);
    else if (cfg == GEMM_128x1) launch_wgrad_mode<T, 128>(mode, total, st, b, err);
    else if (cfg == GEMM_64x1) launch_wgrad_mode<T, 64>(mode, total, st, b, err);
    else err = hipErrorInvalidValue;
    return;
  }
  switch (cfg) {
    case GEMM_128x1: launch_chain_mode<T, 128, 4, 1>(mode, total, st, b, err); break;
    case GEMM_64x1: launch_chain_mode<T, 64, 4, 1>(mode, total, st, b, err); break;
    case GEMM_64x4: launch_chain_mode<T, 64, 4, 4>(mode, total, st, b, err); break;
    case GEMM_32x8: launch_chain_mode<T, 32, 1, 8>(mode, total, st, b, err); break;
    case GEMM_128x64: launch_rect_mode<T>(mode, total, st, b, err); break;
    default: err = hipErrorInvalidValue; break;
  }
}

// compute units of the current device (asked once; every device of a node is the same part)
static int resident_cus() {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
      cus = n;
    else { (void)hipGetLastError(); cus = 256; }
  }
  return cus;
}

int gemm_ktile_elems(Elem elem) { return GEMM_NCH * (elem == ELEM_BF16 ? 8 : 4); }
int gemm_cfg_tile(int cfg) { return cfg == GEMM_128x1 ? 128 : cfg == GEMM_32x8 ? 32 : 64; }   // (columns, for 128x64)
static int gemm_cfg_tile_rows(int cfg) { return cfg == GEMM_128x64 ? 128 : gemm_cfg_tile(cfg); }
static int gemm_cfg_waves(int cfg) { return cfg == GEMM_64x4 ? 16 : cfg == GEMM_32x8 ? 8 : 4; }

void launch_gemm_batch(Ctx& ctx, Elem elem, int cfg, GemmBatch& b, double flops, double bytes) {
  const int bt = gemm_cfg_tile(cfg);
  const int rows_per_block = gemm_cfg_waves(cfg);
  int blocks = 0;
  for (int i = 0; i < b.n; ++i) {
    b.block_begin[i] = blocks;
    blocks += (b.p[i].g.Mp / gemm_cfg_tile_rows(cfg)) * (b.p[i].g.Np / bt);
  }
  b.block_begin[b.n] = blocks;
  b.gemm_blocks = blocks;
  b.walkers = blocks < 2 * resident_cus() ? blocks : 2 * resident_cus();
  int bias_blocks = 0;
  for (int i = 0; i < b.n_bias; ++i) {
    b.bias_begin[i] = bias_blocks;
    bias_blocks += (b.bias[i].rows + rows_per_block - 1) / rows_per_block;
  }
  b.bias_begin[b.n_bias] = bias_blocks;
  const int total = blocks + bias_blocks;
  if (total <= 0) return;
  const int mode0 = b.p[0].e.mode;
  const int kind = mode0 == EPI_WGRAD_NEUMANN ? BETTY_K_GEMM_UPDATE
                 : mode0 == EPI_WGRAD_NEUMANN_L2 ? BETTY_K_GEMM_UPDATE_FINAL
                 : (mode0 == EPI_RFWD || mode0 == EPI_RFWD_LAST || mode0 == EPI_RFWD_LAST_HESS) ? BETTY_K_GEMM_RFWD
                 : mode0 == EPI_RBWD ? BETTY_K_GEMM_RBWD : BETTY_K_GEMM;
  Launch l(ctx, kind, flops, bytes);
  hipError_t err = hipSuccess;
  if (elem == ELEM_BF16) launch_elem<__bf16>(cfg, b.p[0].e.mode, total, ctx.stream, b, err);
  else launch_elem<float>(cfg, b.p[0].e.mode, total, ctx.stream, b, err);
  if (err != hipSuccess && ctx.first_error == hipSuccess) ctx.first_error = err;
}

}  // namespace betty

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
// flattened on blockIdx.x.  A problem may be split along K into S slices; the S workgroups of a
// tile write their accumulators to a partials buffer in register order, and the last one to
// arrive (an atomic ticket per tile, no spinning) re-reads all S slices in slice order - so the
// sum is bit-reproducible - and runs the epilogue.  The ticket is reset by that workgroup.
//
// Tiling: 256 threads (4 wavefronts, 2 x 2) own a BM x BN tile; a wavefront owns TM x TN MFMA
// blocks of 32 x 32.  K is consumed in tiles of NCH 16-byte chunks per row: global -> registers
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

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

template <typename T> struct MfmaChunk;

template <> struct MfmaChunk<__bf16> {
  static __device__ __forceinline__ void run(const uint4& a, const uint4& b, f32x16& acc) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b),
                                                  acc, 0, 0, 0);
  }
};

template <> struct MfmaChunk<float> {
  static __device__ __forceinline__ void run(const uint4& a, const uint4& b, f32x16& acc) {
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
  }
};

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

// One register quad: rows row0..row0+3 (row0 % 4 == 0) of column col.  M, N = valid extent.
template <typename T>
__device__ __forceinline__ void epilogue_quad(const Epilogue& e, int M, int N, int row0, int col,
                                              const float (&acc)[4]) {
  if (col >= N || row0 >= M) return;
  float val[4];
  bool dual = true;
  switch (e.mode) {
    case EPI_STORE: {
#pragma unroll
      for (int k = 0; k < 4; ++k)
        if (row0 + k < M) e.C[(long long)(row0 + k) * e.ldc + col] = acc[k];
      return;
    }
    case EPI_FWD: {
      const float b = e.colvec ? e.colvec[col] : 0.f;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        val[k] = 0.f;
        if (row0 + k < M) {
          const long long o = (long long)(row0 + k) * e.ldf + col;
          float a, d1, d2;
          act_eval(e.act, acc[k] + b, a, d1, d2);
          e.dphi_out[o] = d1;
          if (e.d2_out) e.d2_out[o] = d2;
          val[k] = a;
        }
      }
      break;
    }
    case EPI_FWD_LAST:
    case EPI_RFWD_LAST: {
      const float b = e.colvec ? e.colvec[col] : 0.f;
#pragma unroll
      for (int k = 0; k < 4; ++k)
        if (row0 + k < M) e.f0[(long long)(row0 + k) * e.ldf + col] = acc[k] + b;
      return;
    }
    case EPI_BWD: {
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        val[k] = 0.f;
        if (row0 + k < M) {
          const long long o = (long long)(row0 + k) * e.ldf + col;
          if (e.e_io) e.e_io[o] = acc[k] * e.e_io[o];
          val[k] = acc[k] * e.dphi[o];
        }
      }
      break;
    }
    case EPI_RFWD: {
      const float b = e.colvec ? e.colvec[col] : 0.f;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        val[k] = 0.f;
        if (row0 + k < M) {
          const long long o = (long long)(row0 + k) * e.ldf + col;
          const float rz = acc[k] + b;
          e.f0[o] = rz;
          val[k] = e.dphi[o] * rz;
        }
      }
      break;
    }
    case EPI_RBWD: {
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        val[k] = 0.f;
        if (row0 + k < M) {
          const long long o = (long long)(row0 + k) * e.ldf + col;
          float r = acc[k] * e.dphi[o];
          if (e.e) r += e.e[o] * e.Rz[o];
          val[k] = r;
        }
      }
      break;
    }
    case EPI_WGRAD: {             // C = acc (+ 2 e^lam x)
#pragma unroll
      for (int k = 0; k < 4; ++k)
        if (row0 + k < M) {
          const long long o = (long long)(row0 + k) * e.ldc + col;
          float gval = acc[k];
          if (e.lam) gval += 2.f * expf(e.lam[o]) * e.x[o];
          e.C[o] = gval;
        }
      return;
    }
    case EPI_WGRAD_INIT: {        // v = p = acc ; operand copies of v
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        val[k] = 0.f;
        if (row0 + k < M) {
          const long long o = (long long)(row0 + k) * e.ldc + col;
          e.v[o] = acc[k];
          e.p[o] = acc[k];
          val[k] = acc[k];
        }
      }
      dual = e.out != nullptr;
      break;
    }
    case EPI_WGRAD_NEUMANN: {     // Hv = acc (+ 2 e^lam v); v <- v - alpha Hv; p <- p + v; copies of v
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        val[k] = 0.f;
        if (row0 + k < M) {
          const long long o = (long long)(row0 + k) * e.ldc + col;
          const float vo = e.v[o];
          float hv = acc[k];
          if (e.lam) hv += 2.f * expf(e.lam[o]) * vo;
          const float vn = vo - e.alpha * hv;
          e.v[o] = vn;
          e.p[o] += vn;
          val[k] = vn;
        }
      }
      dual = e.out != nullptr;
      break;
    }
    default:
      return;
  }
  if (!dual) return;
  if (e.out) {
    T* o = (T*)e.out;
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (row0 + k < M) store1<T>(o + (long long)(row0 + k) * e.ld + col, val[k]);
  }
  if (e.outT) store4<T>((T*)e.outT + (long long)col * e.ldT + row0, val);
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
template <typename T>
__device__ void bias_rows(const BiasJob& j, int local_block) {
  const int row = local_block * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= j.rows) return;
  const T* p = (const T*)j.Mt + (long long)row * j.ld;
  float acc = 0.f;
  for (int c = lane; c < j.k; c += 64) acc += (float)p[c];
  acc = wave_sum_f(acc);
  if (lane != 0) return;
  switch (j.mode) {
    case EPI_WGRAD: {
      float g = acc;
      if (j.lam) g += 2.f * expf(j.lam[row]) * j.x[row];
      j.C[row] = g;
      break;
    }
    case EPI_WGRAD_INIT:
      j.v[row] = acc; j.p[row] = acc;
      break;
    case EPI_WGRAD_NEUMANN: {
      const float vo = j.v[row];
      float hv = acc;
      if (j.lam) hv += 2.f * expf(j.lam[row]) * vo;
      const float vn = vo - j.alpha * hv;
      j.v[row] = vn;
      j.p[row] += vn;
      break;
    }
    default: break;
  }
}

template <typename T, int BM, int BN, int NCH>
__global__ __launch_bounds__(256) void gemm_fused_kernel(GemmBatch batch) {
  constexpr int ROW = NCH + 1;                     // LDS row pitch in 16-byte chunks
  constexpr int EPC = 16 / (int)sizeof(T);         // elements per chunk
  constexpr int KT = NCH * EPC;                    // elements per k-tile
  constexpr int TM = BM / 64, TN = BN / 64;        // 32x32 blocks per wavefront
  constexpr int LA = BM * NCH / 256, LB = BN * NCH / 256;
  constexpr int NACC = TM * TN * 16;
  static_assert(BM % 64 == 0 && BN % 64 == 0 && (BM * NCH) % 256 == 0 && (BN * NCH) % 256 == 0, "tile");
  __shared__ uint4 sA[BM * ROW];
  __shared__ uint4 sB[BN * ROW];
  __shared__ int s_last;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  // ---- which job is this workgroup?
  int bid = blockIdx.x;
  if (bid >= batch.gemm_blocks) {
    bid -= batch.gemm_blocks;
    int j = 0;
    while (j + 1 < batch.n_bias && bid >= batch.bias_begin[j + 1]) ++j;
    bias_rows<T>(batch.bias[j], bid - batch.bias_begin[j]);
    return;
  }
  int pi = 0;
  while (pi + 1 < batch.n && bid >= batch.block_begin[pi + 1]) ++pi;
  const GemmArgs& g = batch.p[pi].g;
  const int local = bid - batch.block_begin[pi];
  const int S = g.splitk;
  const int tile = local / S, s = local - tile * S;
  const int tiles_n = g.Np / BN;
  const int m0 = (tile / tiles_n) * BM, n0 = (tile % tiles_n) * BN;

  const int T0 = g.Kp[0] / KT, T1 = g.Kp[1] / KT, TT = T0 + T1;
  const int tb = (int)((long long)TT * s / S);
  const int te = (int)((long long)TT * (s + 1) / S);

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  uint4 ra[LA], rb[LB];
  auto gload = [&](int t) {
    const int pair = t >= T0 ? 1 : 0;
    const int tt = pair ? t - T0 : t;
    const T* Ab = (const T*)g.A[pair];
    const T* Bb = (const T*)g.B[pair];
    const long long lda = g.lda[pair], ldb = g.ldb[pair];
#pragma unroll
    for (int i = 0; i < LA; ++i) {
      const int idx = tid + i * 256, r = idx / NCH, c = idx % NCH;
      ra[i] = *(const uint4*)(Ab + (long long)(m0 + r) * lda + (long long)tt * KT + c * EPC);
    }
#pragma unroll
    for (int i = 0; i < LB; ++i) {
      const int idx = tid + i * 256, r = idx / NCH, c = idx % NCH;
      rb[i] = *(const uint4*)(Bb + (long long)(n0 + r) * ldb + (long long)tt * KT + c * EPC);
    }
  };

  if (tb < te) gload(tb);
  for (int t = tb; t < te; ++t) {
    if (t > tb) __syncthreads();
#pragma unroll
    for (int i = 0; i < LA; ++i) {
      const int idx = tid + i * 256;
      sA[(idx / NCH) * ROW + idx % NCH] = ra[i];
    }
#pragma unroll
    for (int i = 0; i < LB; ++i) {
      const int idx = tid + i * 256;
      sB[(idx / NCH) * ROW + idx % NCH] = rb[i];
    }
    __syncthreads();
    if (t + 1 < te) gload(t + 1);
#pragma unroll
    for (int j = 0; j < NCH / 2; ++j) {
      const int c = 2 * j + (lane >> 5);
      uint4 af[TM], bf[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) af[i] = sA[(wm * TM * 32 + i * 32 + (lane & 31)) * ROW + c];
#pragma unroll
      for (int i = 0; i < TN; ++i) bf[i] = sB[(wn * TN * 32 + i * 32 + (lane & 31)) * ROW + c];
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int jn = 0; jn < TN; ++jn) MfmaChunk<T>::run(af[i], bf[jn], acc[i][jn]);
    }
  }

  // ---- split-K: publish this slice; the last workgroup of the tile sums all slices in order
  if (S > 1) {
    float* part = batch.partials + ((long long)(batch.p[pi].partial_base + (long long)tile * S)) * (NACC * 256);
    float* mine = part + (long long)s * (NACC * 256) + tid;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int jn = 0; jn < TN; ++jn)
#pragma unroll
        for (int r = 0; r < 16; ++r) mine[((i * TN + jn) * 16 + r) * 256] = acc[i][jn][r];
    __threadfence();
    __syncthreads();
    if (tid == 0) {
      int* ticket = batch.tickets + batch.p[pi].ticket_base + tile;
      const int old = atomicAdd(ticket, 1);
      const int last = old == S - 1;
      if (last) *ticket = 0;
      s_last = last;
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int jn = 0; jn < TN; ++jn)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][jn][r] = 0.f;
    for (int s2 = 0; s2 < S; ++s2) {
      const float* src = part + (long long)s2 * (NACC * 256) + tid;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int jn = 0; jn < TN; ++jn)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[i][jn][r] += src[((i * TN + jn) * 16 + r) * 256];
    }
  }

  // ---- epilogue from registers
  const Epilogue& e = batch.p[pi].e;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int jn = 0; jn < TN; ++jn) {
      const int col = n0 + wn * TN * 32 + jn * 32 + (lane & 31);
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int row0 = m0 + wm * TM * 32 + i * 32 + 8 * q + 4 * (lane >> 5);
        const float quad[4] = {acc[i][jn][4 * q], acc[i][jn][4 * q + 1], acc[i][jn][4 * q + 2], acc[i][jn][4 * q + 3]};
        epilogue_quad<T>(e, g.M, g.N, row0, col, quad);
      }
    }
}

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------

int gemm_ktile_elems(Elem elem) { return GEMM_NCH * (elem == ELEM_BF16 ? 8 : 4); }

void launch_gemm_batch(Ctx& ctx, Elem elem, int tile, GemmBatch& b, double flops) {
  const int bt = tile == TILE_128 ? 128 : 64;
  int blocks = 0;
  for (int i = 0; i < b.n; ++i) {
    b.block_begin[i] = blocks;
    blocks += (b.p[i].g.Mp / bt) * (b.p[i].g.Np / bt) * b.p[i].g.splitk;
  }
  b.block_begin[b.n] = blocks;
  b.gemm_blocks = blocks;
  int bias_blocks = 0;
  for (int i = 0; i < b.n_bias; ++i) {
    b.bias_begin[i] = bias_blocks;
    bias_blocks += (b.bias[i].rows + 3) / 4;
  }
  b.bias_begin[b.n_bias] = bias_blocks;
  const int total = blocks + bias_blocks;
  if (total <= 0) return;
  Launch l(ctx, BETTY_K_GEMM, flops, 0);
  if (elem == ELEM_BF16) {
    if (tile == TILE_128) gemm_fused_kernel<__bf16, 128, 128, GEMM_NCH><<<total, 256, 0, ctx.stream>>>(b);
    else gemm_fused_kernel<__bf16, 64, 64, GEMM_NCH><<<total, 256, 0, ctx.stream>>>(b);
  } else {
    if (tile == TILE_128) gemm_fused_kernel<float, 128, 128, GEMM_NCH><<<total, 256, 0, ctx.stream>>>(b);
    else gemm_fused_kernel<float, 64, 64, GEMM_NCH><<<total, 256, 0, ctx.stream>>>(b);
  }
}

}  // namespace betty

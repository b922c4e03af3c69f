// MFMA GEMM for gfx950:  C (fp32) = sum_p A_p * B_p^T  over one or two operand pairs.
//
// Every dense contraction of the hypergradient path (forward, backward, and the forward-
// over-reverse passes of the Hessian-vector product; paper Sec. 3.2) is brought to this one
// shape by keeping each operand in the workspace with its reduction index contiguous
// ("K-major") and zero-padded to a multiple of 128 in both extents.  The two-pair form is
// the concatenated-K product of the R-op passes, e.g. Rz = Ra W + a V as [Ra | a] [W ; V].
//
// Tiling: one workgroup of 256 threads (4 wavefronts, 2 x 2) owns a BM x BN tile of C; each
// wavefront owns (BM/2) x (BN/2) as 32 x 32 MFMA blocks.  K is consumed in tiles of NCH 16-byte
// chunks per row.  Global -> registers -> LDS with the next tile's global loads in flight
// while the current one is multiplied.  LDS rows are padded by one chunk so that the 16-byte
// fragment reads of 8 consecutive rows fall in distinct banks.
//
// Fragment layout: lane l of a wavefront supplies row (l % 32) of the A block and row (l % 32)
// of the B block; lanes 0-31 take the even chunks of the k-tile and lanes 32-63 the odd ones.
// A chunk is 8 bf16 (one v_mfma_f32_32x32x16_bf16) or 4 floats (four v_mfma_f32_32x32x2_f32).
// Since A and B use the same chunk assignment the order of k inside the product is irrelevant.
// The accumulator holds C[8*(r/4) + 4*(l/32) + r%4][l%32] in register r of lane l.
#include "internal.h"

namespace betty {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

template <typename T> struct MfmaChunk;

template <> struct MfmaChunk<__bf16> {
  static __device__ __forceinline__ void run(const uint4& a, const uint4& b, f32x16& acc) {
    bf16x8 av = __builtin_bit_cast(bf16x8, a);
    bf16x8 bv = __builtin_bit_cast(bf16x8, b);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc, 0, 0, 0);
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

template <typename T, int BM, int BN, int NCH>
__global__ __launch_bounds__(256) void gemm_kk_kernel(GemmArgs g) {
  constexpr int ROW = NCH + 1;                     // LDS row pitch in 16-byte chunks
  constexpr int EPC = 16 / (int)sizeof(T);         // elements per chunk
  constexpr int KT = NCH * EPC;                    // elements per k-tile
  constexpr int TM = BM / 64, TN = BN / 64;        // 32x32 blocks per wavefront
  constexpr int LA = BM * NCH / 256, LB = BN * NCH / 256;
  static_assert(BM % 64 == 0 && BN % 64 == 0 && (BM * NCH) % 256 == 0 && (BN * NCH) % 256 == 0, "tile");
  __shared__ uint4 sA[BM * ROW];
  __shared__ uint4 sB[BN * ROW];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int T0 = g.Kp[0] / KT, T1 = g.Kp[1] / KT, TT = T0 + T1;
  const int s = blockIdx.z;
  const int tb = (int)((long long)TT * s / g.splitk);
  const int te = (int)((long long)TT * (s + 1) / g.splitk);

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

  float* C = g.C + (long long)s * g.split_stride;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int jn = 0; jn < TN; ++jn) {
      const int col = n0 + wn * TN * 32 + jn * 32 + (lane & 31);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm * TM * 32 + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (row < g.M && col < g.N) C[(long long)row * g.ldc + col] = acc[i][jn][r];
      }
    }
}

void launch_gemm(Ctx& ctx, Elem elem, const GemmArgs& g, double flops) {
  constexpr int BM = 128, BN = 128, NCH = 4;
  dim3 grid(g.Np / BN, g.Mp / BM, g.splitk);
  Launch l(ctx, BETTY_K_GEMM, flops, 0);
  if (elem == ELEM_BF16)
    gemm_kk_kernel<__bf16, BM, BN, NCH><<<grid, 256, 0, ctx.stream>>>(g);
  else
    gemm_kk_kernel<float, BM, BN, NCH><<<grid, 256, 0, ctx.stream>>>(g);
}

}  // namespace betty

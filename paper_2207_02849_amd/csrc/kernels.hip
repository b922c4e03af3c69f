// Non-GEMM kernels of the hypergradient path: conversion of flat fp32 parameters into GEMM
// operands in both orientations, the row-wise loss kernels, the two narrow-output-layer kernels
// (last layer of the first-order and of the R-op passes when the output has at most 16 columns),
// the weight-net kernels, and the streaming kernels over the flat parameter-shaped vectors
// (finite-difference steps, conjugate gradient, mixed VJPs, Adam).
#include <algorithm>

#include "internal.h"

namespace betty {

// ------------------------------------------------------------------------------------------
// small device helpers
// ------------------------------------------------------------------------------------------

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}
__device__ __forceinline__ double wave_sum(double x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}
__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
  return x;
}

// sum over a 256-thread block, result valid in every thread; fixed combination order
template <typename R>
__device__ __forceinline__ R block_sum(R x, R* smem4) {
  x = wave_sum(x);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) smem4[threadIdx.x >> 6] = x;
  __syncthreads();
  return smem4[0] + smem4[1] + smem4[2] + smem4[3];
}

template <typename T> __device__ __forceinline__ T from_float(float x);
template <> __device__ __forceinline__ float from_float<float>(float x) { return x; }
template <> __device__ __forceinline__ __bf16 from_float<__bf16>(float x) { return (__bf16)x; }  // RNE
template <typename T> __device__ __forceinline__ float to_float(T x) { return (float)x; }

// ------------------------------------------------------------------------------------------
// operand conversion: fp32 source -> operand type, row-major and transposed, through a 64x64
// LDS tile; up to MAX_PROBLEMS matrices per launch
// ------------------------------------------------------------------------------------------

// four consecutive elements of the operand type as one store
template <typename T> __device__ __forceinline__ void store_quad(T* p, float a, float b, float c, float d);
template <> __device__ __forceinline__ void store_quad<float>(float* p, float a, float b, float c, float d) {
  *(float4*)p = make_float4(a, b, c, d);
}
template <> __device__ __forceinline__ void store_quad<__bf16>(__bf16* p, float a, float b, float c, float d) {
  typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
  bf16x4 v = {(__bf16)a, (__bf16)b, (__bf16)c, (__bf16)d};
  *(bf16x4*)p = v;
}

template <typename T>
__global__ __launch_bounds__(256) void convert_batch_kernel(ConvertBatch b) {
  __shared__ float tile[64][65];
  int bid = blockIdx.x, ji = 0;
  while (ji + 1 < b.n && bid >= b.block_begin[ji + 1]) ++ji;
  const ConvertJob& j = b.j[ji];
  bid -= b.block_begin[ji];
  const int tiles_x = (j.cols + 63) / 64;
  const int c0 = (bid % tiles_x) * 64, r0 = (bid / tiles_x) * 64;
  T* out = (T*)j.out;
  T* outT = (T*)j.outT;
  // Four elements per thread and access when the source rows and all destinations allow aligned
  // 16-byte loads (every weight matrix whose width is a multiple of four); else one by one.
  const bool quads = j.cols % 4 == 0 && j.lds % 4 == 0 && j.ld % 4 == 0 && j.ldT % 4 == 0 &&
                     ((uintptr_t)j.src & 15) == 0 && ((uintptr_t)j.out & 15) == 0 &&
                     ((uintptr_t)j.outT & 15) == 0 && ((uintptr_t)j.outT32 & 15) == 0;
  if (quads) {
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int rl = ty + 16 * i, r = r0 + rl, c = c0 + 4 * tx;
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (r < j.rows && c < j.cols) {
        v = *(const float4*)(j.src + (long long)r * j.lds + c);
        v.x *= j.scale; v.y *= j.scale; v.z *= j.scale; v.w *= j.scale;
        if (out) store_quad<T>(out + (long long)r * j.ld + c, v.x, v.y, v.z, v.w);
      }
      tile[rl][4 * tx] = v.x; tile[rl][4 * tx + 1] = v.y; tile[rl][4 * tx + 2] = v.z; tile[rl][4 * tx + 3] = v.w;
    }
    if (!outT) return;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int cl = ty + 16 * i, c = c0 + cl, r = r0 + 4 * tx;
      if (c >= j.cols || r >= j.rows) continue;
      const float v0 = tile[4 * tx][cl], v1 = tile[4 * tx + 1][cl], v2 = tile[4 * tx + 2][cl], v3 = tile[4 * tx + 3][cl];
      T* o = outT + (long long)c * j.ldT + r;
      float* o32 = j.outT32 ? j.outT32 + (long long)c * j.ldT + r : nullptr;
      if (r + 3 < j.rows) {
        store_quad<T>(o, v0, v1, v2, v3);
        if (o32) store_quad<float>(o32, v0, v1, v2, v3);
      } else {                                     // last rows of a height that is no multiple of four
        const float v[4] = {v0, v1, v2, v3};
        for (int k = 0; k < 4 && r + k < j.rows; ++k) {
          o[k] = from_float<T>(v[k]);
          if (o32) o32[k] = v[k];
        }
      }
    }
    return;
  }
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
#pragma unroll 4
  for (int i = 0; i < 16; ++i) {
    const int r = r0 + ty + 4 * i, c = c0 + tx;
    float val = 0.f;
    if (r < j.rows && c < j.cols) {
      val = j.scale * j.src[(long long)r * j.lds + c];
      if (out) out[(long long)r * j.ld + c] = from_float<T>(val);
    }
    tile[ty + 4 * i][tx] = val;
  }
  if (!outT) return;
  __syncthreads();
#pragma unroll 4
  for (int i = 0; i < 16; ++i) {
    const int c = c0 + ty + 4 * i, r = r0 + tx;
    if (r < j.rows && c < j.cols) {
      outT[(long long)c * j.ldT + r] = from_float<T>(tile[tx][ty + 4 * i]);
      if (j.outT32) j.outT32[(long long)c * j.ldT + r] = tile[tx][ty + 4 * i];
    }
  }
}

void launch_convert_batch(Ctx& ctx, Elem elem, ConvertBatch& b) {
  int blocks = 0;
  double bytes = 0;
  for (int i = 0; i < b.n; ++i) {
    b.block_begin[i] = blocks;
    blocks += ((b.j[i].cols + 63) / 64) * ((b.j[i].rows + 63) / 64);
    bytes += (double)b.j[i].rows * b.j[i].cols * (4.0 + ((b.j[i].out ? 1 : 0) + (b.j[i].outT ? 1 : 0)) * elem_size(elem));
  }
  b.block_begin[b.n] = blocks;
  if (blocks <= 0) return;
  Launch l(ctx, BETTY_K_SHADOW, 0, bytes);
  if (elem == ELEM_BF16) convert_batch_kernel<__bf16><<<blocks, 256, 0, ctx.stream>>>(b);
  else convert_batch_kernel<float><<<blocks, 256, 0, ctx.stream>>>(b);
}

void launch_convert_dual(Ctx& ctx, Elem elem, const float* src, long long lds, float scale,
                         int rows, int cols, void* out, int ld, void* outT, int ldT) {
  ConvertBatch b;
  b.n = 1;
  b.j[0] = ConvertJob{src, lds, scale, rows, cols, out, ld, outT, ldT};
  launch_convert_batch(ctx, elem, b);
}

// ------------------------------------------------------------------------------------------
// row-wise loss kernels: one wavefront per sample
// ------------------------------------------------------------------------------------------

template <typename T>
__global__ __launch_bounds__(256) void loss_rows_kernel(LossBatch lb) {
  const int blocks0 = (lb.a[0].rows + 3) / 4;
  const int which = (lb.n > 1 && (int)blockIdx.x >= blocks0) ? 1 : 0;
  const LossArgs& a = lb.a[which];
  const int row = ((int)blockIdx.x - (which ? blocks0 : 0)) * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= a.rows) return;
  const float* z = a.Z + (long long)row * a.ldz;
  float ell, m = 0.f, sum = 1.f;
  int y = 0;
  if (a.loss == BETTY_LOSS_SOFTMAX_CE) {
    m = -INFINITY;
    for (int c = lane; c < a.C; c += 64) m = fmaxf(m, z[c]);
    m = wave_max(m);
    sum = 0.f;
    for (int c = lane; c < a.C; c += 64) sum += expf(z[c] - m);
    sum = wave_sum(sum);
    // a label outside [0, C) is clamped into the range, for the gather and the one-hot alike
    y = min(max(a.y[row], 0), a.C - 1);
    ell = logf(sum) + m - z[y];                  // integer gather of the label's logit
  } else {
    const float* t = a.target + (long long)row * a.C;
    float acc = 0.f;
    for (int c = lane; c < a.C; c += 64) { const float r = z[c] - t[c]; acc += r * r; }
    ell = wave_sum(acc);
  }
  float omega = 1.f;
  if (a.reweight && a.omega_fixed) {
    omega = a.omega_fixed[row];
  } else if (a.reweight) {
    const int H = a.hidden;
    float part = 0.f;
    for (int j = lane; j < H; j += 64)
      part += a.theta[2 * H + j] * fmaxf(a.theta[j] * ell + a.theta[H + j], 0.f);
    part = wave_sum(part) + a.theta[3 * H];
    omega = 1.f / (1.f + expf(-part));
    // sigmoid'(x) = sigmoid(x) sigmoid(-x): no 1 - omega, which loses every digit once omega rounds to 1
    if (lane == 0 && a.dsig) a.dsig[row] = omega / (1.f + expf(part));
  }
  const float s = omega * a.inv_batch;
  if (lane == 0) { a.ell[row] = ell; a.s[row] = s; a.omega[row] = omega; }
  T* D = (T*)a.D + (long long)row * a.ldD;
  T* Dt = (T*)a.Dt + row;
  if (a.loss == BETTY_LOSS_SOFTMAX_CE) {
    float* P = a.P + (long long)row * a.ldz;
    const float inv = 1.f / sum;
    for (int c = lane; c < a.C; c += 64) {
      const float p = expf(z[c] - m) * inv;
      P[c] = p;
      const T dv = from_float<T>(s * (p - (c == y ? 1.f : 0.f)));
      D[c] = dv;
      Dt[(long long)c * a.ldDt] = dv;
    }
  } else {
    const float* t = a.target + (long long)row * a.C;
    for (int c = lane; c < a.C; c += 64) {
      const T dv = from_float<T>(s * 2.f * (z[c] - t[c]));
      D[c] = dv;
      Dt[(long long)c * a.ldDt] = dv;
    }
  }
}

void launch_loss_rows(Ctx& ctx, Elem elem, const LossBatch& lb) {
  int blocks = 0;
  for (int i = 0; i < lb.n; ++i) blocks += (lb.a[i].rows + 3) / 4;
  if (blocks <= 0) return;
  Launch l(ctx, BETTY_K_LOSS);
  if (elem == ELEM_BF16) loss_rows_kernel<__bf16><<<blocks, 256, 0, ctx.stream>>>(lb);
  else loss_rows_kernel<float><<<blocks, 256, 0, ctx.stream>>>(lb);
}

template <typename T>
__global__ __launch_bounds__(256) void loss_hessian_rows_kernel(int loss, const float* P, const float* Rz,
                                                                long long ld, const float* s, int rows,
                                                                int C, T* D, int ldD, T* Dt, int ldDt) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= rows) return;
  const float* rz = Rz + (long long)row * ld;
  T* o = D + (long long)row * ldD;
  T* ot = Dt + row;
  const float si = s[row];
  if (loss == BETTY_LOSS_SOFTMAX_CE) {
    const float* p = P + (long long)row * ld;
    float dot = 0.f;
    for (int c = lane; c < C; c += 64) dot += p[c] * rz[c];
    dot = wave_sum(dot);
    for (int c = lane; c < C; c += 64) {
      const T v = from_float<T>(si * (p[c] * rz[c] - p[c] * dot));
      o[c] = v;
      ot[(long long)c * ldDt] = v;
    }
  } else {
    for (int c = lane; c < C; c += 64) {
      const T v = from_float<T>(si * 2.f * rz[c]);
      o[c] = v;
      ot[(long long)c * ldDt] = v;
    }
  }
}

void launch_loss_hessian_rows(Ctx& ctx, Elem elem, int loss, const float* P, const float* Rz, long long ld,
                              const float* s, int rows, int C, void* D, int ldD, void* Dt, int ldDt) {
  if (rows <= 0) return;
  Launch l(ctx, BETTY_K_LOSS);
  if (elem == ELEM_BF16)
    loss_hessian_rows_kernel<__bf16><<<(rows + 3) / 4, 256, 0, ctx.stream>>>(loss, P, Rz, ld, s, rows, C, (__bf16*)D, ldD, (__bf16*)Dt, ldDt);
  else
    loss_hessian_rows_kernel<float><<<(rows + 3) / 4, 256, 0, ctx.stream>>>(loss, P, Rz, ld, s, rows, C, (float*)D, ldD, (float*)Dt, ldDt);
}

__global__ __launch_bounds__(256) void loss_directional_rows_kernel(int loss, const float* P, const float* Z,
                                                                    const int32_t* y, const float* target,
                                                                    const float* Rz, long long ld, int rows,
                                                                    int C, float* cvec) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= rows) return;
  const float* rz = Rz + (long long)row * ld;
  float acc = 0.f;
  if (loss == BETTY_LOSS_SOFTMAX_CE) {
    const float* p = P + (long long)row * ld;
    for (int c = lane; c < C; c += 64) acc += p[c] * rz[c];
    acc = wave_sum(acc);
    const int yy = min(max(y[row], 0), C - 1);
    acc -= rz[yy];
  } else {
    const float* z = Z + (long long)row * ld;
    const float* t = target + (long long)row * C;
    for (int c = lane; c < C; c += 64) acc += 2.f * (z[c] - t[c]) * rz[c];
    acc = wave_sum(acc);
  }
  if (lane == 0) cvec[row] = acc;
}

// ------------------------------------------------------------------------------------------
// last layer of the R-op passes for narrow outputs (see LastRopArgs)
// ------------------------------------------------------------------------------------------

// Workgroup = 16 wavefronts, 4 samples.  Both small products run as zero-padded 32 x 32 MFMA
// blocks (rows = the 4 samples; only lanes that own a real operand row load anything):
//  phase 1  Rz_L block (4 x C): K = n_in sliced over the wavefronts in chunk pairs, partial blocks
//           combined through LDS in wavefront order;
//  phase 2  (one wavefront) loss Hessian per sample with 16-lane butterflies -> R delta_L, kept in
//           LDS in operand type next to delta_L;
//  phase 3  each wavefront takes 32 columns j at a time: (R delta_L W^T + delta_L V^T) is one
//           chunk pair of K = 16 classes, then the elementwise part and both output copies.
template <typename T>
__global__ __launch_bounds__(1024) void last_layer_rop_kernel(LastRopArgs a) {
  constexpr int S = 4, CP = LAST_ROP_MAX_C, EPC = 16 / (int)sizeof(T), NW = 16, U = sizeof(T) == 4 ? 2 : 4;
  __shared__ float part[NW][S * CP];
  __shared__ __attribute__((aligned(16))) T rdT[32][CP], dlT[32][CP];   // rows >= S stay zero
  const int t = threadIdx.x, lane = t & 63, ks = t >> 6;
  const int row = lane & 31, half = lane >> 5;
  // blockIdx.y splits the columns j of phase 3; every split repeats phases 1-2 for its samples
  // (cheap), the first one writes R delta_L
  const int i0 = blockIdx.x * S;
  const int jsplit = ((a.n_in + gridDim.y - 1) / gridDim.y + 31) / 32 * 32;
  const int j_begin = blockIdx.y * jsplit, j_end = min(a.n_in, j_begin + jsplit);
  const u32x4 zero = {0u, 0u, 0u, 0u};
  for (int x = t; x < 32 * CP; x += 64 * NW) { (&rdT[0][0])[x] = from_float<T>(0.f); (&dlT[0][0])[x] = from_float<T>(0.f); }

  // Everything phases 2 and 3 read from memory is independent of phase 1: request it now, so the
  // kernel pays one memory round trip instead of three.  (The launcher sizes the column splits so
  // that a wavefront has at most one block of 32 columns.)
  const int jb = j_begin + ks * 32;
  const bool jb_ok = jb < j_end && !a.cvec;                 // the directional form has no phase 3
  const int j = jb + lane;
  const bool j_ok = jb_ok && lane < 32 && j < j_end;
  u32x4 w3[CP / (2 * EPC)], v3[CP / (2 * EPC)];
  float dphi3[S], e23[S], rz3[S];
#pragma unroll
  for (int p = 0; p < CP / (2 * EPC); ++p) { w3[p] = zero; v3[p] = zero; }
#pragma unroll
  for (int ss = 0; ss < S; ++ss) { dphi3[ss] = 0.f; e23[ss] = 0.f; rz3[ss] = 0.f; }
  if (jb_ok) {
    const int jr = jb + row;                                // < n_in_p: rows beyond n_in are zero padding
    const T* wr = (const T*)a.Wn + (long long)jr * a.ldn + half * EPC;
    const T* vr = (const T*)a.Vn + (long long)jr * a.ldn + half * EPC;
#pragma unroll
    for (int p = 0; p < CP / (2 * EPC); ++p) {
      w3[p] = *(const u32x4*)(wr + p * 2 * EPC);
      v3[p] = *(const u32x4*)(vr + p * 2 * EPC);
    }
  }
  if (j_ok) {
#pragma unroll
    for (int ss = 0; ss < S; ++ss)
      if (i0 + ss < a.B) {
        const long long f = (long long)(i0 + ss) * a.ldf + j;
        dphi3[ss] = a.dphi[f];
        if (a.e2) { e23[ss] = a.e2[f]; rz3[ss] = a.Rz[f]; }
      }
  }
  float p2 = 0.f, s2 = 0.f, cb2 = 0.f;
  T d2 = from_float<T>(0.f);
  if (ks == 0) {
    const int s = lane >> 4, c = lane & 15, i = i0 + s;
    if (c < a.C && i < a.B) {
      if (a.loss == BETTY_LOSS_SOFTMAX_CE) p2 = a.P[(long long)i * a.ldp + c];
      if (a.cbias) cb2 = a.cbias[c];
      if (!a.cvec) {
        s2 = a.s[i];
        d2 = ((const T*)a.DL)[(long long)i * a.ldd + c];
      }
    }
  }

  // ---- phase 1
  {
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    const bool a_ok = row < S && i0 + row < a.B, b_ok = row < a.C;
    const int pairs = a.n_in_p / (2 * EPC), per = (pairs + NW - 1) / NW;
    const int p_begin = ks * per, p_end = min(pairs, p_begin + per);
    const T* ra = (const T*)a.RA + (long long)(i0 + row) * a.lda + half * EPC;
    const T* av = (const T*)a.A + (long long)(i0 + row) * a.lda + half * EPC;
    const T* w = (const T*)a.Wt + (long long)row * a.ldt + half * EPC;
    const T* v = (const T*)a.Vt + (long long)row * a.ldt + half * EPC;
    for (int p0 = p_begin; p0 < p_end; p0 += U) {
      u32x4 r8[U], a8[U], w8[U], v8[U];
#pragma unroll
      for (int u = 0; u < U; ++u) { r8[u] = zero; a8[u] = zero; w8[u] = zero; v8[u] = zero; }
      if (a_ok) {
#pragma unroll
        for (int u = 0; u < U; ++u)
          if (p0 + u < p_end) {
            r8[u] = *(const u32x4*)(ra + (p0 + u) * 2 * EPC);
            a8[u] = *(const u32x4*)(av + (p0 + u) * 2 * EPC);
          }
      }
      if (b_ok) {
#pragma unroll
        for (int u = 0; u < U; ++u)
          if (p0 + u < p_end) {
            w8[u] = *(const u32x4*)(w + (p0 + u) * 2 * EPC);
            v8[u] = *(const u32x4*)(v + (p0 + u) * 2 * EPC);
          }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {                         // all-zero chunks add nothing
        MfmaChunk<T>::run(r8[u], w8[u], acc);
        MfmaChunk<T>::run(a8[u], v8[u], acc);
      }
    }
    // registers 0..3 of lanes 0..15 hold samples 0..3 of class `lane`
    if (lane < CP) {
#pragma unroll
      for (int r = 0; r < S; ++r) part[ks][r * CP + lane] = acc[r];
    }
  }
  __syncthreads();

  // ---- phase 2
  if (ks == 0) {
    const int s = lane >> 4, c = lane & 15, i = i0 + s;
    float rz = 0.f;
#pragma unroll
    for (int q = 0; q < NW; ++q) rz += part[q][lane];
    const bool ok = c < a.C && i < a.B;
    rz = ok ? rz + cb2 : 0.f;
    if (a.cvec) {                                           // directional form: one number per sample
      float term = 0.f;
      if (ok) {
        if (a.loss == BETTY_LOSS_SOFTMAX_CE) {
          const int yy = min(max(a.y[i], 0), a.C - 1);
          term = p2 * rz - (c == yy ? rz : 0.f);
        } else {
          term = 2.f * (a.Z[(long long)i * a.ldp + c] - a.target[(long long)i * a.C + c]) * rz;
        }
      }
#pragma unroll
      for (int o = 8; o > 0; o >>= 1) term += __shfl_xor(term, o, 64);
      if (c == 0 && i < a.B) a.cvec[i] = term;
    } else {
      const float si = s2;
      float val;
      if (a.loss == BETTY_LOSS_SOFTMAX_CE) {
        const float p = p2;
        float dot = p * rz;
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) dot += __shfl_xor(dot, o, 64);
        val = si * (p * rz - p * dot);
      } else {
        val = si * 2.f * rz;
      }
      const T vt = from_float<T>(val);
      if (ok) {
        rdT[s][c] = vt;
        dlT[s][c] = d2;
        if (blockIdx.y == 0) {
          ((T*)a.RDL)[(long long)i * a.ldd + c] = vt;
          ((T*)a.RDLt)[(long long)c * a.ldRDLt + i] = vt;
        }
      }
    }
  }
  __syncthreads();                                          // (every wavefront reaches this, in both forms)

  // ---- phase 3
  if (jb_ok) {
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
    for (int p = 0; p < CP / (2 * EPC); ++p) {
      const u32x4 r8 = *(const u32x4*)(&rdT[row][p * 2 * EPC + half * EPC]);
      const u32x4 d8 = *(const u32x4*)(&dlT[row][p * 2 * EPC + half * EPC]);
      MfmaChunk<T>::run(r8, w3[p], acc);
      MfmaChunk<T>::run(d8, v3[p], acc);
    }
    // registers 0..3 of lanes 0..31: samples i0..i0+3 of column jb + lane
    if (j_ok) {
      float out[S];
#pragma unroll
      for (int ss = 0; ss < S; ++ss) {
        const int ii = i0 + ss;
        float o = 0.f;
        if (ii < a.B) {
          o = acc[ss] * dphi3[ss] + e23[ss] * rz3[ss];
          ((T*)a.RD)[(long long)ii * a.ldRD + j] = from_float<T>(o);
        }
        out[ss] = o;                                       // rows beyond the batch: zero padding
      }
      T* ot = (T*)a.RDt + (long long)j * a.ldRDt + i0;
#pragma unroll
      for (int ss = 0; ss < S; ++ss) ot[ss] = from_float<T>(out[ss]);
    }
  }
}

void launch_last_layer_rop(Ctx& ctx, Elem elem, const LastRopArgs& a) {
  if (a.B <= 0) return;
  Launch l(ctx, BETTY_K_LAST_LAYER, 8.0 * a.B * a.n_in * a.C, 0);      // two pairs in each of two products
  const int blocks = (a.B + 3) / 4;
  // column splits: at most one block of 32 columns per wavefront (16 x 32 per workgroup), and
  // enough workgroups to occupy the chip
  const int splits = a.cvec ? 1 : std::max((a.n_in + 511) / 512, std::max(1, std::min(256 / blocks, (a.n_in + 31) / 32)));
  const dim3 grid(blocks, splits);
  if (elem == ELEM_BF16) last_layer_rop_kernel<__bf16><<<grid, 1024, 0, ctx.stream>>>(a);
  else last_layer_rop_kernel<float><<<grid, 1024, 0, ctx.stream>>>(a);
}

// Same layout as last_layer_rop_kernel (16 wavefronts, 4 samples, zero-padded MFMA blocks);
// blockIdx.z selects the batch.
template <typename T>
__global__ __launch_bounds__(1024) void last_layer_grad_kernel(LastGradArgs a) {
  constexpr int S = 4, CP = LAST_ROP_MAX_C, EPC = 16 / (int)sizeof(T), NW = 16, U = sizeof(T) == 4 ? 2 : 4;
  __shared__ float part[NW][S * CP];
  __shared__ __attribute__((aligned(16))) T dlT[32][CP];   // rows >= S stay zero
  const LastGradSide& sd = a.side[blockIdx.z];
  const int t = threadIdx.x, lane = t & 63, ks = t >> 6;
  const int row = lane & 31, half = lane >> 5;
  const int i0 = blockIdx.x * S;
  if (i0 >= sd.B) return;                                   // the two batches may differ in size
  const int jsplit = ((a.n_in + gridDim.y - 1) / gridDim.y + 31) / 32 * 32;
  const int j_begin = blockIdx.y * jsplit, j_end = min(a.n_in, j_begin + jsplit);
  const u32x4 zero = {0u, 0u, 0u, 0u};
  for (int x = t; x < 32 * CP; x += 64 * NW) (&dlT[0][0])[x] = from_float<T>(0.f);

  // inputs of phase 3 that do not depend on the earlier phases
  const int jb = j_begin + ks * 32;
  const bool jb_ok = jb < j_end;
  const int j = jb + lane;
  const bool j_ok = jb_ok && lane < 32 && j < j_end;
  u32x4 w3[CP / (2 * EPC)];
  float dphi3[S], e23[S];
#pragma unroll
  for (int p = 0; p < CP / (2 * EPC); ++p) w3[p] = zero;
#pragma unroll
  for (int ss = 0; ss < S; ++ss) { dphi3[ss] = 0.f; e23[ss] = 0.f; }
  if (jb_ok) {
    const T* wr = (const T*)a.Wn + (long long)(jb + row) * a.ldn + half * EPC;
#pragma unroll
    for (int p = 0; p < CP / (2 * EPC); ++p) w3[p] = *(const u32x4*)(wr + p * 2 * EPC);
  }
  if (j_ok) {
#pragma unroll
    for (int ss = 0; ss < S; ++ss)
      if (i0 + ss < sd.B) {
        const long long f = (long long)(i0 + ss) * sd.ldf + j;
        dphi3[ss] = sd.dphi[f];
        if (sd.e2) e23[ss] = sd.e2[f];
      }
  }

  // ---- phase 1: logits block (4 x C), K = n_in sliced over the wavefronts
  {
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    const bool a_ok = row < S && i0 + row < sd.B, b_ok = row < a.C;
    const int pairs = a.n_in_p / (2 * EPC), per = (pairs + NW - 1) / NW;
    const int p_begin = ks * per, p_end = min(pairs, p_begin + per);
    const T* av = (const T*)sd.A + (long long)(i0 + row) * sd.lda + half * EPC;
    const T* w = (const T*)a.Wt + (long long)row * a.ldt + half * EPC;
    for (int p0 = p_begin; p0 < p_end; p0 += U) {
      u32x4 a8[U], w8[U];
#pragma unroll
      for (int u = 0; u < U; ++u) { a8[u] = zero; w8[u] = zero; }
      if (a_ok) {
#pragma unroll
        for (int u = 0; u < U; ++u)
          if (p0 + u < p_end) a8[u] = *(const u32x4*)(av + (p0 + u) * 2 * EPC);
      }
      if (b_ok) {
#pragma unroll
        for (int u = 0; u < U; ++u)
          if (p0 + u < p_end) w8[u] = *(const u32x4*)(w + (p0 + u) * 2 * EPC);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) MfmaChunk<T>::run(a8[u], w8[u], acc);
    }
    if (lane < CP) {
#pragma unroll
      for (int r = 0; r < S; ++r) part[ks][r * CP + lane] = acc[r];
    }
  }
  __syncthreads();

  // ---- phase 2: 16 lanes per sample (lane % 16 = class)
  if (ks == 0) {
    const int s = lane >> 4, c = lane & 15, i = i0 + s;
    const bool iok = i < sd.B, ok = iok && c < a.C;
    float z = 0.f;
#pragma unroll
    for (int q = 0; q < NW; ++q) z += part[q][lane];
    if (ok && a.bias) z += a.bias[c];
    float ell, p = 0.f, dz;
    int y = 0;
    if (a.loss == BETTY_LOSS_SOFTMAX_CE) {
      float m = ok ? z : -INFINITY;
#pragma unroll
      for (int o = 8; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
      const float ex = ok ? expf(z - m) : 0.f;
      float sum = ex;
#pragma unroll
      for (int o = 8; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
      y = min(max(iok ? sd.y[i] : 0, 0), a.C - 1);      // clamped into [0, C), for the gather and the one-hot alike
      const float zy = __shfl(z, (lane & ~15) + y, 64);
      ell = logf(sum) + m - zy;
      p = ex / sum;
      dz = p - (c == y ? 1.f : 0.f);
    } else {
      const float r = ok ? z - sd.target[(long long)i * a.C + c] : 0.f;
      float acc2 = r * r;
#pragma unroll
      for (int o = 8; o > 0; o >>= 1) acc2 += __shfl_xor(acc2, o, 64);
      ell = acc2;
      dz = 2.f * r;
    }
    float omega = 1.f;
    if (sd.reweight && sd.omega_fixed) {
      omega = iok ? sd.omega_fixed[i] : 1.f;
    } else if (sd.reweight) {
      const int H = a.hidden;
      float pw = 0.f;
      for (int hj = c; hj < H; hj += 16) pw += a.theta[2 * H + hj] * fmaxf(a.theta[hj] * ell + a.theta[H + hj], 0.f);
#pragma unroll
      for (int o = 8; o > 0; o >>= 1) pw += __shfl_xor(pw, o, 64);
      const float logit = pw + a.theta[3 * H];
      omega = 1.f / (1.f + expf(-logit));
      if (blockIdx.y == 0 && iok && c == 0 && sd.dsig) sd.dsig[i] = omega / (1.f + expf(logit));
    }
    const float sc = omega * sd.inv_batch;
    const T dv = from_float<T>(sc * dz);
    if (ok) dlT[s][c] = dv;
    if (blockIdx.y == 0) {
      if (iok && c == 0) { sd.ell[i] = ell; sd.s[i] = sc; sd.omega[i] = omega; }
      if (ok) {
        sd.ZL[(long long)i * sd.ldz + c] = z;
        if (a.loss == BETTY_LOSS_SOFTMAX_CE) sd.P[(long long)i * sd.ldz + c] = p;
        ((T*)sd.DL)[(long long)i * sd.ldd + c] = dv;
        ((T*)sd.DLt)[(long long)c * sd.ldDLt + i] = dv;
      }
    }
  }
  __syncthreads();

  // ---- phase 3: delta_{L-1} for 32 columns per wavefront
  if (jb_ok) {
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
    for (int p = 0; p < CP / (2 * EPC); ++p) {
      const u32x4 d8 = *(const u32x4*)(&dlT[row][p * 2 * EPC + half * EPC]);
      MfmaChunk<T>::run(d8, w3[p], acc);
    }
    if (j_ok) {
      float out[S];
#pragma unroll
      for (int ss = 0; ss < S; ++ss) {
        const int ii = i0 + ss;
        float o = 0.f;
        if (ii < sd.B) {
          o = acc[ss] * dphi3[ss];
          ((T*)sd.D)[(long long)ii * sd.ldD + j] = from_float<T>(o);
          if (sd.e2) sd.e2[(long long)ii * sd.ldf + j] = acc[ss] * e23[ss];
        }
        out[ss] = o;
      }
      T* ot = (T*)sd.Dt + (long long)j * sd.ldDt + i0;
#pragma unroll
      for (int ss = 0; ss < S; ++ss) ot[ss] = from_float<T>(out[ss]);
    }
  }
}

void launch_last_layer_grad(Ctx& ctx, Elem elem, const LastGradArgs& a) {
  int blocks = 0;
  for (int i = 0; i < a.n_sides; ++i) blocks = std::max(blocks, (a.side[i].B + 3) / 4);
  if (blocks <= 0) return;
  double flops = 0;
  for (int i = 0; i < a.n_sides; ++i) flops += 4.0 * a.side[i].B * a.n_in * a.C;
  Launch l(ctx, BETTY_K_LAST_LAYER, flops, 0);
  const int splits = std::max((a.n_in + 511) / 512, std::max(1, std::min(256 / (blocks * a.n_sides), (a.n_in + 31) / 32)));
  const dim3 grid(blocks, splits, a.n_sides);
  if (elem == ELEM_BF16) last_layer_grad_kernel<__bf16><<<grid, 1024, 0, ctx.stream>>>(a);
  else last_layer_grad_kernel<float><<<grid, 1024, 0, ctx.stream>>>(a);
}

void launch_loss_directional_rows(Ctx& ctx, int loss, const float* P, const float* Z, const int32_t* y,
                                  const float* target, const float* Rz, long long ld, int rows, int C,
                                  float* c) {
  if (rows <= 0) return;
  Launch l(ctx, BETTY_K_LOSS);
  loss_directional_rows_kernel<<<(rows + 3) / 4, 256, 0, ctx.stream>>>(loss, P, Z, y, target, Rz, ld, rows, C, c);
}

// one block per hidden unit (and one for the output bias): fixed-order sums over the samples
__global__ __launch_bounds__(256) void wnet_theta_vjp_kernel(const float* ell, const float* dsig,
                                                             const float* cvec, const float* theta, int H,
                                                             int rows, float inv_batch, float* out) {
  __shared__ float red[4];
  const int j = blockIdx.x;
  float a1 = 0.f, a2 = 0.f, a3 = 0.f;
  if (j < H) {
    const float u1 = theta[j], b1 = theta[H + j], u2 = theta[2 * H + j];
    for (int i = threadIdx.x; i < rows; i += 256) {
      const float ds = cvec[i] * dsig[i];
      const float pre = u1 * ell[i] + b1;
      const float on = pre > 0.f ? 1.f : 0.f;
      a1 += ds * u2 * on * ell[i];
      a2 += ds * u2 * on;
      a3 += ds * fmaxf(pre, 0.f);
    }
    a1 = block_sum(a1, red); a2 = block_sum(a2, red); a3 = block_sum(a3, red);
    if (threadIdx.x == 0) {
      out[j] = -inv_batch * a1; out[H + j] = -inv_batch * a2; out[2 * H + j] = -inv_batch * a3;
    }
  } else {
    for (int i = threadIdx.x; i < rows; i += 256) a1 += cvec[i] * dsig[i];
    a1 = block_sum(a1, red);
    if (threadIdx.x == 0) out[3 * H] = -inv_batch * a1;
  }
}

void launch_wnet_theta_vjp(Ctx& ctx, const float* ell, const float* dsig, const float* c,
                           const float* theta, int hidden, int rows, float inv_batch, float* out) {
  Launch l(ctx, BETTY_K_WNET);
  wnet_theta_vjp_kernel<<<hidden + 1, 256, 0, ctx.stream>>>(ell, dsig, c, theta, hidden, rows, inv_batch, out);
}

// ------------------------------------------------------------------------------------------
// streaming kernels over flat vectors
// ------------------------------------------------------------------------------------------

static inline unsigned flat_grid(size_t n) {
  size_t b = (n + 255) / 256;
  if (b > 8192) b = 8192;
  if (b < 1) b = 1;
  return (unsigned)b;
}

#define FLAT_LOOP(i, n) \
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < (n); i += (size_t)gridDim.x * 256)

__global__ __launch_bounds__(256) void fill_zero_kernel(uint4* p, size_t n16) {
  FLAT_LOOP(i, n16) p[i] = make_uint4(0, 0, 0, 0);
}
void launch_fill_zero(Ctx& ctx, void* p, size_t bytes) {
  if (!bytes) return;
  Launch l(ctx, BETTY_K_OTHER, 0, (double)bytes);
  fill_zero_kernel<<<flat_grid(bytes / 16), 256, 0, ctx.stream>>>((uint4*)p, bytes / 16);
}

__global__ __launch_bounds__(256) void scale_copy_kernel(const float* src, float scale, float* dst, size_t n) {
  FLAT_LOOP(i, n) dst[i] = scale * src[i];
}
void launch_scale_copy(Ctx& ctx, const float* src, float scale, float* dst, size_t n) {
  Launch l(ctx, BETTY_K_VECTOR, 0, 8.0 * n);
  scale_copy_kernel<<<flat_grid(n), 256, 0, ctx.stream>>>(src, scale, dst, n);
}

__global__ __launch_bounds__(256) void mixed_l2_kernel(const float* lam, const float* w, const float* p, float alpha, float* out, size_t n) {
  FLAT_LOOP(i, n) out[i] = -2.f * expf(lam[i]) * w[i] * (alpha * p[i]);
}
void launch_mixed_l2(Ctx& ctx, const float* lam, const float* w, const float* p, float alpha, float* out, size_t n) {
  Launch l(ctx, BETTY_K_VECTOR, 0, 16.0 * n);
  mixed_l2_kernel<<<flat_grid(n), 256, 0, ctx.stream>>>(lam, w, p, alpha, out, n);
}

__global__ __launch_bounds__(256) void mixed_prox_kernel(const float* logrho, const float* p, float alpha, float* out, size_t n) {
  FLAT_LOOP(i, n) out[i] = 2.f * expf(logrho[i]) * (alpha * p[i]);
}
void launch_mixed_prox(Ctx& ctx, const float* logrho, const float* p, float alpha, float* out, size_t n) {
  Launch l(ctx, BETTY_K_VECTOR, 0, 12.0 * n);
  mixed_prox_kernel<<<flat_grid(n), 256, 0, ctx.stream>>>(logrho, p, alpha, out, n);
}

__global__ __launch_bounds__(256) void diff_kernel(const float* a, const float* b, float* out, size_t n) {
  FLAT_LOOP(i, n) out[i] = a[i] - b[i];
}
void launch_diff(Ctx& ctx, const float* a, const float* b, float* out, size_t n) {
  Launch l(ctx, BETTY_K_VECTOR, 0, 12.0 * n);
  diff_kernel<<<flat_grid(n), 256, 0, ctx.stream>>>(a, b, out, n);
}

__global__ __launch_bounds__(256) void fill_value_kernel(float* p, float value, size_t n) {
  FLAT_LOOP(i, n) p[i] = value;
}
void launch_fill_value(Ctx& ctx, float* p, float value, size_t n) {
  if (n == 0) return;
  Launch l(ctx, BETTY_K_VECTOR, 0, 4.0 * n);
  fill_value_kernel<<<flat_grid(n), 256, 0, ctx.stream>>>(p, value, n);
}

// two-stage deterministic reductions: per-block partials, then one block in fixed order
constexpr int RED_BLOCKS = 1024;

template <int MODE>   // 0: sum x^2   1: sum exp(lam) x^2   2: sum lam x  (lam = second vector)
__global__ __launch_bounds__(256) void reduce_stage1_kernel(const float* lam, const float* x, size_t n, double* partials) {
  __shared__ double red[4];
  float acc = 0.f;
  double dacc = 0.0;
  int cnt = 0;
  FLAT_LOOP(i, n) {
    const float xi = x[i];
    acc += MODE == 0 ? xi * xi : MODE == 1 ? expf(lam[i]) * xi * xi : lam[i] * xi;
    if (++cnt == 64) { dacc += acc; acc = 0.f; cnt = 0; }
  }
  dacc += acc;
  dacc = block_sum(dacc, red);
  if (threadIdx.x == 0) partials[blockIdx.x] = dacc;
}

__global__ __launch_bounds__(256) void reduce_stage2_kernel(const double* partials, int nb, float* out) {
  __shared__ double red[4];
  double acc = 0.0;
  for (int i = threadIdx.x; i < nb; i += 256) acc += partials[i];
  acc = block_sum(acc, red);
  if (threadIdx.x == 0) out[0] = (float)acc;
}

static void launch_reduce(Ctx& ctx, int mode, const float* lam, const float* x, size_t n, double* partials, float* out) {
  unsigned nb = flat_grid(n);
  if (nb > RED_BLOCKS) nb = RED_BLOCKS;
  {
    Launch l(ctx, BETTY_K_REDUCE, 0, (mode ? 8.0 : 4.0) * n);
    if (mode == 0) reduce_stage1_kernel<0><<<nb, 256, 0, ctx.stream>>>(lam, x, n, partials);
    else if (mode == 1) reduce_stage1_kernel<1><<<nb, 256, 0, ctx.stream>>>(lam, x, n, partials);
    else reduce_stage1_kernel<2><<<nb, 256, 0, ctx.stream>>>(lam, x, n, partials);
  }
  {
    Launch l(ctx, BETTY_K_REDUCE);
    reduce_stage2_kernel<<<1, 256, 0, ctx.stream>>>(partials, (int)nb, out);
  }
}
void launch_sumsq(Ctx& ctx, const float* x, size_t n, double* partials, float* out) {
  launch_reduce(ctx, 0, nullptr, x, n, partials, out);
}
void launch_l2_cost(Ctx& ctx, const float* lam, const float* w, size_t n, double* partials, float* out) {
  launch_reduce(ctx, 1, lam, w, n, partials, out);
}
void launch_dot(Ctx& ctx, const float* x, const float* y, size_t n, double* partials, float* out) {
  launch_reduce(ctx, 2, y, x, n, partials, out);
}

// ---- conjugate gradient (scalars stay on the device; nothing here reads them on the host)
__global__ __launch_bounds__(256) void cg_init_kernel(const float* r, float* d, float* q, size_t n) {
  FLAT_LOOP(i, n) { d[i] = r[i]; q[i] = 0.f; }
}
void launch_cg_init(Ctx& ctx, const float* r, float* d, float* q, size_t n) {
  Launch l(ctx, BETTY_K_VECTOR, 0, 12.0 * n);
  cg_init_kernel<<<flat_grid(n), 256, 0, ctx.stream>>>(r, d, q, n);
}

__global__ __launch_bounds__(256) void cg_step_kernel(float* q, float* r, const float* d, const float* Hd,
                                                      const float* rs, const float* dHd, size_t n, double* partials) {
  __shared__ double red[4];
  const float num = rs[0], den = dHd[0];
  const float a = (num != 0.f && den != 0.f) ? num / den : 0.f;
  float acc = 0.f;
  double dacc = 0.0;
  int cnt = 0;
  FLAT_LOOP(i, n) {
    q[i] += a * d[i];
    const float ri = r[i] - a * Hd[i];
    r[i] = ri;
    acc += ri * ri;
    if (++cnt == 64) { dacc += acc; acc = 0.f; cnt = 0; }
  }
  dacc += acc;
  dacc = block_sum(dacc, red);
  if (threadIdx.x == 0) partials[blockIdx.x] = dacc;
}
void launch_cg_step(Ctx& ctx, float* q, float* r, const float* d, const float* Hd, const float* rs, const float* dHd,
                    size_t n, double* partials, float* rs_new) {
  unsigned nb = flat_grid(n);
  if (nb > RED_BLOCKS) nb = RED_BLOCKS;
  {
    Launch l(ctx, BETTY_K_VECTOR, 0, 24.0 * n);
    cg_step_kernel<<<nb, 256, 0, ctx.stream>>>(q, r, d, Hd, rs, dHd, n, partials);
  }
  {
    Launch l(ctx, BETTY_K_REDUCE);
    reduce_stage2_kernel<<<1, 256, 0, ctx.stream>>>(partials, (int)nb, rs_new);
  }
}

__global__ __launch_bounds__(256) void cg_dir_kernel(float* d, const float* r, const float* rs, const float* rs_new, size_t n) {
  const float den = rs[0];
  const float beta = den != 0.f ? rs_new[0] / den : 0.f;
  FLAT_LOOP(i, n) d[i] = r[i] + beta * d[i];
}
void launch_cg_dir(Ctx& ctx, float* d, const float* r, const float* rs, const float* rs_new, size_t n) {
  Launch l(ctx, BETTY_K_VECTOR, 0, 12.0 * n);
  cg_dir_kernel<<<flat_grid(n), 256, 0, ctx.stream>>>(d, r, rs, rs_new, n);
}

// Adam on the upper parameters: bias1 = 1 - beta1^t, bias2 = 1 - beta2^t are formed on the host
__global__ __launch_bounds__(256) void adam_kernel(float* x, const float* g, float* m, float* v, float lr, float beta1,
                                                   float beta2, float eps, float bias1, float bias2, size_t n) {
  FLAT_LOOP(i, n) {
    const float gi = g[i];
    const float mi = beta1 * m[i] + (1.f - beta1) * gi;
    const float vi = beta2 * v[i] + (1.f - beta2) * gi * gi;
    m[i] = mi;
    v[i] = vi;
    x[i] -= lr * (mi / bias1) / (sqrtf(vi / bias2) + eps);
  }
}
void launch_adam(Ctx& ctx, float* x, const float* g, float* m, float* v, float lr, float beta1, float beta2, float eps,
                 float bias1, float bias2, size_t n) {
  Launch l(ctx, BETTY_K_VECTOR, 0, 28.0 * n);
  adam_kernel<<<flat_grid(n), 256, 0, ctx.stream>>>(x, g, m, v, lr, beta1, beta2, eps, bias1, bias2, n);
}

__global__ __launch_bounds__(256) void fd_loss_diff_kernel(const float* lp, const float* lm, const float* eps_dev, int rows, float* c) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= rows) return;
  const float e = eps_dev[0];
  c[i] = e > 0.f ? (lp[i] - lm[i]) / (2.f * e) : 0.f;
}
void launch_fd_loss_diff(Ctx& ctx, const float* lp, const float* lm, const float* eps_dev, int rows, float* c) {
  if (rows <= 0) return;
  Launch l(ctx, BETTY_K_OTHER);
  fd_loss_diff_kernel<<<(rows + 255) / 256, 256, 0, ctx.stream>>>(lp, lm, eps_dev, rows, c);
}

__global__ __launch_bounds__(256) void weighted_loss_sum_kernel(const float* s, const float* ell, int rows, const float* add, float* out) {
  __shared__ double red[4];
  double acc = 0.0;
  for (int i = threadIdx.x; i < rows; i += 256) acc += (double)s[i] * (double)ell[i];
  acc = block_sum(acc, red);
  if (threadIdx.x == 0) out[0] = (float)(acc + (add ? (double)add[0] : 0.0));
}
void launch_weighted_loss_sum(Ctx& ctx, const float* s, const float* ell, int rows, const float* add, float* out) {
  Launch l(ctx, BETTY_K_REDUCE);
  weighted_loss_sum_kernel<<<1, 256, 0, ctx.stream>>>(s, ell, rows, add, out);
}

__global__ void fd_eps_kernel(const float* nrm2, float eps_scale, float vscale, float* eps_dev) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    const float nrm = sqrtf(nrm2[0]) * fabsf(vscale);
    eps_dev[0] = nrm > 0.f ? eps_scale / nrm : 0.f;
  }
}
void launch_fd_eps(Ctx& ctx, const float* nrm2, float eps_scale, float vscale, float* eps_dev) {
  Launch l(ctx, BETTY_K_OTHER);
  fd_eps_kernel<<<1, 64, 0, ctx.stream>>>(nrm2, eps_scale, vscale, eps_dev);
}

__global__ __launch_bounds__(256) void fd_perturb_kernel(const float* w, const float* v, const float* eps_dev, float sign, float* out, size_t n) {
  const float e = sign * eps_dev[0];
  FLAT_LOOP(i, n) out[i] = w[i] + e * v[i];
}
void launch_fd_perturb(Ctx& ctx, const float* w, const float* v, const float* eps_dev, float sign, float* out, size_t n) {
  Launch l(ctx, BETTY_K_VECTOR, 0, 12.0 * n);
  fd_perturb_kernel<<<flat_grid(n), 256, 0, ctx.stream>>>(w, v, eps_dev, sign, out, n);
}

__global__ __launch_bounds__(256) void fd_update_kernel(float* v, float* p, const float* Gp, const float* Gm, const float* eps_dev, float alpha, size_t n) {
  const float e = eps_dev[0];
  const float k = e > 0.f ? alpha / (2.f * e) : 0.f;     // v = 0 has the zero product
  FLAT_LOOP(i, n) {
    const float vn = v[i] - k * (Gp[i] - Gm[i]);
    v[i] = vn;
    p[i] += vn;
  }
}
void launch_fd_update(Ctx& ctx, float* v, float* p, const float* Gp, const float* Gm, const float* eps_dev, float alpha, size_t n) {
  Launch l(ctx, BETTY_K_VECTOR, 0, 24.0 * n);
  fd_update_kernel<<<flat_grid(n), 256, 0, ctx.stream>>>(v, p, Gp, Gm, eps_dev, alpha, n);
}

// central difference of grad_lambda (e^lam w^2) along q = alpha p, formed in fp64 registers so
// that the subtraction of the two squares does not lose the signal
__global__ __launch_bounds__(256) void mixed_l2_fd_kernel(const float* lam, const float* w, const float* p, float alpha, const float* eps_dev, float* out, size_t n) {
  const double e = (double)eps_dev[0];
  FLAT_LOOP(i, n) {
    if (e > 0.0) {
      const double q = (double)alpha * (double)p[i], wi = (double)w[i], el = exp((double)lam[i]);
      const double up = wi + e * q, dn = wi - e * q;
      out[i] = (float)(-(el * up * up - el * dn * dn) / (2.0 * e));
    } else {
      out[i] = 0.f;
    }
  }
}
void launch_mixed_l2_fd(Ctx& ctx, const float* lam, const float* w, const float* p, float alpha, const float* eps_dev, float* out, size_t n) {
  Launch l(ctx, BETTY_K_VECTOR, 0, 16.0 * n);
  mixed_l2_fd_kernel<<<flat_grid(n), 256, 0, ctx.stream>>>(lam, w, p, alpha, eps_dev, out, n);
}

__global__ __launch_bounds__(256) void label_noise_kernel(const int32_t* y, const uint32_t* words, const int32_t* alt,
                                                          unsigned long long threshold, int n, int32_t* y_out, uint8_t* mask) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const bool hit = (unsigned long long)words[i] < threshold;
  y_out[i] = hit ? alt[i] : y[i];
  if (mask) mask[i] = hit ? 1 : 0;
}
void launch_label_noise(Ctx& ctx, const int32_t* y, const uint32_t* words, const int32_t* alt,
                        unsigned long long threshold, int n, int32_t* y_out, uint8_t* mask) {
  if (n <= 0) return;
  Launch l(ctx, BETTY_K_OTHER);
  label_noise_kernel<<<(n + 255) / 256, 256, 0, ctx.stream>>>(y, words, alt, threshold, n, y_out, mask);
}

}  // namespace betty

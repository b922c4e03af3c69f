// Non-GEMM kernels of the hypergradient path: fused epilogues that turn fp32 GEMM output
// (optionally split-K partials) into the next GEMM's operands in both orientations, the
// row-wise loss kernels, the weight-net kernels, and the streaming kernels over the flat
// parameter-shaped vectors (Neumann recurrence, finite-difference steps, mixed VJP).
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

// phi, phi', phi'' ; GELU is the exact erf form, ReLU has derivative 0 at 0
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

__device__ __forceinline__ float split_sum(const SplitSrc& s, int r, int c) {
  const float* p = s.part + (long long)r * s.ld + c;
  float t = p[0];
  for (int k = 1; k < s.S; ++k) t += p[(long long)k * s.stride];
  return t;
}

// ------------------------------------------------------------------------------------------
// 64x64 tile kernel: value f(r, c) -> row-major `out` and transposed `outT`
// ------------------------------------------------------------------------------------------

template <typename T, typename F>
__global__ __launch_bounds__(256) void tile_dual_kernel(F f, int rows, int cols, T* out, int ld,
                                                        T* outT, int ldT) {
  __shared__ float tile[64][65];
  const int c0 = blockIdx.x * 64, r0 = blockIdx.y * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
#pragma unroll 4
  for (int i = 0; i < 16; ++i) {
    const int r = r0 + ty + 4 * i, c = c0 + tx;
    float val = 0.f;
    if (r < rows && c < cols) {
      val = f(r, c);
      if (out) out[(long long)r * ld + c] = from_float<T>(val);
    }
    tile[ty + 4 * i][tx] = val;
  }
  if (!outT) return;
  __syncthreads();
#pragma unroll 4
  for (int i = 0; i < 16; ++i) {
    const int c = c0 + ty + 4 * i, r = r0 + tx;
    if (r < rows && c < cols) outT[(long long)c * ldT + r] = from_float<T>(tile[tx][ty + 4 * i]);
  }
}

template <typename F>
static void launch_tile_dual(Ctx& ctx, Elem elem, int kind, double bytes, F f, int rows, int cols,
                             void* out, int ld, void* outT, int ldT) {
  if (rows <= 0 || cols <= 0) return;
  dim3 grid((cols + 63) / 64, (rows + 63) / 64);
  Launch l(ctx, kind, 0, bytes);
  if (elem == ELEM_BF16)
    tile_dual_kernel<__bf16, F><<<grid, 256, 0, ctx.stream>>>(f, rows, cols, (__bf16*)out, ld, (__bf16*)outT, ldT);
  else
    tile_dual_kernel<float, F><<<grid, 256, 0, ctx.stream>>>(f, rows, cols, (float*)out, ld, (float*)outT, ldT);
}

struct FwdEpi {
  SplitSrc src; const float* bias; int act; int last;
  float* z; float* dphi; float* d2phi; long long ldf;
  __device__ float operator()(int r, int c) const {
    float zz = split_sum(src, r, c);
    if (bias) zz += bias[c];
    const long long o = (long long)r * ldf + c;
    if (last) { z[o] = zz; return zz; }
    float a, d1, d2;
    act_eval(act, zz, a, d1, d2);
    dphi[o] = d1;
    if (d2phi) d2phi[o] = d2;
    return a;
  }
};

void launch_fwd_epilogue(Ctx& ctx, Elem elem, SplitSrc src, const float* bias, int act, bool last,
                         int rows, int cols, float* z_out, float* dphi, float* d2phi, long long ldf,
                         void* out, int ld, void* outT, int ldT) {
  FwdEpi f{src, bias, act, last ? 1 : 0, z_out, dphi, d2phi, ldf};
  launch_tile_dual(ctx, elem, BETTY_K_EPILOGUE, 0, f, rows, cols, last ? nullptr : out, ld,
                   last ? nullptr : outT, ldT);
}

struct BwdEpi {
  SplitSrc src; const float* dphi; float* e; long long ldf;
  __device__ float operator()(int r, int c) const {
    const float t = split_sum(src, r, c);
    const long long o = (long long)r * ldf + c;
    if (e) e[o] = t * e[o];
    return t * dphi[o];
  }
};

void launch_bwd_epilogue(Ctx& ctx, Elem elem, SplitSrc src, const float* dphi, float* e,
                         long long ldf, int rows, int cols, void* out, int ld, void* outT, int ldT) {
  BwdEpi f{src, dphi, e, ldf};
  launch_tile_dual(ctx, elem, BETTY_K_EPILOGUE, 0, f, rows, cols, out, ld, outT, ldT);
}

struct RFwdEpi {
  SplitSrc src; const float* cb; int last; const float* dphi; float* Rz; long long ldf;
  __device__ float operator()(int r, int c) const {
    float rz = split_sum(src, r, c);
    if (cb) rz += cb[c];
    const long long o = (long long)r * ldf + c;
    Rz[o] = rz;
    return last ? rz : dphi[o] * rz;
  }
};

void launch_rfwd_epilogue(Ctx& ctx, Elem elem, SplitSrc src, const float* cb, bool last,
                          const float* dphi, float* Rz, long long ldf, int rows, int cols, void* out,
                          int ld, void* outT, int ldT) {
  RFwdEpi f{src, cb, last ? 1 : 0, dphi, Rz, ldf};
  launch_tile_dual(ctx, elem, BETTY_K_EPILOGUE, 0, f, rows, cols, last ? nullptr : out, ld,
                   last ? nullptr : outT, ldT);
}

struct RBwdEpi {
  SplitSrc src; const float* dphi; const float* e; const float* Rz; long long ldf;
  __device__ float operator()(int r, int c) const {
    const float t = split_sum(src, r, c);
    const long long o = (long long)r * ldf + c;
    float out = t * dphi[o];
    if (e) out += e[o] * Rz[o];
    return out;
  }
};

void launch_rbwd_epilogue(Ctx& ctx, Elem elem, SplitSrc src, const float* dphi, const float* e,
                          const float* Rz, long long ldf, int rows, int cols, void* out, int ld,
                          void* outT, int ldT) {
  RBwdEpi f{src, dphi, e, Rz, ldf};
  launch_tile_dual(ctx, elem, BETTY_K_EPILOGUE, 0, f, rows, cols, out, ld, outT, ldT);
}

struct ConvertSrc {
  const float* src; long long lds; float scale;
  __device__ float operator()(int r, int c) const { return scale * src[(long long)r * lds + c]; }
};

void launch_convert_dual(Ctx& ctx, Elem elem, const float* src, long long lds, float scale,
                         int rows, int cols, void* out, int ld, void* outT, int ldT) {
  ConvertSrc f{src, lds, scale};
  const double bytes = (double)rows * cols * (4.0 + 2.0 * elem_size(elem));
  launch_tile_dual(ctx, elem, BETTY_K_SHADOW, bytes, f, rows, cols, out, ld, outT, ldT);
}

// ------------------------------------------------------------------------------------------
// row-wise loss kernels: one wavefront per sample
// ------------------------------------------------------------------------------------------

__global__ __launch_bounds__(256) void loss_rows_kernel(LossArgs a) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
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
    y = a.y[row];
    const int yy = min(max(y, 0), a.C - 1);      // integer gather of the label's logit
    ell = logf(sum) + m - z[yy];
  } else {
    const float* t = a.target + (long long)row * a.C;
    float acc = 0.f;
    for (int c = lane; c < a.C; c += 64) { const float r = z[c] - t[c]; acc += r * r; }
    ell = wave_sum(acc);
  }
  float omega = 1.f;
  if (a.reweight) {
    const int H = a.hidden;
    float part = 0.f;
    for (int j = lane; j < H; j += 64)
      part += a.theta[2 * H + j] * fmaxf(a.theta[j] * ell + a.theta[H + j], 0.f);
    part = wave_sum(part) + a.theta[3 * H];
    omega = 1.f / (1.f + expf(-part));
  }
  const float s = omega * a.inv_batch;
  if (lane == 0) { a.ell[row] = ell; a.s[row] = s; a.omega[row] = omega; }
  float* dz = a.dZ + (long long)row * a.lddz;
  if (a.loss == BETTY_LOSS_SOFTMAX_CE) {
    float* P = a.P + (long long)row * a.ldz;
    const float inv = 1.f / sum;
    for (int c = lane; c < a.C; c += 64) {
      const float p = expf(z[c] - m) * inv;
      P[c] = p;
      dz[c] = s * (p - (c == y ? 1.f : 0.f));
    }
  } else {
    const float* t = a.target + (long long)row * a.C;
    for (int c = lane; c < a.C; c += 64) dz[c] = s * 2.f * (z[c] - t[c]);
  }
}

void launch_loss_rows(Ctx& ctx, const LossArgs& a) {
  if (a.rows <= 0) return;
  Launch l(ctx, BETTY_K_LOSS);
  loss_rows_kernel<<<(a.rows + 3) / 4, 256, 0, ctx.stream>>>(a);
}

__global__ __launch_bounds__(256) void loss_hessian_rows_kernel(int loss, const float* P, const float* Rz,
                                                                long long ld, const float* s, int rows,
                                                                int C, float* out, long long ldo) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= rows) return;
  const float* rz = Rz + (long long)row * ld;
  float* o = out + (long long)row * ldo;
  const float si = s[row];
  if (loss == BETTY_LOSS_SOFTMAX_CE) {
    const float* p = P + (long long)row * ld;
    float dot = 0.f;
    for (int c = lane; c < C; c += 64) dot += p[c] * rz[c];
    dot = wave_sum(dot);
    for (int c = lane; c < C; c += 64) o[c] = si * (p[c] * rz[c] - p[c] * dot);
  } else {
    for (int c = lane; c < C; c += 64) o[c] = si * 2.f * rz[c];
  }
}

void launch_loss_hessian_rows(Ctx& ctx, int loss, const float* P, const float* Rz, long long ld,
                              const float* s, int rows, int C, float* out, long long ldo) {
  if (rows <= 0) return;
  Launch l(ctx, BETTY_K_LOSS);
  loss_hessian_rows_kernel<<<(rows + 3) / 4, 256, 0, ctx.stream>>>(loss, P, Rz, ld, s, rows, C, out, ldo);
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

void launch_loss_directional_rows(Ctx& ctx, int loss, const float* P, const float* Z, const int32_t* y,
                                  const float* target, const float* Rz, long long ld, int rows, int C,
                                  float* c) {
  if (rows <= 0) return;
  Launch l(ctx, BETTY_K_LOSS);
  loss_directional_rows_kernel<<<(rows + 3) / 4, 256, 0, ctx.stream>>>(loss, P, Z, y, target, Rz, ld, rows, C, c);
}

// one block per hidden unit (and one for the output bias): fixed-order sums over the samples
__global__ __launch_bounds__(256) void wnet_theta_vjp_kernel(const float* ell, const float* omega,
                                                             const float* cvec, const float* theta, int H,
                                                             int rows, float inv_batch, float* out) {
  __shared__ float red[4];
  const int j = blockIdx.x;
  float a1 = 0.f, a2 = 0.f, a3 = 0.f;
  if (j < H) {
    const float u1 = theta[j], b1 = theta[H + j], u2 = theta[2 * H + j];
    for (int i = threadIdx.x; i < rows; i += 256) {
      const float om = omega[i], ds = cvec[i] * om * (1.f - om);
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
    for (int i = threadIdx.x; i < rows; i += 256) {
      const float om = omega[i];
      a1 += cvec[i] * om * (1.f - om);
    }
    a1 = block_sum(a1, red);
    if (threadIdx.x == 0) out[3 * H] = -inv_batch * a1;
  }
}

void launch_wnet_theta_vjp(Ctx& ctx, const float* ell, const float* omega, const float* c,
                           const float* theta, int hidden, int rows, float inv_batch, float* out) {
  Launch l(ctx, BETTY_K_WNET);
  wnet_theta_vjp_kernel<<<hidden + 1, 256, 0, ctx.stream>>>(ell, omega, c, theta, hidden, rows, inv_batch, out);
}

template <typename T>
__global__ __launch_bounds__(256) void row_sums_kernel(const T* M, int ld, int rows, int k, float* out) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= rows) return;
  const T* p = M + (long long)row * ld;
  float acc = 0.f;
  for (int c = lane; c < k; c += 64) acc += to_float(p[c]);
  acc = wave_sum(acc);
  if (lane == 0) out[row] = acc;
}

void launch_row_sums(Ctx& ctx, Elem elem, const void* M, int ld, int rows, int k, float* out) {
  if (rows <= 0) return;
  Launch l(ctx, BETTY_K_REDUCE);
  if (elem == ELEM_BF16)
    row_sums_kernel<__bf16><<<(rows + 3) / 4, 256, 0, ctx.stream>>>((const __bf16*)M, ld, rows, k, out);
  else
    row_sums_kernel<float><<<(rows + 3) / 4, 256, 0, ctx.stream>>>((const float*)M, ld, rows, k, out);
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

__global__ __launch_bounds__(256) void copy2_kernel(const float* src, float* a, float* b, size_t n) {
  FLAT_LOOP(i, n) { const float x = src[i]; a[i] = x; b[i] = x; }
}
void launch_copy2(Ctx& ctx, const float* src, float* a, float* b, size_t n) {
  Launch l(ctx, BETTY_K_VECTOR, 0, 12.0 * n);
  copy2_kernel<<<flat_grid(n), 256, 0, ctx.stream>>>(src, a, b, n);
}

__global__ __launch_bounds__(256) void scale_copy_kernel(const float* src, float scale, float* dst, size_t n) {
  FLAT_LOOP(i, n) dst[i] = scale * src[i];
}
void launch_scale_copy(Ctx& ctx, const float* src, float scale, float* dst, size_t n) {
  Launch l(ctx, BETTY_K_VECTOR, 0, 8.0 * n);
  scale_copy_kernel<<<flat_grid(n), 256, 0, ctx.stream>>>(src, scale, dst, n);
}

__global__ __launch_bounds__(256) void add_l2_term_kernel(float* out, const float* lam, const float* x, size_t n) {
  FLAT_LOOP(i, n) out[i] += 2.f * expf(lam[i]) * x[i];
}
void launch_add_l2_term(Ctx& ctx, float* out, const float* lam, const float* x, size_t n) {
  Launch l(ctx, BETTY_K_VECTOR, 0, 16.0 * n);
  add_l2_term_kernel<<<flat_grid(n), 256, 0, ctx.stream>>>(out, lam, x, n);
}

__global__ __launch_bounds__(256) void neumann_update_kernel(float* v, float* p, const float* Hv, float alpha, size_t n) {
  FLAT_LOOP(i, n) {
    const float vn = v[i] - alpha * Hv[i];
    v[i] = vn;
    p[i] += vn;
  }
}
void launch_neumann_update(Ctx& ctx, float* v, float* p, const float* Hv, float alpha, size_t n) {
  Launch l(ctx, BETTY_K_VECTOR, 0, 20.0 * n);
  neumann_update_kernel<<<flat_grid(n), 256, 0, ctx.stream>>>(v, p, Hv, alpha, n);
}

__global__ __launch_bounds__(256) void mixed_l2_kernel(const float* lam, const float* w, const float* p, float alpha, float* out, size_t n) {
  FLAT_LOOP(i, n) out[i] = -2.f * expf(lam[i]) * w[i] * (alpha * p[i]);
}
void launch_mixed_l2(Ctx& ctx, const float* lam, const float* w, const float* p, float alpha, float* out, size_t n) {
  Launch l(ctx, BETTY_K_VECTOR, 0, 16.0 * n);
  mixed_l2_kernel<<<flat_grid(n), 256, 0, ctx.stream>>>(lam, w, p, alpha, out, n);
}

// two-stage deterministic reductions: per-block partials, then one block in fixed order
constexpr int RED_BLOCKS = 1024;

template <int MODE>   // 0: sum x^2   1: sum exp(lam) x^2
__global__ __launch_bounds__(256) void reduce_stage1_kernel(const float* lam, const float* x, size_t n, double* partials) {
  __shared__ double red[4];
  float acc = 0.f;
  double dacc = 0.0;
  int cnt = 0;
  FLAT_LOOP(i, n) {
    const float xi = x[i];
    acc += MODE == 0 ? xi * xi : expf(lam[i]) * xi * xi;
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
    else reduce_stage1_kernel<1><<<nb, 256, 0, ctx.stream>>>(lam, x, n, partials);
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

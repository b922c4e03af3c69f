// Internal declarations shared by the translation units of libbetty_hip.so.
// Nothing here is part of the public ABI (see include/betty_hip.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "betty_hip.h"

namespace betty {

// Every operand matrix of a GEMM lives in the workspace as [rows_p][k_p] with both extents
// rounded up to PAD and the padding zero-filled, so the GEMM main loop needs no bounds
// checks.  PAD is a multiple of every tile extent used by the kernels.
constexpr int PAD = 128;
inline int padup(int n) { return (n + PAD - 1) / PAD * PAD; }

enum Elem { ELEM_F32 = 0, ELEM_BF16 = 1 };
inline size_t elem_size(Elem e) { return e == ELEM_F32 ? 4 : 2; }

// C (fp32) = sum over up to two operand pairs of A_p (M x K_p) * B_p^T (B_p is N x K_p).
// Both operands are "K-major": element (row, k) at base[row * ld + k].
struct GemmArgs {
  const void* A[2];
  const void* B[2];
  int lda[2], ldb[2];        // leading dimensions in elements
  int Kp[2];                 // padded reduction extents in elements; 0 = pair absent
  float* C;
  long long ldc;
  int M, N;                  // valid output extent (stores are bounds-checked against it)
  int Mp, Np;                // padded extents (define the grid)
  int splitk;                // number of K slices; slice s writes C + s * split_stride
  long long split_stride;
};

// Launch context: stream + optional per-launch event timing.
struct ProfRec { int kind; double flops, bytes; hipEvent_t e0, e1; float ms; };
struct Ctx {
  hipStream_t stream = nullptr;
  bool profiling = false;
  std::vector<ProfRec> recs;
  hipError_t first_error = hipSuccess;
  void begin(int kind, double flops, double bytes);
  void end();
};

struct Launch {   // RAII bracket around one kernel launch
  Ctx& c;
  Launch(Ctx& ctx, int kind, double flops = 0, double bytes = 0) : c(ctx) { c.begin(kind, flops, bytes); }
  ~Launch() { c.end(); }
};

// ---- gemm.hip
void launch_gemm(Ctx& ctx, Elem elem, const GemmArgs& g, double algorithmic_flops);

// ---- kernels.hip : fused elementwise stages ------------------------------------------------
// "dual" outputs: out is [rows_p][ld] row-major, outT is [cols_p][ldT]; either may be null.

struct SplitSrc { const float* part; long long ld; int S; long long stride; };

// a = phi(sum_s part + bias); writes dphi (and d2phi for GELU) in fp32; last layer writes z only
void launch_fwd_epilogue(Ctx&, Elem, SplitSrc src, const float* bias_or_null, int act, bool last,
                         int rows, int cols, float* z_out_or_null, float* dphi, float* d2phi_or_null,
                         long long ldf, void* out, int ld, void* outT, int ldT);
// delta = t * dphi,  e = t * d2phi (in place over d2phi) with t = sum_s part
void launch_bwd_epilogue(Ctx&, Elem, SplitSrc src, const float* dphi, float* e_inout_or_null,
                         long long ldf, int rows, int cols, void* out, int ld, void* outT, int ldT);
// Rz = sum_s part + cbias; Ra = dphi * Rz (hidden layers)
void launch_rfwd_epilogue(Ctx&, Elem, SplitSrc src, const float* cbias_or_null, bool last,
                          const float* dphi_or_null, float* Rz, long long ldf, int rows, int cols,
                          void* out, int ld, void* outT, int ldT);
// Rdelta = t * dphi + e * Rz
void launch_rbwd_epilogue(Ctx&, Elem, SplitSrc src, const float* dphi, const float* e_or_null,
                          const float* Rz, long long ldf, int rows, int cols, void* out, int ld,
                          void* outT, int ldT);
// out/outT = convert(scale * src[r * lds + c])
void launch_convert_dual(Ctx&, Elem, const float* src, long long lds, float scale, int rows,
                         int cols, void* out, int ld, void* outT, int ldT);

// ---- kernels.hip : loss rows ---------------------------------------------------------------
struct LossArgs {
  int loss, reweight, hidden;
  const float* Z; long long ldz;        // logits [rows][ldz]
  const int32_t* y; const float* target; int C;
  const float* theta;                   // weight net (reweight only)
  int rows; float inv_batch;
  float* ell; float* s; float* omega;   // per-sample outputs
  float* P;                             // softmax probabilities [rows][ldz] (CE)
  float* dZ; long long lddz;            // s_i * dl_i/dz  (fp32 scratch)
};
void launch_loss_rows(Ctx&, const LossArgs&);
// Rdelta_L (fp32) = s_i * (d^2 l_i/dz^2) Rz_i
void launch_loss_hessian_rows(Ctx&, int loss, const float* P, const float* Rz, long long ld,
                              const float* s, int rows, int C, float* out, long long ldo);
// c_i = < dl_i/dz, Rz_i >
void launch_loss_directional_rows(Ctx&, int loss, const float* P, const float* Z, const int32_t* y,
                                  const float* target, const float* Rz, long long ld, int rows,
                                  int C, float* c);
// out = -(1/B) sum_i c_i dR(l_i; theta)/dtheta
void launch_wnet_theta_vjp(Ctx&, const float* ell, const float* omega, const float* c,
                           const float* theta, int hidden, int rows, float inv_batch, float* out);
// bias-shaped sums: out[r] = sum_k M[r][k]   (rows of a K-major operand matrix)
void launch_row_sums(Ctx&, Elem, const void* Mtx, int ld, int rows, int k, float* out);

// ---- kernels.hip : flat parameter-shaped vectors ------------------------------------------
void launch_fill_zero(Ctx&, void* p, size_t bytes);
void launch_copy2(Ctx&, const float* src, float* a, float* b, size_t n);
void launch_scale_copy(Ctx&, const float* src, float scale, float* dst, size_t n);
void launch_add_l2_term(Ctx&, float* out, const float* lam, const float* x, size_t n);   // out += 2 e^lam x
void launch_neumann_update(Ctx&, float* v, float* p, const float* Hv, float alpha, size_t n);
void launch_mixed_l2(Ctx&, const float* lam, const float* w, const float* p, float alpha, float* out, size_t n);
void launch_sumsq(Ctx&, const float* x, size_t n, double* partials, float* out_scalar);
void launch_l2_cost(Ctx&, const float* lam, const float* w, size_t n, double* partials, float* out_scalar);
void launch_weighted_loss_sum(Ctx&, const float* s, const float* ell, int rows, const float* add_or_null, float* out);
// eps_dev = eps_scale / sqrt(nrm2) (0 if nrm2 == 0);  out = w + sign * eps_dev * scale * v
void launch_fd_eps(Ctx&, const float* nrm2, float eps_scale, float vscale, float* eps_dev);
void launch_fd_perturb(Ctx&, const float* w, const float* v, const float* eps_dev, float sign, float* out, size_t n);
void launch_fd_update(Ctx&, float* v, float* p, const float* Gp, const float* Gm, const float* eps_dev, float alpha, size_t n);
void launch_mixed_l2_fd(Ctx&, const float* lam, const float* w, const float* p, float alpha, const float* eps_dev, float* out, size_t n);
void launch_label_noise(Ctx&, const int32_t* y, const uint32_t* words, const int32_t* alt,
                        unsigned long long threshold, int n, int32_t* y_out, uint8_t* mask);

}  // namespace betty

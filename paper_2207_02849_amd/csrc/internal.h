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

// Accumulators = sum over up to two operand pairs of A_p (M x K_p) * B_p^T (B_p is N x K_p).
// Both operands are "K-major": element (row, k) at base[row * ld + k].
struct GemmArgs {
  const void* A[2];
  const void* B[2];
  int lda[2], ldb[2];        // leading dimensions in elements
  int Kp[2];                 // padded reduction extents in elements; 0 = pair absent
  int M, N;                  // valid output extent (epilogue stores are bounds-checked against it)
  int Mp, Np;                // padded extents (define the tile grid)
  // Workgroups go to the eight XCDs round-robin, so tiles t, t+8, t+16, ... of a problem share an
  // L2.  With xgm x xgn = 8 those tiles are laid out as one compact (tiles_m/xgm) x (tiles_n/xgn)
  // rectangle, which cuts the operand panels each L2 has to fetch; 0 = row-major tile order.
  int xgm, xgn;
};

// What happens to a finished accumulator tile.
enum EpiMode {
  EPI_FWD = 1,             // z = acc + bias; out = phi(z); dphi_out = phi'(z); d2_out = phi''(z)
  EPI_FWD_LAST,          // f0 = acc + bias                       (logits)
  EPI_BWD,               // out = acc * dphi; e_io = acc * e_io   (delta of the layer below)
  EPI_RFWD,              // f0 = rz = acc + cbias; out = dphi * rz
  EPI_RFWD_LAST,         // f0 = acc + cbias
  EPI_RBWD,              // out = acc * dphi + e * Rz
  // Last layer of the R-forward with the loss Hessian applied in place (outputs of at most 32
  // columns, so that one MFMA block holds whole rows): rz = acc + cbias;
  // out = e[row] * (dphi .* rz - dphi * <dphi, rz>_row) for softmax cross-entropy (dphi = the
  // softmax probabilities, e = the per-sample scale), out = 2 e[row] rz for the squared error;
  // `act` carries the loss kind.
  EPI_RFWD_LAST_HESS,
  EPI_WGRAD,             // C = acc (+ 2 exp(lam) x)                       flat parameter layout
  EPI_WGRAD_INIT,        // v = acc (and p = acc when p is given); out = operand copies
  // One step of the Neumann partial sum in nested form, s_{j+1} = g + (I - alpha H) s_j with s_0 = g
  // (the same sum_{i<=j} (I - alpha H)^i g as the term-by-term recurrence, one state vector instead
  // of two): s is read from x, g from v;  Hs = acc (+ 2 exp(lam) s);  p = g + s - alpha Hs;  out =
  // operand copies of the new s.
  EPI_WGRAD_NEUMANN,
  EPI_WGRAD_NEUMANN_L2,  // last step for L2 decay: s read from p, new s kept in registers, C = -2 exp(lam) x (alpha s)
  EPI_WGRAD_SGD          // g = acc (+ 2 exp(lam) p) + gamma p; v <- beta v + g; p <- p - alpha v  (p = w, v = momentum)
};

struct Epilogue {
  int mode, act;
  const float* colvec;                   // per-column addend (bias or bias direction), may be null
  float* f0;                             // fp32 [row * ldf + col]
  float* dphi_out; float* d2_out;
  const float* dphi; float* e_io; const float* e; const float* Rz;
  long long ldf;
  void* out; int ld;                     // operand-typed, row-major [row][col]
  void* outT; int ldT;                   // operand-typed, transposed [col][row]
  void* out2; void* outT2;               // EPI_FWD only: further copies of `out` in bf16 (same ld, ldT), or null
  float* C; long long ldc;               // fp32 row-major (flat parameter slice for the WGRAD modes)
  const float* lam; const float* x;      // same indexing as C
  float* v; float* p; float alpha, beta, gamma;
};

struct GemmProblem { GemmArgs g; Epilogue e; };

// out[row] from sum_k Mt[row][k]: bias-shaped slices of the WGRAD modes
struct BiasJob {
  const void* Mt; int ld, rows, k, mode;
  float* C; const float* lam; const float* x; float* v; float* p; float alpha, beta, gamma;
};

constexpr int MAX_PROBLEMS = 8;
constexpr int GEMM_NCH = 8;              // 16-byte chunks per row of a k-tile
// tile extent x number of K groups per workgroup; a group is 2 x 2 wavefronts, except in 32x8
// (32-tile, eight groups of one wavefront)
enum { GEMM_128x1 = 0, GEMM_64x1 = 2, GEMM_64x4 = 3, GEMM_32x8 = 4, GEMM_128x64 = 5 };

struct GemmBatch {
  int n = 0, n_bias = 0, gemm_blocks = 0;
  int walkers = 0;                       // wgrad128_kernel: workgroups that walk the tiles (set by launch_gemm_batch)
  int block_begin[MAX_PROBLEMS + 1];
  int bias_begin[MAX_PROBLEMS + 1];
  GemmProblem p[MAX_PROBLEMS];
  BiasJob bias[MAX_PROBLEMS];
};
static_assert(sizeof(GemmBatch) <= 3584, "GemmBatch is passed by value as a kernel argument (4 KiB limit)");

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

// One 16-byte chunk of K for a 32 x 32 MFMA block: 8 bf16 (one v_mfma_f32_32x32x16_bf16) or 4 floats
// (four v_mfma_f32_32x32x2_f32).  Lane l supplies row l % 32 of A and of B; lanes 0-31 hold the
// even chunks of a chunk pair, lanes 32-63 the odd ones.  Register r of lane l of the result holds
// C[8*(r/4) + 4*(l/32) + r%4][l%32].
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));   // one 16-byte chunk

template <typename T> struct MfmaChunk;

template <> struct MfmaChunk<__bf16> {
  static __device__ __forceinline__ void run(const u32x4& a, const u32x4& b, f32x16& acc) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b),
                                                  acc, 0, 0, 0);
  }
};

template <> struct MfmaChunk<float> {
  static __device__ __forceinline__ void run(const u32x4& a, const u32x4& b, f32x16& acc) {
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
  }
};

// ---- gemm.hip
int gemm_ktile_elems(Elem elem);
int gemm_cfg_tile(int cfg);
void launch_gemm_batch(Ctx& ctx, Elem elem, int cfg, GemmBatch& batch, double algorithmic_flops,
                       double algorithmic_bytes = 0);

// ---- kernels.hip : operand conversion -----------------------------------------------------
// out (row-major [rows_p][ld]) and outT ([cols_p][ldT]) = convert(scale * src[r * lds + c]); either may be null
struct ConvertJob {
  const float* src; long long lds; float scale; int rows, cols;
  void* out; int ld; void* outT; int ldT;
  float* outT32 = nullptr;    // optional further transposed copy in fp32 (same ldT)
};
struct ConvertBatch {
  int n = 0;
  int block_begin[MAX_PROBLEMS + 1];
  ConvertJob j[MAX_PROBLEMS];
};
void launch_convert_batch(Ctx&, Elem, ConvertBatch&);
void launch_convert_dual(Ctx&, Elem, const float* src, long long lds, float scale, int rows,
                         int cols, void* out, int ld, void* outT, int ldT);

// ---- kernels.hip : loss rows ---------------------------------------------------------------
struct LossArgs {
  int loss, reweight, hidden;
  const float* Z; long long ldz;        // logits [rows][ldz]
  const int32_t* y; const float* target; int C;
  const float* theta;                   // weight net (reweight only)
  const float* omega_fixed;             // reweight only: use these weights instead of R(l_i; theta)
  int rows; float inv_batch;
  float* ell; float* s; float* omega;   // per-sample outputs
  float* dsig;                          // omega_i (1 - omega_i), formed without cancellation (weight net evaluated here only)
  float* P;                             // softmax probabilities [rows][ldz] (CE)
  void* D; int ldD; void* Dt; int ldDt;  // s_i * dl_i/dz as GEMM operands, both orientations
};
struct LossBatch { int n = 0; LossArgs a[2]; };     // up to two batches (train, validation) per launch
void launch_loss_rows(Ctx&, Elem, const LossBatch&);
// Rdelta_L (fp32) = s_i * (d^2 l_i/dz^2) Rz_i
// The last layer of the R-op passes when the network output is narrow (at most 16 columns): one
// launch computes Rz_L = Ra_{L-1} W_L + a_{L-1} V_L + c_L, applies the loss Hessian (R delta_L) and
// propagates through the last layer, R delta_{L-1} = (R delta_L W_L^T + delta_L V_L^T) .* phi'
// + e2 .* Rz_{L-1}, with plain vector arithmetic (the products have 16 or fewer columns or
// reduction terms, a poor fit for 32-wide MFMA tiles).
struct LastRopArgs {
  const void* RA; const void* A; int lda;               // Ra_{L-1}, a_{L-1}: [B][n_in_p], operand type
  const void* Wt; const void* Vt; int ldt;              // W_L, V_L as [n_out_p][n_in_p]
  const void* Wn; const void* Vn; int ldn;              // W_L, V_L as [n_in_p][n_out_p]
  const float* cbias;                                   // bias direction of the last layer, or null
  const float* P; const float* s; int ldp;              // softmax probabilities [B][ldp], per-sample scale
  const void* DL; int ldd;                              // delta_L [B][ldd], operand type
  const float* dphi; const float* e2; const float* Rz; int ldf;   // layer L-1, fp32 [B][ldf]; e2 may be null
  void* RDL; void* RDLt; int ldRDLt;                    // out: R delta_L [B][ldd] and [n_out_p][ldRDLt]
  void* RD; int ldRD; void* RDt; int ldRDt;             // out: R delta_{L-1} [B][ldRD] and [n_in_p][ldRDt]
  int B, n_in, n_in_p, C, loss;
  // Directional form (cvec non-null): only c_i = <dl_i/dz, Rz_L,i> per sample leaves the kernel
  // (the per-sample directional derivative of the loss, for the reweighting mixed term);
  // y / (Z, target) give dl/dz for cross-entropy / squared error.
  float* cvec; const int32_t* y; const float* Z; const float* target;
};
constexpr int LAST_ROP_MAX_C = 16;
void launch_last_layer_rop(Ctx&, Elem, const LastRopArgs&);

// The first-order counterpart for narrow outputs: logits z_L = a_{L-1} W_L + b_L, per-sample loss,
// sample weight and output delta (what loss_rows_kernel computes), and
// delta_{L-1} = (delta_L W_L^T) .* phi'(z_{L-1}) (with e2 <- (delta_L W_L^T) .* e2 in place when e2
// is given), for up to two batches (train, validation) in one launch.
struct LastGradSide {
  const void* A; int lda;                        // a_{L-1} [B][lda], operand type
  const int32_t* y; const float* target;         // labels, or targets [B][C]
  const float* omega_fixed;                      // sample weights to use instead of the weight net, or null
  float* ZL; float* P; int ldz;                  // out: logits, softmax probabilities, fp32 [B][ldz]
  float* ell; float* s; float* omega;            // out: per-sample loss, scale, weight
  float* dsig;                                   // out: omega (1 - omega) without cancellation (weight net evaluated here only)
  void* DL; void* DLt; int ldd, ldDLt;           // out: delta_L [B][ldd] and [n_out_p][ldDLt]
  const float* dphi; float* e2; int ldf;         // layer L-1, fp32 [B][ldf]
  void* D; int ldD; void* Dt; int ldDt;          // out: delta_{L-1} [B][ldD] and [n_in_p][ldDt]
  int B, reweight; float inv_batch;
};
struct LastGradArgs {
  LastGradSide side[2]; int n_sides;
  const void* Wt; int ldt; const void* Wn; int ldn;   // W_L as [n_out_p][n_in_p] and [n_in_p][n_out_p]
  const float* bias;                                  // b_L (fp32), or null
  const float* theta; int hidden;                     // weight net (sides with reweight set)
  int n_in, n_in_p, C, loss;
};
void launch_last_layer_grad(Ctx&, Elem, const LastGradArgs&);

void launch_loss_hessian_rows(Ctx&, Elem, int loss, const float* P, const float* Rz, long long ld,
                              const float* s, int rows, int C, void* D, int ldD, void* Dt, int ldDt);
// c_i = < dl_i/dz, Rz_i >
void launch_loss_directional_rows(Ctx&, int loss, const float* P, const float* Z, const int32_t* y,
                                  const float* target, const float* Rz, long long ld, int rows,
                                  int C, float* c);
// out = -(1/B) sum_i c_i dR(l_i; theta)/dtheta
void launch_wnet_theta_vjp(Ctx&, const float* ell, const float* dsig, const float* c,
                           const float* theta, int hidden, int rows, float inv_batch, float* out);

// ---- kernels.hip : flat parameter-shaped vectors ------------------------------------------
void launch_fill_zero(Ctx&, void* p, size_t bytes);
void launch_scale_copy(Ctx&, const float* src, float scale, float* dst, size_t n);
void launch_mixed_l2(Ctx&, const float* lam, const float* w, const float* p, float alpha, float* out, size_t n);
// out = 2 exp(logrho) (alpha p): the mixed VJP of the proximal cost into its anchor
void launch_mixed_prox(Ctx&, const float* logrho, const float* p, float alpha, float* out, size_t n);
void launch_diff(Ctx&, const float* a, const float* b, float* out, size_t n);        // out = a - b
void launch_fill_value(Ctx&, float* p, float value, size_t n);
void launch_sumsq(Ctx&, const float* x, size_t n, double* partials, float* out_scalar);
void launch_dot(Ctx&, const float* x, const float* y, size_t n, double* partials, float* out_scalar);
// conjugate gradient on device scalars: a = rs / dHd (0 if either is 0); q += a d; r -= a Hd; rs_new = r.r
void launch_cg_init(Ctx&, const float* r, float* d, float* q, size_t n);
void launch_cg_step(Ctx&, float* q, float* r, const float* d, const float* Hd, const float* rs, const float* dHd,
                    size_t n, double* partials, float* rs_new);
// d = r + (rs_new / rs) d   (beta = 0 if rs == 0)
void launch_cg_dir(Ctx&, float* d, const float* r, const float* rs, const float* rs_new, size_t n);
// c_i = (lp_i - lm_i) / (2 eps)   (0 if eps == 0)
void launch_adam(Ctx&, float* x, const float* g, float* m, float* v, float lr, float beta1, float beta2, float eps,
                 float bias1, float bias2, size_t n);
void launch_fd_loss_diff(Ctx&, const float* lp, const float* lm, const float* eps_dev, int rows, float* c);
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

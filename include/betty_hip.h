/*
 * betty_hip.h -- C ABI of the MI355X (gfx950) hypergradient library.
 *
 * The library computes the base operation of gradient-based multilevel
 * optimisation stated in the paper's Sec. 3.2 (Eq. 3-4): given a lower problem
 *     w*(lambda) = argmin_w L_L(w, lambda)
 * and an upper cost L_U(w*), the product of the best-response Jacobian with the
 * upper direct gradient (Eq. 1 with one lower problem),
 *     dL_U/dlambda = - (d^2 L_L / dlambda dw) H^{-1} grad_w L_U ,  H = d^2 L_L / dw dw,
 * evaluated right-to-left with matrix-vector products only (Sec. 3.2), by the
 * approximate-implicit-differentiation variants the paper lists there: the Neumann
 * series (AID-NMN), finite differences (AID-FD) and conjugate gradient (AID-CG); the same
 * operation on an arbitrary vector, and chained over two lower problems (Eq. 2).
 *
 * Model family: an MLP classifier/regressor with L linear layers
 *     a_0 = X,  z_l = a_{l-1} W_l + b_l,  a_l = phi(z_l) (l < L),  output z_L,
 * per-sample loss l_i (softmax cross-entropy on int labels, or squared error),
 * lower cost either
 *     BETTY_HP_L2_DECAY:      mean_i l_i + sum_j exp(lambda_j) w_j^2   (App. D.1 structure:
 *                             one weight-decay hyperparameter per parameter), or
 *     BETTY_HP_REWEIGHT_NET:  mean_i R(l_i; theta) l_i with R a 1-H-1 MLP (ReLU hidden,
 *                             sigmoid output) fed the value of l_i as a constant
 *                             (App. B Listing 3, App. C "Meta-Weight-Network"), or
 *     BETTY_HP_PROXIMAL:      mean_i l_i + sum_j rho_j (w_j - a_j)^2 with the anchor a as the
 *                             upper variable (finetuning level of Sec. 4.3, App. B Listing 5),
 * and upper cost mean_i l_i on the validation batch (Listing 3, level 2).
 *
 * Conventions common to every call
 *  - All data pointers are DEVICE pointers unless a comment says "host".
 *  - Parameter-shaped vectors (w, v, q, Hv, grad, and lambda for L2 decay) are flat fp32:
 *    [W_1 (n_0 x n_1, row-major), b_1 (n_1), ..., W_L, b_L]; biases absent if has_bias == 0.
 *    For the weight net lambda = theta = [u1 (H), b1 (H), u2 (H), b2 (1)].
 *  - X is row-major batch x n_0 fp32; labels are int32 in [0, n_L) (a label outside that range
 *    is read as the nearest class, 0 or n_L - 1, in the loss and in every derivative alike);
 *    targets are row-major batch x n_L fp32.
 *  - The caller owns every buffer, including the workspace.  The compute calls never
 *    allocate or free device memory and never synchronise: work is enqueued on the bound
 *    stream, outputs are valid once the caller has synchronised that stream.
 *  - Outputs must not overlap inputs.  Pointers must be 4-byte aligned; the workspace 256-byte.
 *  - Every call returns a betty_status; arguments are validated on the host before any
 *    launch, so a failing call leaves its outputs untouched.  betty_last_error() returns
 *    text for the most recent failure on that handle.
 *  - Results are deterministic: identical inputs give bit-identical outputs.
 *  - A handle is not thread-safe; use one handle per host thread/stream.
 */
#ifndef BETTY_HIP_H
#define BETTY_HIP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct betty_handle_s* betty_handle;

typedef enum {
  BETTY_OK = 0,
  BETTY_EINVAL = -1,       /* bad scalar argument (K < 0, non-finite alpha, ...)        */
  BETTY_ENULL = -2,        /* a required pointer is NULL                                */
  BETTY_ESHAPE = -3,       /* inconsistent problem description                          */
  BETTY_EWORKSPACE = -4,   /* workspace missing or too small / batches not set          */
  BETTY_EALIGN = -5,       /* misaligned pointer                                        */
  BETTY_EUNSUPPORTED = -6, /* combination not implemented                               */
  BETTY_EDEVICE = -7       /* a HIP runtime call failed                                 */
} betty_status;

typedef enum { BETTY_ACT_NONE = 0, BETTY_ACT_RELU = 1, BETTY_ACT_GELU_ERF = 2 } betty_act;
typedef enum { BETTY_LOSS_MSE = 0, BETTY_LOSS_SOFTMAX_CE = 1 } betty_loss;
/* What the upper-level variable `lambda` is (length: betty_num_hyper):
 *  L2_DECAY      per-parameter log weight decay, cost term sum_j exp(lambda_j) w_j^2  (App. D.1)
 *  REWEIGHT_NET  parameters of the 1-H-1 sample-weighting net fed the detached loss    (Sec. 4.1)
 *  PROXIMAL      anchor parameters a, cost term sum_j rho_j (w_j - a_j)^2: the finetuning level
 *                of the three-level program of Sec. 4.3, whose anchor is the optimum of the
 *                pretraining level (length d, same layout as w)                               */
typedef enum { BETTY_HP_L2_DECAY = 0, BETTY_HP_REWEIGHT_NET = 1, BETTY_HP_PROXIMAL = 2 } betty_hp;
/* Arithmetic of the GEMMs: fp32 operands, or operands rounded to bf16 (round to nearest
 * even) with fp32 accumulation.  Loss math, reductions and all parameter-shaped vectors
 * are fp32 in both.  Two exceptions under BETTY_PREC_BF16_FP32ACC, each because a bf16 operand
 * would destroy the quantity being computed: the finite-difference variant always uses fp32
 * operands (the perturbation e v is far below a bf16 ulp of w), and for BETTY_ACT_RELU the forward
 * products z_l = a_{l-1} W_l are formed from fp32 operands so that the sign of z_l, i.e. the ReLU
 * mask, is decided at fp32 accuracy; every backward and forward-over-reverse product of a ReLU
 * network still takes bf16 operands. */
typedef enum { BETTY_PREC_FP32 = 0, BETTY_PREC_BF16_FP32ACC = 1 } betty_prec;

typedef struct {
  int n_layers;        /* L >= 1 linear layers                                          */
  const int* dims;     /* host, L+1 entries n_0..n_L, copied by betty_create            */
  int has_bias;
  betty_act act;
  betty_loss loss;
  betty_hp hp;
  betty_prec prec;
  int batch_train;     /* samples in the lower (train) batch                            */
  int batch_val;       /* samples in the upper (validation) batch                       */
  int wnet_hidden;     /* H of the 1-H-1 weight net (REWEIGHT_NET only)                 */
  float prox_rho;      /* PROXIMAL only: rho >= 0                                       */
  int prox_skip_last;  /* PROXIMAL only: non-zero = rho_j is 0 on the last layer's W, b  */
} betty_problem_desc;

typedef struct {
  const float* x;        /* batch x n_0                                                 */
  const int32_t* y;      /* labels, required for BETTY_LOSS_SOFTMAX_CE, else NULL       */
  const float* target;   /* batch x n_L, required for BETTY_LOSS_MSE, else NULL         */
} betty_batch;

/* ---- set-up ---------------------------------------------------------------------- */

/* Validates the description and builds the host-side plan.  No device work. */
betty_status betty_create(const betty_problem_desc* desc, betty_handle* out);
void betty_destroy(betty_handle h);
const char* betty_last_error(betty_handle h);   /* host string owned by the handle */

/* Number of parameters d, and the length of lambda (d, or 3H+1). */
size_t betty_num_params(betty_handle h);
size_t betty_num_hyper(betty_handle h);

/* Bytes of device workspace the handle needs. */
size_t betty_workspace_bytes(betty_handle h);

/* Binds a caller-owned device workspace and a HIP stream (hipStream_t passed as void*,
 * NULL = the default stream).  Enqueues a zero-fill of the workspace on that stream. */
betty_status betty_bind(betty_handle h, void* workspace, size_t bytes, void* hip_stream);

/* Registers the train (lower) and validation (upper) batches and enqueues the conversion
 * of X into the operand layouts of the workspace.  The label/target pointers are kept and
 * read by later calls, so they must stay valid; x may be released after the stream has
 * run past this call. */
betty_status betty_set_batches(betty_handle h, betty_batch train, betty_batch val);

/* ---- the hot path (Sec. 3.2) --------------------------------------------------- */

/* grad_w L_L(w, lambda) on the train batch (the "direct gradient" of the lower cost, Eq. 1);
 * loss_or_null receives L_L (1 float). */
betty_status betty_lower_grad(betty_handle h, const float* w, const float* lambda,
                              float* grad_w, float* loss_or_null);

/* grad_w L_U(w) on the validation batch; loss_or_null receives L_U. */
betty_status betty_upper_grad(betty_handle h, const float* w, float* grad_w, float* loss_or_null);

/* Hv = (d^2 L_L / dw dw) v at (w, lambda): forward-over-reverse product, H never formed. */
betty_status betty_hvp(betty_handle h, const float* w, const float* lambda, const float* v,
                       float* Hv);

/* betty_hvp for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): the same product on the same kernels, with the
 * workspace taken from a fixed array of BETTY_STATIC_SCRATCH_BYTES inside the library's device image
 * (each GPU the library runs on holds one copy of it until the process ends) instead of a bound
 * caller workspace.  The handle needs neither betty_bind nor betty_set_batches: the train batch and
 * the stream are arguments (x, and y or target, are device pointers as in betty_set_batches; NULL
 * stream = the default stream), and a binding the handle already has is left as it was.  The call
 * allocates and frees nothing on the device, never synchronises, and launches directly (no graph is
 * recorded).  It returns BETTY_EWORKSPACE, before any device work, when betty_workspace_bytes(h)
 * exceeds BETTY_STATIC_SCRATCH_BYTES.  Every call on a GPU uses that GPU's one array (it is cleared
 * at the start of each call): calls that overlap in time on one GPU, from any handles or streams,
 * race; calls ordered on one stream do not. */
#define BETTY_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
size_t betty_static_scratch_bytes(void);
betty_status betty_hvp_static(betty_handle h, betty_batch train, void* hip_stream, const float* w,
                              const float* lambda, const float* v, float* Hv);

/* out = - grad_lambda < grad_w L_L(w, lambda), q >   (q held constant), length of lambda. */
betty_status betty_mixed_vjp(betty_handle h, const float* w, const float* lambda,
                             const float* q, float* out);

/* Neumann-series hypergradient (AID-NMN):
 *   g = grad_w L_U(w); v = p = g; K times { v <- v - alpha H v; p <- p + v }; q = alpha p;
 *   dlambda = betty_mixed_vjp(q).     K >= 0, alpha finite.
 * (The partial sum p is carried in the equivalent nested form p <- g + (I - alpha H) p, so the
 * result agrees with the term-by-term recurrence up to fp32 rounding order.) */
betty_status betty_hypergrad_neumann(betty_handle h, const float* w, const float* lambda, int K,
                                     float alpha, float* dlambda);

/* Finite-difference hypergradient (AID-FD): as above with
 *   H v := [grad_w L_L(w + e v) - grad_w L_L(w - e v)] / (2 e),  e = eps_scale / ||v||_2,
 * and the mixed term by the same central difference of grad_lambda L_L along q.  Only
 * first-order gradients are evaluated; K = 0 gives q = alpha g.  fp32 operands throughout.
 * For BETTY_HP_REWEIGHT_NET the sample weights and the loss values fed to the weight net are
 * those of the unperturbed w in every perturbed evaluation (the cost holds them constant in w). */
betty_status betty_hypergrad_fd(betty_handle h, const float* w, const float* lambda, int K,
                                float alpha, float eps_scale, float* dlambda);

/* Conjugate-gradient hypergradient (AID-CG, Sec. 3.2): K conjugate-gradient iterations on
 * H q = g from q = 0 with g = grad_w L_U(w), then dlambda = betty_mixed_vjp(q).  K >= 0.
 * H must be positive definite for the iteration to be meaningful; a zero curvature d'Hd or a
 * zero residual freezes the iterate (no division by zero). */
betty_status betty_hypergrad_cg(betty_handle h, const float* w, const float* lambda, int K,
                                float* dlambda);

/* The base operation of Sec. 3.2 (Eq. 3-4) on an arbitrary vector: out = (dw* / dlambda) u
 *   = -(d^2 L_L / dlambda dw) q,  q = alpha * sum_{j<=K} (I - alpha H)^j u,
 * i.e. betty_hypergrad_neumann with the device vector u (d floats) in place of grad_w L_U(w).
 * This is one factor of a path product of Eq. 2: a program with more than two levels applies it
 * once per lower-to-upper edge, from the right.  out has betty_num_hyper entries and must not
 * overlap w, lambda or u.  Same argument checks as betty_hypergrad_neumann. */
betty_status betty_best_response_neumann(betty_handle h, const float* w, const float* lambda,
                                         const float* u, int K, float alpha, float* out);

/* Three-level chain theta -> w*(theta) -> v*(w*) -> L_U(v*) (Eq. 2 with its single path; the
 * reweight / pretrain / finetune program of Sec. 4.3):
 *   dtheta = (dw* / dtheta) (dv* / dw) grad_v L_U(v),
 * evaluated from the right with two Neumann best-response products.
 *   h_finetune  BETTY_HP_PROXIMAL handle: parameters v, anchor w, its train batch is the
 *               finetuning data and its validation batch carries L_U
 *   h_pretrain  handle of the pretraining problem: parameters w, upper variable theta
 *               (REWEIGHT_NET or L2_DECAY); only its train batch is used
 * Both handles must describe the same number of parameters and be bound to the same stream.
 * w, v: d floats; theta, dtheta: betty_num_hyper(h_pretrain) floats; all device pointers.
 * Errors are reported on h_pretrain (betty_last_error).  A call repeated with identical arguments
 * replays one captured graph over both handles; binding or setting batches on either handle
 * discards it.  Per-launch timing must be off on h_finetune. */
betty_status betty_hypergrad_chain3(betty_handle h_pretrain, betty_handle h_finetune, const float* w,
                                    const float* theta, const float* v, int K_pretrain,
                                    float alpha_pretrain, int K_finetune, float alpha_finetune,
                                    float* dtheta);

/* ---- the optimisation steps around the path (Sec. 3.3; optimisers as in App. C) ----------- */

/* One step of the lower problem, in place: momentum SGD on L_L(w, lambda) over the train batch,
 *   g = grad_w L_L(w, lambda) + weight_decay * w;  momentum <- mu * momentum + g;  w <- w - lr * momentum.
 * loss_or_null receives L_L at the w before the step.  Calling it `unroll` times and then a
 * hypergradient call at the resulting w is the paper's unrolled lower optimisation. */
betty_status betty_lower_sgd_step(betty_handle h, float* w, const float* lambda, float* momentum,
                                  float lr, float mu, float weight_decay, float* loss_or_null);

/* One Adam step on the upper parameters, in place, given their hypergradient; t >= 1 is the
 * step counter of the bias correction; m, v are the moment buffers (length of lambda). */
betty_status betty_upper_adam_step(betty_handle h, float* lambda, const float* dlambda, float* m,
                                   float* v, int t, float lr, float beta1, float beta2, float eps);

/* Uniform label noise as integer work: T = floor(p * 2^32);
 *   mask_i = words_i < T;  y_out_i = mask_i ? alt_i : y_i.   n >= 0 elements, p in [0, 1].
 * mask_or_null receives 0/1 bytes.  Runs on the handle's stream. */
betty_status betty_apply_label_noise(betty_handle h, const int32_t* y, const uint32_t* words,
                                     const int32_t* alt, double p, int n, int32_t* y_out,
                                     uint8_t* mask_or_null);

/* ---- per-kernel timing (measurement aid) ---------------------------------------- */

typedef struct {
  int kind;          /* BETTY_K_* below                                                 */
  float ms;          /* duration of this launch between two events on the stream        */
  double flops;      /* algorithmic flops of this launch (GEMMs), else 0                */
  double bytes;      /* algorithmic bytes of this launch (vector kernels), else 0       */
} betty_profile_rec;

enum {
  BETTY_K_GEMM = 0, BETTY_K_EPILOGUE = 1, BETTY_K_LOSS = 2, BETTY_K_SHADOW = 3,
  BETTY_K_VECTOR = 4, BETTY_K_REDUCE = 5, BETTY_K_WNET = 6, BETTY_K_OTHER = 7,
  BETTY_K_GEMM_UPDATE = 8,  /* weight-gradient GEMM whose epilogue applies one step of the Neumann sum:
                               flops = its 2MNK, bytes = per parameter s, g (and the diagonal) read,
                               s and two operand-type copies written (20 with a diagonal term)        */
  BETTY_K_GEMM_UPDATE_FINAL = 9,  /* the same for the last step of the L2-decay kind, which writes
                               d(lambda) only (s, g, lambda, w read: 20 bytes per parameter)         */
  BETTY_K_LAST_LAYER = 10,  /* the narrow-output-layer kernels (flops = their products)              */
  BETTY_K_GEMM_RFWD = 11,   /* one link of the R-forward chain  Rz_l = [Ra_{l-1} | a_{l-1}] [W_l ; V_l]     */
  BETTY_K_GEMM_RBWD = 12    /* one link of the R-backward chain R delta_{l-1} = [R delta_l | delta_l] [W_l^T ; V_l^T] .* phi' + ... */
};

/* While enabled, every kernel launch of the handle is bracketed by HIP events on the
 * bound stream.  betty_profile_collect synchronises the stream, converts the events to
 * durations and returns how many records are available; betty_profile_get copies record i.
 * Enabling clears earlier records.  Timing this way perturbs the launch pipeline: use it
 * for per-kernel durations only, never inside a throughput measurement. */
betty_status betty_profile_enable(betty_handle h, int on);
int betty_profile_collect(betty_handle h);
betty_status betty_profile_get(betty_handle h, int i, betty_profile_rec* out);

#ifdef __cplusplus
}
#endif
#endif /* BETTY_HIP_H */

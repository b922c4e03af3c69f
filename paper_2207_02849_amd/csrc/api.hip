// Host side of libbetty_hip.so: handle, argument validation, workspace plan, and the launch
// sequences of the five hot-path calls (paper Sec. 3.2; Neumann and finite-difference
// approximate implicit differentiation followed by the mixed second-order VJP).
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <new>
#include <cstring>
#include <mutex>

#include "internal.h"

using namespace betty;

namespace betty {

void Ctx::begin(int kind, double flops, double bytes) {
  if (!profiling) return;
  ProfRec r{};
  r.kind = kind; r.flops = flops; r.bytes = bytes; r.ms = -1.f;
  if (hipEventCreate(&r.e0) != hipSuccess || hipEventCreate(&r.e1) != hipSuccess) { profiling = false; return; }
  (void)hipEventRecord(r.e0, stream);
  recs.push_back(r);
}

void Ctx::end() {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess && first_error == hipSuccess) first_error = e;
  if (profiling && !recs.empty()) (void)hipEventRecord(recs.back().e1, stream);
}

}  // namespace betty

namespace {

struct LayerInfo {
  int n_in, n_out, n_in_p, n_out_p;
  size_t w_off, b_off;       // offsets (in floats) into a flat parameter vector
};

// Buffers that depend on which batch (train / validation) is being propagated.
struct SideBuf {
  int B = 0, Bp = 0;
  size_t X = 0, XT = 0;                       // a_0 and its transpose
  std::vector<size_t> A, At, D, Dt;           // a_l (1..L-1), delta_l (1..L), each in both orientations
  std::vector<size_t> dphi, e2;               // fp32 phi'(z_l); phi''(z_l) then (delta W^T) phi''
  size_t ZL = 0, P = 0, ell = 0, s = 0, omega = 0, dsig = 0;   // dsig: omega (1 - omega)
  size_t ell_bar = 0, omega_bar = 0, dsig_bar = 0, ell_p = 0;   // frozen / perturbed per-sample values (finite differences, reweighting)
};

// One complete set of GEMM operands in a given element type.
struct OperandSet {
  Elem elem = ELEM_F32;
  bool present = false;
  SideBuf side[2];                            // 0 = train (lower), 1 = validation (upper)
  std::vector<size_t> Wn, Wt, Vn, Vt;         // W_l as stored / transposed; same for the direction
  std::vector<size_t> Vn2, Vt2;               // second set of direction copies (pipelined recurrence; main set only)
  std::vector<size_t> RA, RAt, RD, RDt, Rz;   // R-op quantities (train side only)
  size_t cvec = 0;
};

}  // namespace

struct betty_handle_s {
  betty_problem_desc desc{};
  std::vector<int> dims;
  std::vector<LayerInfo> layers;
  int L = 0;
  size_t d = 0, n_hyper = 0;
  int max_np = 0, max_Bp = 0;
  std::string err;
  Ctx ctx;
  char* ws = nullptr;
  size_t ws_need = 0;
  bool bound = false, batches = false;
  unsigned long long epoch = 0;   // process-wide unique stamp of the last betty_bind / betty_set_batches
  betty_batch batch[2]{};
  OperandSet sets[2];        // [0]: element type of desc.prec; [1]: fp32 set for finite differences when prec is bf16
  OperandSet fd_minus;       // fp32, train side only: the evaluation at w - eps v, which runs beside the one at w + eps v
  size_t vec_g = 0, vec_v = 0, vec_p = 0, vec_Hv = 0, vec_wpm = 0, vec_Gm = 0;
  size_t vec_wpm2 = 0, vec_g2 = 0;   // the second evaluation's perturbed point and anchor distance
  size_t partials = 0, scalars = 0;
  size_t logrho = 0;         // proximal cost: log(rho_j) per parameter (a large negative value where rho_j = 0)
  // a hypergradient call repeated with the same arguments is replayed from a captured HIP graph
  struct GraphSlot {
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
    const void* w = nullptr; const void* lam = nullptr; const void* u = nullptr; void* out = nullptr;
    int K = -1; float alpha = 0.f, eps = 0.f;
    int K2 = -1; float alpha2 = 0.f; const void* other = nullptr;   // second level of the three-level chain
    unsigned long long other_epoch = 0;                             // ... and the state of its handle when recorded
    int seen = 0;
  };
  GraphSlot graph_neumann, graph_fd, graph_cg, graph_br, graph_chain;
  bool use_graphs = true;
  int tune_target_blocks = 256, tune_tile128_min = 512;   // see plan_chain (measured on 512x4096x8192: 64-tiles beat 128-tiles until the grid is several waves deep)
  int tune_wgrad_cfg = GEMM_64x1;
  int tune_rect_max = 1024, tune_rect_min_tt = 16;  // see plan_chain
  int tune_wgrad128_min = 512;                // 128-tiles a bf16 weight-gradient launch needs to use the 128-tile kernel (0 = never)
  // For large models the Neumann recurrence overlaps each layer's weight-gradient launch
  // (bandwidth-bound) with the rest of the R-backward chain on a second stream of the same
  // priority.  Every cross-stream dependency costs several microseconds (measured: 5 per product,
  // about 37 us in total), so it only pays when the launches it hides are far longer than that:
  // it is switched on from 32M parameters (+1 % at 116M parameters, -25 % at 5M).
  hipStream_t side_stream = nullptr;
  std::vector<hipEvent_t> fork_events;        // one per layer
  hipEvent_t join_event = nullptr;
  bool use_pipeline = false;
  // Finite differences: the gradient evaluations at w + eps v and w - eps v are independent and run
  // side by side on the two streams when one of them alone leaves part of the chip idle
  // (measured: -10 % per hypergradient at 1M parameters, -1 % at 5M, +0.5 % at 116M, where each
  // evaluation is bandwidth-bound already), so below the same 32M-parameter mark.
  bool fd_two_streams = false;

  template <typename T = void> T* at(size_t off) const { return (T*)(ws + off); }
  float* f(size_t off) const { return (float*)(ws + off); }
};

namespace {

betty_status fail(betty_handle h, betty_status st, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (h) h->err = buf;
  return st;
}

struct Planner {
  size_t off = 0;
  size_t take(size_t bytes) {
    size_t o = off;
    off += (bytes + 255) / 256 * 256;
    return o;
  }
};

void plan_side(betty_handle h, Planner& pl, SideBuf& sb, Elem elem, int B, bool lower) {
  const int L = h->L;
  const size_t es = elem_size(elem);
  sb.B = B;
  sb.Bp = padup(B);
  const size_t Bp = sb.Bp;
  sb.X = pl.take(Bp * h->layers[0].n_in_p * es);
  sb.XT = pl.take((size_t)h->layers[0].n_in_p * Bp * es);
  sb.A.assign(L + 1, 0); sb.At.assign(L + 1, 0); sb.D.assign(L + 1, 0); sb.Dt.assign(L + 1, 0);
  sb.dphi.assign(L + 1, 0); sb.e2.assign(L + 1, 0);
  for (int l = 1; l <= L; ++l) {
    const size_t np = h->layers[l - 1].n_out_p;
    if (l < L) {
      sb.A[l] = pl.take(Bp * np * es);
      sb.At[l] = pl.take(np * Bp * es);
      sb.dphi[l] = pl.take(Bp * np * 4);
      if (lower && h->desc.act == BETTY_ACT_GELU_ERF) sb.e2[l] = pl.take(Bp * np * 4);
    }
    sb.D[l] = pl.take(Bp * np * es);
    sb.Dt[l] = pl.take(np * Bp * es);
  }
  const size_t Cp = h->layers[L - 1].n_out_p;
  sb.ZL = pl.take(Bp * Cp * 4);
  sb.P = pl.take(Bp * Cp * 4);
  sb.ell = pl.take(Bp * 4);
  sb.s = pl.take(Bp * 4);
  sb.omega = pl.take(Bp * 4);
  sb.ell_bar = pl.take(Bp * 4);
  sb.omega_bar = pl.take(Bp * 4);
  sb.dsig = pl.take(Bp * 4);
  sb.dsig_bar = pl.take(Bp * 4);
  sb.ell_p = pl.take(Bp * 4);
}

// How much of an operand set exists:
//  SET_FULL          everything (first-order passes on both batches and the forward-over-reverse passes)
//  SET_FIRST_ORDER   what first-order gradients on both batches touch (the fp32 set that serves the
//                    finite-difference variant and the fp32 forward of ReLU networks beside bf16 operands)
//  SET_TRAIN_ONLY    just what a gradient of the lower cost on the train batch touches
enum SetScope { SET_FULL, SET_FIRST_ORDER, SET_TRAIN_ONLY };

void plan_set(betty_handle h, Planner& pl, OperandSet& os, Elem elem, bool second_direction_set, SetScope scope) {
  const int L = h->L;
  const size_t es = elem_size(elem);
  os.elem = elem;
  os.present = true;
  plan_side(h, pl, os.side[0], elem, h->desc.batch_train, true);
  os.Wn.assign(L, 0); os.Wt.assign(L, 0); os.Vn.assign(L, 0); os.Vt.assign(L, 0);
  for (int i = 0; i < L; ++i) {
    const size_t m = (size_t)h->layers[i].n_in_p * h->layers[i].n_out_p * es;
    os.Wn[i] = pl.take(m); os.Wt[i] = pl.take(m);
    if (scope == SET_FULL) { os.Vn[i] = pl.take(m); os.Vt[i] = pl.take(m); }
  }
  if (scope == SET_TRAIN_ONLY) return;
  plan_side(h, pl, os.side[1], elem, h->desc.batch_val, false);
  const size_t Bp = os.side[0].Bp;
  os.cvec = pl.take(Bp * 4);
  if (scope == SET_FIRST_ORDER) return;
  if (second_direction_set) {
    os.Vn2.assign(L, 0); os.Vt2.assign(L, 0);
    for (int i = 0; i < L; ++i) {
      const size_t m = (size_t)h->layers[i].n_in_p * h->layers[i].n_out_p * es;
      os.Vn2[i] = pl.take(m); os.Vt2[i] = pl.take(m);
    }
  }
  os.RA.assign(L + 1, 0); os.RAt.assign(L + 1, 0); os.RD.assign(L + 1, 0); os.RDt.assign(L + 1, 0);
  os.Rz.assign(L + 1, 0);
  for (int l = 1; l <= L; ++l) {
    const size_t np = h->layers[l - 1].n_out_p;
    if (l < L) { os.RA[l] = pl.take(Bp * np * es); os.RAt[l] = pl.take(np * Bp * es); }
    os.RD[l] = pl.take(Bp * np * es);
    os.RDt[l] = pl.take(np * Bp * es);
    os.Rz[l] = pl.take(Bp * np * 4);
  }
}

void plan(betty_handle h) {
  Planner pl;
  const Elem main_elem = h->desc.prec == BETTY_PREC_BF16_FP32ACC ? ELEM_BF16 : ELEM_F32;
  plan_set(h, pl, h->sets[0], main_elem, true, SET_FULL);
  if (main_elem == ELEM_BF16) plan_set(h, pl, h->sets[1], ELEM_F32, false, SET_FIRST_ORDER);
  const size_t vb = h->d * 4;
  h->vec_g = pl.take(vb); h->vec_v = pl.take(vb); h->vec_p = pl.take(vb); h->vec_Hv = pl.take(vb);
  h->vec_wpm = pl.take(vb); h->vec_Gm = pl.take(vb);
  if (h->fd_two_streams) {
    plan_set(h, pl, h->fd_minus, ELEM_F32, false, SET_TRAIN_ONLY);
    h->vec_wpm2 = pl.take(vb);
    if (h->desc.hp == BETTY_HP_PROXIMAL) h->vec_g2 = pl.take(vb);
  }
  if (h->desc.hp == BETTY_HP_PROXIMAL) h->logrho = pl.take(vb);
  h->partials = pl.take(1024 * 8);
  h->scalars = pl.take(256);
  h->ws_need = pl.off;
}

// The lower cost's parameter-diagonal term is sum_j exp(c_j) (.)^2 with c = lambda for L2 decay and
// c = log(rho) for the proximal cost; the reweighting cost has none.
const float* diag_log(betty_handle h, const float* lambda) {
  if (h->desc.hp == BETTY_HP_L2_DECAY) return lambda;
  if (h->desc.hp == BETTY_HP_PROXIMAL) return h->f(h->logrho);
  return nullptr;
}
// the weight-net parameters, for the cost that has a weight net
const float* wnet_theta(betty_handle h, const float* lambda) {
  return h->desc.hp == BETTY_HP_REWEIGHT_NET ? lambda : nullptr;
}

OperandSet& fd_operands(betty_handle h) { return h->sets[1].present ? h->sets[1] : h->sets[0]; }

// Kernel configuration of an activation-shaped GEMM (M = batch), from its tile count and the
// number of k-tiles TT (thresholds from timings on this chip):
//  * 128-tiles once there are enough of them to fill the chip several times over;
//  * 32-tiles with an eight-way K split inside the workgroup when even 64-tiles would leave half
//    the compute units idle (batch 256 against 1024-wide layers);
//  * 64-tiles with K split four ways while the grid is still small;
//  * 128 x 64 tiles when 64-tiles would come to between one and four per compute unit and the
//    reduction is long: such a launch is bound by what a compute unit can pull through its L1
//    (measured: about 63 GB/s each with all of them pulling), and a 128 x 64 tile fetches 192
//    operand rows for the 8192 outputs that two 64-tiles fetch 256 for (121M-parameter model,
//    batch 512: R-forward link 73 -> 66 us, backward link 76 -> 60 us);
//  * otherwise plain 64-tiles.
// Measured and dropped: 128-tiles with a two-way K split (2 x 512 x 4096 x 4096: 78 us against
// 73 us for plain 64-tiles), and 64-tiles computed by one wavefront each over a quarter of K
// (faster stand-alone, 54 against 62 us on 512 x 4096 x 8192, but 4 % slower with the real
// epilogues, whose loads cannot be issued ahead of the k loop for four MFMA blocks per wavefront).
int plan_chain(betty_handle h, Elem elem, int tiles128, int Ktot_p) {
  const int TT = Ktot_p / gemm_ktile_elems(elem);
  if (tiles128 >= h->tune_tile128_min) return GEMM_128x1;
  const int tiles64 = 4 * tiles128;
  if (tiles64 <= h->tune_target_blocks / 2 && TT >= 16) return GEMM_32x8;
  if (tiles64 < h->tune_target_blocks && TT >= 8) return GEMM_64x4;
  if (tiles64 <= h->tune_rect_max && TT >= h->tune_rect_min_tt) return GEMM_128x64;
  return GEMM_64x1;
}

void set_pairs(GemmArgs& g, const void* A0, int lda0, const void* B0, int ldb0, int K0p, const void* A1,
               int lda1, const void* B1, int ldb1, int K1p) {
  g.A[0] = A0; g.B[0] = B0; g.lda[0] = lda0; g.ldb[0] = ldb0; g.Kp[0] = K0p;
  g.A[1] = A1 ? A1 : A0; g.B[1] = A1 ? B1 : B0; g.lda[1] = A1 ? lda1 : lda0; g.ldb[1] = A1 ? ldb1 : ldb0;
  g.Kp[1] = A1 ? K1p : 0;
  g.xgm = g.xgn = 0;
}

// one activation-shaped GEMM with a fused epilogue
void chain_gemm(betty_handle h, Elem elem, const void* A0, int lda0, const void* B0, int ldb0, int K0p,
                const void* A1, int lda1, const void* B1, int ldb1, int K1p, int M, int N, int Mp, int Np,
                const Epilogue& e, double flops) {
  GemmBatch b;
  b.n = 1;
  GemmProblem& p = b.p[0];
  set_pairs(p.g, A0, lda0, B0, ldb0, K0p, A1, lda1, B1, ldb1, K1p);
  p.g.M = M; p.g.N = N; p.g.Mp = Mp; p.g.Np = Np;
  p.e = e;
  launch_gemm_batch(h->ctx, elem, plan_chain(h, elem, (Mp / 128) * (Np / 128), p.g.Kp[0] + p.g.Kp[1]), b, flops);
}

Epilogue blank_epilogue(int mode, int act = 0) {
  Epilogue e;
  memset(&e, 0, sizeof e);
  e.mode = mode;
  e.act = act;
  return e;
}

// operand copies of a flat parameter-shaped vector: per layer, as stored (n_in x n_out) and
// transposed; all layers in one launch (eight per launch)
void make_shadows(betty_handle h, OperandSet& os, const float* flat, float scale,
                  std::vector<size_t>* N, std::vector<size_t>* T, std::vector<size_t>* T32 = nullptr) {
  for (int i0 = 0; i0 < h->L; i0 += MAX_PROBLEMS) {
    ConvertBatch b;
    b.n = std::min(MAX_PROBLEMS, h->L - i0);
    for (int k = 0; k < b.n; ++k) {
      const LayerInfo& li = h->layers[i0 + k];
      b.j[k] = ConvertJob{flat + li.w_off, li.n_out, scale, li.n_in, li.n_out,
                          N ? h->at<void>((*N)[i0 + k]) : nullptr, li.n_out_p,
                          T ? h->at<void>((*T)[i0 + k]) : nullptr, li.n_in_p};
      if (T32) b.j[k].outT32 = h->f((*T32)[i0 + k]);
    }
    launch_convert_batch(h->ctx, os.elem, b);
  }
}

// A ReLU mask is a discontinuous function of the pre-activation: deciding it from bf16-rounded
// operands flips about one unit in a thousand, which alone costs a few percent of relative error
// in every gradient that passes through the mask.  With bf16 operands the forward products of a
// ReLU network are therefore formed from the fp32 operand set; all other GEMMs stay bf16.
bool hybrid_forward(betty_handle h, const OperandSet& os) {
  return os.elem == ELEM_BF16 && h->desc.act == BETTY_ACT_RELU && h->sets[1].present;
}

// operand copies of the parameters w for everything that follows
void make_weight_operands(betty_handle h, OperandSet& os, const float* w) {
  // (with the fp32 forward of ReLU networks the same launch also leaves the fp32 transposed copies)
  make_shadows(h, os, w, 1.f, &os.Wn, &os.Wt, hybrid_forward(h, os) ? &h->sets[1].Wt : nullptr);
}

// Which batches a pass covers: the train (lower) side, the validation (upper) side, or both in
// the same launches (same weights, two independent problems per launch).
enum { SIDE_TRAIN = 1, SIDE_VAL = 2, SIDE_BOTH = 3 };
inline bool has_side(int mask, int side) { return (mask >> side) & 1; }

// a_l, phi'(z_l) (and phi'' on the lower side), logits, per-sample loss, output delta
void forward_and_loss(betty_handle h, OperandSet& os, int sides, const float* w, const float* theta,
                      const float* omega_fixed = nullptr, bool skip_last = false) {
  const int L = h->L;
  const bool hybrid = hybrid_forward(h, os);
  OperandSet& fs = hybrid ? h->sets[1] : os;          // operands of the forward products
  for (int l = 1; l <= (skip_last ? L - 1 : L); ++l) {
    const LayerInfo& li = h->layers[l - 1];
    const bool last = l == L;
    GemmBatch b;
    double flops = 0;
    int tiles128 = 0;
    for (int side = 0; side < 2; ++side) {
      if (!has_side(sides, side)) continue;
      SideBuf& sb = os.side[side];
      SideBuf& fb = fs.side[side];
      GemmProblem& p = b.p[b.n++];
      const void* Aop = l == 1 ? h->at<void>(fb.X) : h->at<void>(fb.A[l - 1]);
      set_pairs(p.g, Aop, li.n_in_p, h->at<void>(fs.Wt[l - 1]), li.n_in_p, li.n_in_p, nullptr, 0, nullptr, 0, 0);
      p.g.M = sb.B; p.g.N = li.n_out; p.g.Mp = sb.Bp; p.g.Np = li.n_out_p;
      Epilogue e = blank_epilogue(last ? EPI_FWD_LAST : EPI_FWD, h->desc.act);
      e.colvec = h->desc.has_bias ? w + li.b_off : nullptr;
      e.ldf = li.n_out_p;
      if (last) {
        e.f0 = h->f(sb.ZL);
      } else {
        e.dphi_out = h->f(sb.dphi[l]);
        e.d2_out = sb.e2[l] ? h->f(sb.e2[l]) : nullptr;
        e.out = h->at<void>(fb.A[l]); e.ld = li.n_out_p;
        e.outT = hybrid ? nullptr : h->at<void>(fb.At[l]); e.ldT = sb.Bp;
        if (hybrid) { e.out2 = h->at<void>(sb.A[l]); e.outT2 = h->at<void>(sb.At[l]); }
      }
      p.e = e;
      flops += 2.0 * sb.B * li.n_in * li.n_out;
      tiles128 += (sb.Bp / 128) * (li.n_out_p / 128);
    }
    launch_gemm_batch(h->ctx, fs.elem, plan_chain(h, fs.elem, tiles128, li.n_in_p), b, flops);
  }
  if (skip_last) return;
  const LayerInfo& lo = h->layers[L - 1];
  LossBatch lb;
  for (int side = 0; side < 2; ++side) {
    if (!has_side(sides, side)) continue;
    SideBuf& sb = os.side[side];
    LossArgs& a = lb.a[lb.n++];
    a = LossArgs{};
    a.loss = h->desc.loss;
    a.reweight = (side == 0 && h->desc.hp == BETTY_HP_REWEIGHT_NET) ? 1 : 0;
    a.hidden = h->desc.wnet_hidden;
    a.Z = h->f(sb.ZL); a.ldz = lo.n_out_p;
    a.y = h->batch[side].y; a.target = h->batch[side].target; a.C = lo.n_out;
    a.theta = theta;
    a.omega_fixed = side == 0 ? omega_fixed : nullptr;
    a.rows = sb.B; a.inv_batch = 1.0f / (float)sb.B;
    a.ell = h->f(sb.ell); a.s = h->f(sb.s); a.omega = h->f(sb.omega); a.dsig = h->f(sb.dsig);
    a.P = h->f(sb.P);
    a.D = h->at<void>(sb.D[L]); a.ldD = lo.n_out_p;
    a.Dt = h->at<void>(sb.Dt[L]); a.ldDt = sb.Bp;
  }
  launch_loss_rows(h->ctx, os.elem, lb);
}

// delta_l for every layer below the output (and (delta W^T) phi'' on the lower side)
void backward_chain(betty_handle h, OperandSet& os, int sides, int l_from = 0) {
  const int L = h->L;
  for (int l = l_from > 0 ? l_from : L; l >= 2; --l) {
    const LayerInfo& li = h->layers[l - 1];
    GemmBatch b;
    double flops = 0;
    int tiles128 = 0;
    for (int side = 0; side < 2; ++side) {
      if (!has_side(sides, side)) continue;
      SideBuf& sb = os.side[side];
      GemmProblem& p = b.p[b.n++];
      set_pairs(p.g, h->at<void>(sb.D[l]), li.n_out_p, h->at<void>(os.Wn[l - 1]), li.n_out_p, li.n_out_p, nullptr, 0,
                nullptr, 0, 0);
      p.g.M = sb.B; p.g.N = li.n_in; p.g.Mp = sb.Bp; p.g.Np = li.n_in_p;
      Epilogue e = blank_epilogue(EPI_BWD);
      e.dphi = h->f(sb.dphi[l - 1]);
      e.e_io = sb.e2[l - 1] ? h->f(sb.e2[l - 1]) : nullptr;
      e.ldf = li.n_in_p;
      e.out = h->at<void>(sb.D[l - 1]); e.ld = li.n_in_p;
      e.outT = h->at<void>(sb.Dt[l - 1]); e.ldT = sb.Bp;
      p.e = e;
      flops += 2.0 * sb.B * li.n_in * li.n_out;
      tiles128 += (sb.Bp / 128) * (li.n_in_p / 128);
    }
    launch_gemm_batch(h->ctx, os.elem, plan_chain(h, os.elem, tiles128, li.n_out_p), b, flops);
  }
}

// Forward pass, loss and backward chain.  A narrow output layer (see LastGradArgs) goes through
// one vector kernel that produces the logits, the loss quantities and delta_{L-1}.
void forward_backward(betty_handle h, OperandSet& os, int sides, const float* w, const float* theta,
                      const float* omega_fixed = nullptr) {
  const int L = h->L;
  const LayerInfo& lo = h->layers[L - 1];
  // (also with the fp32 forward of ReLU networks: the output layer has no mask to protect, and the
  // operand-type copy of a_{L-1} exists either way)
  const bool narrow = L >= 2 && lo.n_out <= LAST_ROP_MAX_C;
  if (!narrow) {
    forward_and_loss(h, os, sides, w, theta, omega_fixed);
    backward_chain(h, os, sides);
    return;
  }
  forward_and_loss(h, os, sides, w, theta, omega_fixed, true);
  LastGradArgs a{};
  for (int side = 0; side < 2; ++side) {
    if (!has_side(sides, side)) continue;
    SideBuf& sb = os.side[side];
    LastGradSide& d = a.side[a.n_sides++];
    d.A = h->at<void>(sb.A[L - 1]); d.lda = lo.n_in_p;
    d.y = h->batch[side].y; d.target = h->batch[side].target;
    d.omega_fixed = side == 0 ? omega_fixed : nullptr;
    d.ZL = h->f(sb.ZL); d.P = h->f(sb.P); d.ldz = lo.n_out_p;
    d.ell = h->f(sb.ell); d.s = h->f(sb.s); d.omega = h->f(sb.omega); d.dsig = h->f(sb.dsig);
    d.DL = h->at<void>(sb.D[L]); d.DLt = h->at<void>(sb.Dt[L]); d.ldd = lo.n_out_p; d.ldDLt = sb.Bp;
    d.dphi = h->f(sb.dphi[L - 1]); d.e2 = sb.e2[L - 1] ? h->f(sb.e2[L - 1]) : nullptr; d.ldf = lo.n_in_p;
    d.D = h->at<void>(sb.D[L - 1]); d.ldD = lo.n_in_p; d.Dt = h->at<void>(sb.Dt[L - 1]); d.ldDt = sb.Bp;
    d.B = sb.B;
    d.reweight = (side == 0 && h->desc.hp == BETTY_HP_REWEIGHT_NET) ? 1 : 0;
    d.inv_batch = 1.0f / (float)sb.B;
  }
  a.Wt = h->at<void>(os.Wt[L - 1]); a.ldt = lo.n_in_p;
  a.Wn = h->at<void>(os.Wn[L - 1]); a.ldn = lo.n_out_p;
  a.bias = h->desc.has_bias ? w + lo.b_off : nullptr;
  a.theta = theta; a.hidden = h->desc.wnet_hidden;
  a.n_in = lo.n_in; a.n_in_p = lo.n_in_p; a.C = lo.n_out; a.loss = h->desc.loss;
  launch_last_layer_grad(h->ctx, os.elem, a);
  backward_chain(h, os, sides, L - 1);
}

// Split of a tile grid over the eight XCDs (see GemmArgs::xgm): the factorisation gm x gn = 8 that
// divides the grid and minimises the operand rows each L2 fetches, gn * tiles_m + gm * tiles_n
// (every XCD reads tiles_m / gm row panels and tiles_n / gn column panels).  gm = gn = 0 when
// nothing fits or the row-major order is already as good.
void xcd_split(int tiles_m, int tiles_n, int& gm, int& gn) {
  gm = gn = 0;
  if ((tiles_m * tiles_n) % 8 != 0 || tiles_m * tiles_n < 256) return;   // small grids: no measurable gain
  long best = tiles_n % 8 == 0 ? 8L * tiles_m + tiles_n : -1;      // row-major order = 1 x 8 when tiles_n % 8 == 0
  for (int a = 1; a <= 8; a *= 2) {
    const int b = 8 / a;
    if (tiles_m % a || tiles_n % b) continue;
    const long cost = (long)b * tiles_m + (long)a * tiles_n;
    if (best < 0 || cost < best) { best = cost; gm = a; gn = b; }
  }
}

// What the grouped weight-gradient launch does with its result.
struct WgradSink {
  int mode;                 // EPI_WGRAD / EPI_WGRAD_INIT / EPI_WGRAD_NEUMANN
  float* C;                 // flat output (EPI_WGRAD)
  const float* lam;         // non-null adds the L2-decay term 2 e^lam x
  const float* x;
  float* v; float* p; float alpha;
  bool copies;              // also write the operand copies of the new v
  bool second_set = false;  // ... into the second set of direction copies (the first is still being read)
  float beta = 0.f, gamma = 0.f;   // EPI_WGRAD_SGD: momentum factor and plain weight decay
};
// (aggregate initialisation in the callers lists the fields up to `copies`)

// All layers' parameter-shaped products in one launch: plain gradient a^T delta (rop = false) or
// the R-op form Ra^T delta + a^T Rdelta (rop = true), bias rows included.
void wgrad_batch(betty_handle h, OperandSet& os, int side, bool rop, const WgradSink& k, int l_first = 1,
                 int l_last = 0) {
  SideBuf& sb = os.side[side];
  const int L = l_last > 0 ? l_last : h->L, B = sb.B, Bp = sb.Bp;
  const std::vector<size_t>& VN = k.second_set ? os.Vn2 : os.Vn;
  const std::vector<size_t>& VT = k.second_set ? os.Vt2 : os.Vt;
  for (int l0 = l_first; l0 <= L; l0 += MAX_PROBLEMS) {
    GemmBatch b;
    b.n = std::min(MAX_PROBLEMS, L - l0 + 1);
    // bf16 launches with enough 128-tiles to fill the chip twice take the 128-tile kernel
    long tiles128 = 0;
    for (int i = 0; i < b.n; ++i) tiles128 += (long)(h->layers[l0 + i - 1].n_in_p / 128) * (h->layers[l0 + i - 1].n_out_p / 128);
    const int cfg = (os.elem == ELEM_BF16 && h->tune_wgrad128_min > 0 && tiles128 >= h->tune_wgrad128_min) ? GEMM_128x1
                                                                                                             : h->tune_wgrad_cfg;
    double flops = 0;
    for (int i = 0; i < b.n; ++i) {
      const int l = l0 + (b.n - 1 - i);         // deepest layer first
      const LayerInfo& li = h->layers[l - 1];
      GemmProblem& p = b.p[i];
      const void* aT = l == 1 ? h->at<void>(sb.XT) : h->at<void>(sb.At[l - 1]);
      if (!rop) {
        set_pairs(p.g, aT, Bp, h->at<void>(sb.Dt[l]), Bp, Bp, nullptr, 0, nullptr, 0, 0);
        flops += 2.0 * B * li.n_in * li.n_out;
      } else if (l == 1) {
        set_pairs(p.g, aT, Bp, h->at<void>(os.RDt[l]), Bp, Bp, nullptr, 0, nullptr, 0, 0);
        flops += 2.0 * B * li.n_in * li.n_out;
      } else {
        set_pairs(p.g, h->at<void>(os.RAt[l - 1]), Bp, h->at<void>(sb.Dt[l]), Bp, Bp, aT, Bp,
                  h->at<void>(os.RDt[l]), Bp, Bp);
        flops += 4.0 * B * li.n_in * li.n_out;
      }
      p.g.M = li.n_in; p.g.N = li.n_out; p.g.Mp = li.n_in_p; p.g.Np = li.n_out_p;
      xcd_split(li.n_in_p / gemm_cfg_tile(cfg), li.n_out_p / gemm_cfg_tile(cfg), p.g.xgm, p.g.xgn);
      Epilogue e = blank_epilogue(k.mode);
      e.ldc = li.n_out;
      e.C = k.C ? k.C + li.w_off : nullptr;
      e.lam = k.lam ? k.lam + li.w_off : nullptr;
      e.x = k.x ? k.x + li.w_off : nullptr;
      e.v = k.v ? k.v + li.w_off : nullptr;
      e.p = k.p ? k.p + li.w_off : nullptr;
      e.alpha = k.alpha; e.beta = k.beta; e.gamma = k.gamma;
      if (k.copies) {
        e.out = h->at<void>(VN[l - 1]); e.ld = li.n_out_p;
        e.outT = h->at<void>(VT[l - 1]); e.ldT = li.n_in_p;
      }
      p.e = e;
      if (h->desc.has_bias) {
        BiasJob& j = b.bias[b.n_bias++];
        j.Mt = rop ? h->at<void>(os.RDt[l]) : h->at<void>(sb.Dt[l]);
        j.ld = Bp; j.rows = li.n_out; j.k = B; j.mode = k.mode;
        j.C = k.C ? k.C + li.b_off : nullptr;
        j.lam = k.lam ? k.lam + li.b_off : nullptr;
        j.x = k.x ? k.x + li.b_off : nullptr;
        j.v = k.v ? k.v + li.b_off : nullptr;
        j.p = k.p ? k.p + li.b_off : nullptr;
        j.alpha = k.alpha; j.beta = k.beta; j.gamma = k.gamma;
      }
    }
    double params = 0;
    for (int i = 0; i < b.n; ++i) {
      const LayerInfo& li = h->layers[l0 + i - 1];
      params += (double)li.n_in * li.n_out + (h->desc.has_bias ? li.n_out : 0);
    }
    // algorithmic bytes per parameter of the epilogue's vector work (fp32 vectors 4 B each way,
    // operand copies 2 x 2 B): Neumann step reads s, g (+ the diagonal), writes s and the copies
    double per_param = 4.0;
    if (k.mode == EPI_WGRAD_NEUMANN) per_param = 8.0 + 4.0 + (k.lam ? 4.0 : 0.0);
    else if (k.mode == EPI_WGRAD_NEUMANN_L2) per_param = 16.0 + 4.0;
    else if (k.mode == EPI_WGRAD_SGD) per_param = 16.0 + (k.lam ? 4.0 : 0.0);
    else if (k.mode == EPI_WGRAD_INIT) per_param = k.p ? 8.0 : 4.0;
    else if (k.lam) per_param = 12.0;
    if (k.copies) per_param += 4.0;
    launch_gemm_batch(h->ctx, os.elem, cfg, b, flops, per_param * params);
  }
}

// R-forward along the direction whose operand copies are in os.Vt and whose fp32 flat form is
// `vflat` (for the bias directions).  Leaves Rz_l (fp32) and Ra_l.
// With fuse_hessian (outputs of at most 32 columns) the last layer's epilogue applies the loss
// Hessian and leaves R delta_L instead of Rz_L.
void r_forward(betty_handle h, OperandSet& os, const float* vflat, bool fuse_hessian = false, int upto = 0) {
  SideBuf& sb = os.side[0];
  const int L = h->L, B = sb.B, Bp = sb.Bp;
  for (int l = 1; l <= (upto > 0 ? upto : L); ++l) {
    const LayerInfo& li = h->layers[l - 1];
    const bool last = l == L;
    const void* a_prev = l == 1 ? h->at<void>(sb.X) : h->at<void>(sb.A[l - 1]);
    Epilogue e = blank_epilogue(last ? (fuse_hessian ? EPI_RFWD_LAST_HESS : EPI_RFWD_LAST) : EPI_RFWD);
    e.colvec = h->desc.has_bias ? vflat + li.b_off : nullptr;
    e.f0 = h->f(os.Rz[l]);
    e.ldf = li.n_out_p;
    if (last && fuse_hessian) {
      e.act = h->desc.loss;
      e.dphi = h->desc.loss == BETTY_LOSS_SOFTMAX_CE ? h->f(sb.P) : nullptr;
      e.e = h->f(sb.s);
      e.out = h->at<void>(os.RD[l]); e.ld = li.n_out_p;
      e.outT = h->at<void>(os.RDt[l]); e.ldT = Bp;
    }
    if (!last) {
      e.dphi = h->f(sb.dphi[l]);
      e.out = h->at<void>(os.RA[l]); e.ld = li.n_out_p;
      e.outT = h->at<void>(os.RAt[l]); e.ldT = Bp;
    }
    if (l == 1)
      chain_gemm(h, os.elem, a_prev, li.n_in_p, h->at<void>(os.Vt[0]), li.n_in_p, li.n_in_p, nullptr, 0, nullptr,
                 0, 0, B, li.n_out, Bp, li.n_out_p, e, 2.0 * B * li.n_in * li.n_out);
    else
      chain_gemm(h, os.elem, h->at<void>(os.RA[l - 1]), li.n_in_p, h->at<void>(os.Wt[l - 1]), li.n_in_p,
                 li.n_in_p, a_prev, li.n_in_p, h->at<void>(os.Vt[l - 1]), li.n_in_p, li.n_in_p, B, li.n_out, Bp,
                 li.n_out_p, e, 4.0 * B * li.n_in * li.n_out);
  }
}

// One Hessian-vector product with the forward/backward cache of the train batch in place; the
// parameter-shaped result goes where `sink` says (plain store, or fused into the recurrence).
// The weight-gradient launch of layer l, enqueued on the second stream as soon as R delta_l exists.
void side_wgrad(betty_handle h, OperandSet& os, const WgradSink& sink, int l) {
  hipStream_t main = h->ctx.stream;
  hipError_t e = hipEventRecord(h->fork_events[l - 1], main);
  if (e == hipSuccess) e = hipStreamWaitEvent(h->side_stream, h->fork_events[l - 1], 0);
  if (e != hipSuccess && h->ctx.first_error == hipSuccess) h->ctx.first_error = e;
  h->ctx.stream = h->side_stream;
  wgrad_batch(h, os, 0, true, sink, l, l);
  h->ctx.stream = main;
}

void hvp_cached(betty_handle h, OperandSet& os, const float* vflat, const WgradSink& sink, bool pipelined = false) {
  SideBuf& sb = os.side[0];
  const int L = h->L, B = sb.B, Bp = sb.Bp;
  const bool pipe = pipelined && h->side_stream && L >= 2;
  const LayerInfo& lo = h->layers[L - 1];
  // a narrow output layer goes through one vector kernel: last R-forward product, loss Hessian and
  // the R-backward step through that layer
  const bool narrow_last = L >= 2 && lo.n_out <= LAST_ROP_MAX_C;
  const bool fused_hessian = !narrow_last && lo.n_out <= 32;
  r_forward(h, os, vflat, fused_hessian, narrow_last ? L - 1 : 0);
  if (narrow_last) {
    LastRopArgs a{};
    a.RA = h->at<void>(os.RA[L - 1]); a.A = h->at<void>(sb.A[L - 1]); a.lda = lo.n_in_p;
    a.Wt = h->at<void>(os.Wt[L - 1]); a.Vt = h->at<void>(os.Vt[L - 1]); a.ldt = lo.n_in_p;
    a.Wn = h->at<void>(os.Wn[L - 1]); a.Vn = h->at<void>(os.Vn[L - 1]); a.ldn = lo.n_out_p;
    a.cbias = h->desc.has_bias ? vflat + lo.b_off : nullptr;
    a.P = h->f(sb.P); a.s = h->f(sb.s); a.ldp = lo.n_out_p;
    a.DL = h->at<void>(sb.D[L]); a.ldd = lo.n_out_p;
    a.dphi = h->f(sb.dphi[L - 1]); a.e2 = sb.e2[L - 1] ? h->f(sb.e2[L - 1]) : nullptr;
    a.Rz = h->f(os.Rz[L - 1]); a.ldf = lo.n_in_p;
    a.RDL = h->at<void>(os.RD[L]); a.RDLt = h->at<void>(os.RDt[L]); a.ldRDLt = Bp;
    a.RD = h->at<void>(os.RD[L - 1]); a.ldRD = lo.n_in_p; a.RDt = h->at<void>(os.RDt[L - 1]); a.ldRDt = Bp;
    a.B = B; a.n_in = lo.n_in; a.n_in_p = lo.n_in_p; a.C = lo.n_out; a.loss = h->desc.loss;
    launch_last_layer_rop(h->ctx, os.elem, a);
    if (pipe) { side_wgrad(h, os, sink, L); side_wgrad(h, os, sink, L - 1); }
  } else {
    if (!fused_hessian)
      launch_loss_hessian_rows(h->ctx, os.elem, h->desc.loss, h->f(sb.P), h->f(os.Rz[L]), lo.n_out_p, h->f(sb.s), B,
                               lo.n_out, h->at<void>(os.RD[L]), lo.n_out_p, h->at<void>(os.RDt[L]), Bp);
    if (pipe) side_wgrad(h, os, sink, L);
  }
  for (int l = narrow_last ? L - 1 : L; l >= 2; --l) {
    const LayerInfo& li = h->layers[l - 1];
    Epilogue e = blank_epilogue(EPI_RBWD);
    e.dphi = h->f(sb.dphi[l - 1]);
    e.e = sb.e2[l - 1] ? h->f(sb.e2[l - 1]) : nullptr;
    e.Rz = h->f(os.Rz[l - 1]);
    e.ldf = li.n_in_p;
    e.out = h->at<void>(os.RD[l - 1]); e.ld = li.n_in_p;
    e.outT = h->at<void>(os.RDt[l - 1]); e.ldT = Bp;
    chain_gemm(h, os.elem, h->at<void>(os.RD[l]), li.n_out_p, h->at<void>(os.Wn[l - 1]), li.n_out_p, li.n_out_p,
               h->at<void>(sb.D[l]), li.n_out_p, h->at<void>(os.Vn[l - 1]), li.n_out_p, li.n_out_p, B, li.n_in, Bp,
               li.n_in_p, e, 4.0 * B * li.n_in * li.n_out);
    if (pipe) side_wgrad(h, os, sink, l - 1);
  }
  if (!pipe) {
    wgrad_batch(h, os, 0, true, sink);
    return;
  }
  // the next product reads every layer's new direction: the main stream waits for the second one
  hipError_t e = hipEventRecord(h->join_event, h->side_stream);
  if (e == hipSuccess) e = hipStreamWaitEvent(h->ctx.stream, h->join_event, 0);
  if (e != hipSuccess && h->ctx.first_error == hipSuccess) h->ctx.first_error = e;
}

// full first-order gradient of the lower cost at w (operand copies of w already made)
void lower_grad_seq(betty_handle h, OperandSet& os, const float* w, const float* lam, float* grad,
                    float* loss_or_null, const float* omega_fixed = nullptr, float* dist_or_null = nullptr) {
  const float* dl = diag_log(h, lam);
  // what the diagonal term multiplies: w itself, or its distance to the anchor (kept in vec_g
  // unless the caller names another place)
  const float* x = w;
  if (h->desc.hp == BETTY_HP_PROXIMAL) {
    float* dist = dist_or_null ? dist_or_null : h->f(h->vec_g);
    launch_diff(h->ctx, w, lam, dist, h->d);
    x = dist;
  }
  forward_backward(h, os, SIDE_TRAIN, w, wnet_theta(h, lam), omega_fixed);
  WgradSink k{EPI_WGRAD, grad, dl, dl ? x : nullptr, nullptr, nullptr, 0.f, false};
  wgrad_batch(h, os, 0, false, k);
  if (loss_or_null) {
    float* add = nullptr;
    if (dl) {
      add = h->f(h->scalars) + 8;
      launch_l2_cost(h->ctx, dl, x, h->d, h->at<double>(h->partials), add);
    }
    launch_weighted_loss_sum(h->ctx, h->f(os.side[0].s), h->f(os.side[0].ell), os.side[0].B, add, loss_or_null);
  }
}

// gradient of the upper cost on the validation batch; the result goes where `sink` says.  With
// with_lower the same launches also build the forward/backward cache of the train batch that the
// R-op passes need (no parameter gradient on that side).
void upper_grad_seq(betty_handle h, OperandSet& os, const float* w, const float* lam, bool with_lower,
                    const WgradSink& sink, float* loss_or_null) {
  const int sides = with_lower ? SIDE_BOTH : SIDE_VAL;
  forward_backward(h, os, sides, w, wnet_theta(h, lam));
  wgrad_batch(h, os, 1, false, sink);
  if (loss_or_null)
    launch_weighted_loss_sum(h->ctx, h->f(os.side[1].s), h->f(os.side[1].ell), os.side[1].B, nullptr, loss_or_null);
}

// forward/backward cache of the train batch for the R-op passes (no parameter gradient)
void prepare_lower(betty_handle h, OperandSet& os, const float* w, const float* lam) {
  forward_backward(h, os, SIDE_TRAIN, w, wnet_theta(h, lam));
}

// out = -(1/B) sum_i c_i dR/dtheta with c_i = <grad_w l_i, scale * qflat>
void mixed_reweight_seq(betty_handle h, OperandSet& os, const float* lam, const float* qflat, float scale,
                        float* out, bool copies_current = false) {
  SideBuf& sb = os.side[0];
  const int L = h->L;
  const LayerInfo& lo = h->layers[L - 1];
  // c_i is linear in the direction, so the scale is applied once, to the final sum over samples
  if (!copies_current) make_shadows(h, os, qflat, 1.f, nullptr, &os.Vt);   // else os.Vt already holds qflat
  if (L >= 2 && lo.n_out <= LAST_ROP_MAX_C) {
    // narrow output layer: the last product and the directional derivative in one vector kernel
    r_forward(h, os, qflat, false, L - 1);
    LastRopArgs a{};
    a.RA = h->at<void>(os.RA[L - 1]); a.A = h->at<void>(sb.A[L - 1]); a.lda = lo.n_in_p;
    a.Wt = h->at<void>(os.Wt[L - 1]); a.Vt = h->at<void>(os.Vt[L - 1]); a.ldt = lo.n_in_p;
    a.cbias = h->desc.has_bias ? qflat + lo.b_off : nullptr;
    a.P = h->f(sb.P); a.ldp = lo.n_out_p;
    a.B = sb.B; a.n_in = lo.n_in; a.n_in_p = lo.n_in_p; a.C = lo.n_out; a.loss = h->desc.loss;
    a.cvec = h->f(os.cvec); a.y = h->batch[0].y; a.Z = h->f(sb.ZL); a.target = h->batch[0].target;
    launch_last_layer_rop(h->ctx, os.elem, a);
  } else {
    r_forward(h, os, qflat);
    launch_loss_directional_rows(h->ctx, h->desc.loss, h->f(sb.P), h->f(sb.ZL), h->batch[0].y,
                                 h->batch[0].target, h->f(os.Rz[L]), lo.n_out_p, sb.B, lo.n_out, h->f(os.cvec));
  }
  launch_wnet_theta_vjp(h->ctx, h->f(sb.ell), h->f(sb.dsig), h->f(os.cvec), lam, h->desc.wnet_hidden, sb.B,
                        scale / (float)sb.B, out);
}

bool overlaps(const void* a, size_t na, const void* b, size_t nb) {
  const char* x = (const char*)a;
  const char* y = (const char*)b;
  return x < y + nb && y < x + na;
}

betty_status check_vec(betty_handle h, const void* p, const char* name) {
  if (!p) return fail(h, BETTY_ENULL, "%s is NULL", name);
  if (((uintptr_t)p) & 3) return fail(h, BETTY_EALIGN, "%s is not 4-byte aligned", name);
  return BETTY_OK;
}

betty_status check_ready(betty_handle h) {
  if (!h) return BETTY_ENULL;
  if (!h->bound) return fail(h, BETTY_EWORKSPACE, "no workspace bound (call betty_bind)");
  if (!h->batches) return fail(h, BETTY_EWORKSPACE, "batches not set (call betty_set_batches)");
  return BETTY_OK;
}

betty_status finish(betty_handle h) {
  if (h->ctx.first_error != hipSuccess) {
    betty_status st = fail(h, BETTY_EDEVICE, "HIP error: %s", hipGetErrorString(h->ctx.first_error));
    h->ctx.first_error = hipSuccess;
    return st;
  }
  return BETTY_OK;
}

#define CHECK(expr) do { betty_status st__ = (expr); if (st__ != BETTY_OK) return st__; } while (0)

}  // namespace

static void release_side_stream(betty_handle h) {
  for (hipEvent_t e : h->fork_events) if (e) (void)hipEventDestroy(e);
  h->fork_events.clear();
  if (h->join_event) (void)hipEventDestroy(h->join_event);
  h->join_event = nullptr;
  if (h->side_stream) (void)hipStreamDestroy(h->side_stream);
  h->side_stream = nullptr;
}

// What a workspace must hold before its first use: zero padding everywhere (fill kernels, no
// memset nodes), and for the proximal cost log(rho_j) per parameter.
static void init_workspace(betty_handle h) {
  launch_fill_zero(h->ctx, h->ws, h->ws_need);
  if (h->desc.hp == BETTY_HP_PROXIMAL) {
    // exp(-200) is exactly 0 in fp32, so parameters outside the proximal term get no curvature
    const LayerInfo& last = h->layers[h->L - 1];
    const size_t cut = h->desc.prox_skip_last ? last.w_off : h->d;
    const float lr = h->desc.prox_rho > 0.f ? std::log(h->desc.prox_rho) : -200.f;
    launch_fill_value(h->ctx, h->f(h->logrho), std::max(lr, -200.f), cut);
    if (cut < h->d) launch_fill_value(h->ctx, h->f(h->logrho) + cut, -200.f, h->d - cut);
  }
}

static unsigned long long next_epoch() {
  static std::atomic<unsigned long long> counter{0};
  return ++counter;
}

static void drop_graph(betty_handle_s::GraphSlot& g) {
  if (g.exec) (void)hipGraphExecDestroy(g.exec);
  if (g.graph) (void)hipGraphDestroy(g.graph);
  g = betty_handle_s::GraphSlot();
}

static void drop_graphs(betty_handle h) {
  drop_graph(h->graph_neumann); drop_graph(h->graph_fd); drop_graph(h->graph_cg); drop_graph(h->graph_br);
  drop_graph(h->graph_chain);
}

// Runs `body` (which only enqueues kernels on the bound stream) directly the first time a given
// argument set is seen, captures it into a graph the second time, and replays the graph from then
// on.  Any capture failure switches graphs off for the handle and runs the body directly.
template <typename Body>
static betty_status run_cached(betty_handle h, betty_handle_s::GraphSlot& g, const void* w, const void* lam,
                               const void* u, void* out, int K, float alpha, float eps, Body body,
                               int K2 = -1, float alpha2 = 0.f, const void* other = nullptr,
                               unsigned long long other_epoch = 0) {
  const bool eligible = h->use_graphs && !h->ctx.profiling && h->ctx.stream != nullptr;
  if (!eligible) { body(); return finish(h); }
  const bool same = g.seen > 0 && g.w == w && g.lam == lam && g.u == u && g.out == out && g.K == K &&
                    g.alpha == alpha && g.eps == eps && g.K2 == K2 && g.alpha2 == alpha2 && g.other == other &&
                    g.other_epoch == other_epoch;
  if (same && g.exec) {
    if (hipGraphLaunch(g.exec, h->ctx.stream) != hipSuccess) return fail(h, BETTY_EDEVICE, "hipGraphLaunch failed");
    return BETTY_OK;
  }
  if (!same) {
    drop_graph(g);
    g.w = w; g.lam = lam; g.u = u; g.out = out; g.K = K; g.alpha = alpha; g.eps = eps; g.seen = 1;
    g.K2 = K2; g.alpha2 = alpha2; g.other = other; g.other_epoch = other_epoch;
    body();
    return finish(h);
  }
  if (hipStreamBeginCapture(h->ctx.stream, hipStreamCaptureModeThreadLocal) != hipSuccess) {
    (void)hipGetLastError();
    h->use_graphs = false;
    body();
    return finish(h);
  }
  body();
  hipGraph_t graph = nullptr;
  const hipError_t e_end = hipStreamEndCapture(h->ctx.stream, &graph);
  hipGraphExec_t exec = nullptr;
  if (e_end != hipSuccess || h->ctx.first_error != hipSuccess || !graph ||
      hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0) != hipSuccess) {
    (void)hipGetLastError();
    if (graph) (void)hipGraphDestroy(graph);
    h->ctx.first_error = hipSuccess;
    h->use_graphs = false;
    body();                     // nothing ran during the failed capture
    return finish(h);
  }
  g.graph = graph; g.exec = exec;
  if (hipGraphLaunch(g.exec, h->ctx.stream) != hipSuccess) return fail(h, BETTY_EDEVICE, "hipGraphLaunch failed");
  return BETTY_OK;
}

static betty_status check_hyper_args(betty_handle h, const float* w, const float* lambda, int K, float alpha,
                                     float* dlambda) {
  CHECK(check_ready(h));
  CHECK(check_vec(h, w, "w")); CHECK(check_vec(h, lambda, "lambda")); CHECK(check_vec(h, dlambda, "dlambda"));
  if (K < 0) return fail(h, BETTY_EINVAL, "K must be >= 0 (got %d)", K);
  if (!std::isfinite(alpha)) return fail(h, BETTY_EINVAL, "alpha must be finite");
  if (overlaps(dlambda, h->n_hyper * 4, w, h->d * 4) || overlaps(dlambda, h->n_hyper * 4, lambda, h->n_hyper * 4))
    return fail(h, BETTY_EINVAL, "dlambda overlaps an input");
  return BETTY_OK;
}

// out = (dw* / dlambda) u by the K-step Neumann series and the mixed VJP; u = grad_w L_U(w) on the
// validation batch when u_or_null is null.  Only enqueues launches on the handle's stream.
// The partial sum is carried in nested form, s <- g + (I - alpha H) s from s = g: after K steps
// s = sum_{j<=K} (I - alpha H)^j g, with one parameter-sized state vector to read and write per step.
static void neumann_seq(betty_handle h, const float* w, const float* lambda, const float* u_or_null, int K,
                        float alpha, float* out) {
  OperandSet& os = h->sets[0];
  const bool l2 = h->desc.hp == BETTY_HP_L2_DECAY, rw = h->desc.hp == BETTY_HP_REWEIGHT_NET;
  const float* dl = diag_log(h, lambda);
  float* s = h->f(h->vec_p);
  const float* g = u_or_null;
  const bool need_lower = K > 0 || rw;      // forward/backward cache of the train batch
  make_weight_operands(h, os, w);
  // the reweighting mixed term runs one more R-forward along the final sum: its operand copies are
  // written by whichever launch produces that sum
  if (u_or_null) {
    if (need_lower) prepare_lower(h, os, w, lambda);
    if (K > 0 || rw) make_shadows(h, os, u_or_null, 1.f, &os.Vn, &os.Vt);
  } else {
    // g = grad_w L_U lands in vec_v, with its operand copies for the first product
    WgradSink init{EPI_WGRAD_INIT, nullptr, nullptr, nullptr, h->f(h->vec_v), nullptr, 0.f, K > 0 || rw};
    upper_grad_seq(h, os, w, lambda, need_lower, init, nullptr);
    g = h->f(h->vec_v);
  }
  const float* s_cur = g;                   // s_0 = g
  for (int k = 0; k < K; ++k) {
    // the step is fused into the weight-gradient epilogues of the product; for L2 decay the last
    // step also applies the mixed VJP, so only d(lambda) is written.
    // With the second stream, layer l's launch runs while the R-backward chain is still reading
    // this product's direction copies of the layers below, so the new copies go to the other set.
    const bool last = k + 1 == K;
    const bool pipe = h->use_pipeline && h->side_stream && h->L >= 2;
    if (last && l2) {
      WgradSink fin{EPI_WGRAD_NEUMANN_L2, out, lambda, w, const_cast<float*>(g), const_cast<float*>(s_cur), alpha, false};
      hvp_cached(h, os, s_cur, fin, pipe);
    } else {
      WgradSink step{EPI_WGRAD_NEUMANN, nullptr, dl, s_cur, const_cast<float*>(g), s, alpha, !last || rw};
      step.second_set = pipe;
      hvp_cached(h, os, s_cur, step, pipe);
      if (pipe && step.copies) { std::swap(os.Vn, os.Vn2); std::swap(os.Vt, os.Vt2); }
    }
    s_cur = s;
  }
  if (l2) {
    if (K == 0) launch_mixed_l2(h->ctx, lambda, w, s_cur, alpha, out, h->d);
  } else if (rw) {
    mixed_reweight_seq(h, os, lambda, s_cur, alpha, out, true);
  } else {
    launch_mixed_prox(h->ctx, h->f(h->logrho), s_cur, alpha, out, h->d);
  }
}

extern "C" {

betty_status betty_create(const betty_problem_desc* desc, betty_handle* out) {
  if (!desc || !out) return BETTY_ENULL;
  *out = nullptr;
  if (!desc->dims) return BETTY_ENULL;
  if (desc->n_layers < 1 || desc->n_layers > 64) return BETTY_ESHAPE;
  for (int i = 0; i <= desc->n_layers; ++i)
    if (desc->dims[i] < 1 || desc->dims[i] > (1 << 20)) return BETTY_ESHAPE;
  if (desc->batch_train < 1 || desc->batch_val < 1 || desc->batch_train > (1 << 20) || desc->batch_val > (1 << 20))
    return BETTY_ESHAPE;
  if (desc->act < BETTY_ACT_NONE || desc->act > BETTY_ACT_GELU_ERF) return BETTY_EINVAL;
  if (desc->loss != BETTY_LOSS_MSE && desc->loss != BETTY_LOSS_SOFTMAX_CE) return BETTY_EINVAL;
  if (desc->hp != BETTY_HP_L2_DECAY && desc->hp != BETTY_HP_REWEIGHT_NET && desc->hp != BETTY_HP_PROXIMAL)
    return BETTY_EINVAL;
  if (desc->hp == BETTY_HP_PROXIMAL && !(std::isfinite(desc->prox_rho) && desc->prox_rho >= 0.f)) return BETTY_EINVAL;
  if (desc->prec != BETTY_PREC_FP32 && desc->prec != BETTY_PREC_BF16_FP32ACC) return BETTY_EINVAL;
  if (desc->hp == BETTY_HP_REWEIGHT_NET && (desc->wnet_hidden < 1 || desc->wnet_hidden > 65536)) return BETTY_ESHAPE;

  // the kernels index one matrix (a layer's weights, an activation) with 32-bit offsets
  {
    const long long bp = padup(std::max(desc->batch_train, desc->batch_val));
    for (int i = 0; i < desc->n_layers; ++i) {
      const long long a = padup(desc->dims[i]), b = padup(desc->dims[i + 1]);
      if (a * b >= (1LL << 31) || bp * a >= (1LL << 31) || bp * b >= (1LL << 31)) return BETTY_ESHAPE;
    }
  }

  betty_handle h = new (std::nothrow) betty_handle_s();
  if (!h) return BETTY_EDEVICE;
  h->desc = *desc;
  h->dims.assign(desc->dims, desc->dims + desc->n_layers + 1);
  h->desc.dims = h->dims.data();
  h->L = desc->n_layers;
  size_t off = 0;
  for (int l = 0; l < h->L; ++l) {
    LayerInfo li{};
    li.n_in = h->dims[l]; li.n_out = h->dims[l + 1];
    li.n_in_p = padup(li.n_in); li.n_out_p = padup(li.n_out);
    li.w_off = off; off += (size_t)li.n_in * li.n_out;
    li.b_off = off;
    if (desc->has_bias) off += li.n_out;
    h->layers.push_back(li);
    h->max_np = std::max(h->max_np, std::max(li.n_in_p, li.n_out_p));
  }
  h->d = off;
  h->n_hyper = desc->hp == BETTY_HP_REWEIGHT_NET ? (size_t)3 * desc->wnet_hidden + 1 : h->d;
  // Large models with fp32 operands overlap each layer's weight-gradient launch with the R-backward
  // chain (see use_pipeline).  With bf16 operands their weight gradients take the 128-tile kernel,
  // all layers in one launch behind the chain: measured on the 121M-parameter model, 7.23 ms per
  // hypergradient against 7.49 ms for the overlapped 64-tile launches and 8.37 ms for overlapped
  // 128-tile ones (the two streams contend for the same memory path).
  const bool large = h->d >= ((size_t)32 << 20);
  h->use_pipeline = large && desc->prec == BETTY_PREC_FP32;
  h->fd_two_streams = !large;
  h->max_Bp = std::max(padup(desc->batch_train), padup(desc->batch_val));
  // tuning overrides for experiments: BETTY_TUNE="wgrad=<cfg>,wgrad128=<n>,tile128=<n>,blocks=<n>,rect=<n>,rectk=<n>,pipe=<0|1>,fd2=<0|1>" (see plan_chain)
  if (const char* t = getenv("BETTY_TUNE")) {
    int v;
    if (const char* q = strstr(t, "wgrad=")) if (sscanf(q + 6, "%d", &v) == 1 && (v == GEMM_128x1 || v == GEMM_64x1)) h->tune_wgrad_cfg = v;
    if (const char* q = strstr(t, "tile128=")) if (sscanf(q + 8, "%d", &v) == 1 && v > 0) h->tune_tile128_min = v;
    if (const char* q = strstr(t, "blocks=")) if (sscanf(q + 7, "%d", &v) == 1 && v > 0) h->tune_target_blocks = v;
    if (const char* q = strstr(t, "rect=")) if (sscanf(q + 5, "%d", &v) == 1 && v >= 0) h->tune_rect_max = v;
    if (const char* q = strstr(t, "rectk=")) if (sscanf(q + 6, "%d", &v) == 1 && v > 0) h->tune_rect_min_tt = v;
    if (const char* q = strstr(t, "wgrad128=")) if (sscanf(q + 9, "%d", &v) == 1 && v >= 0) h->tune_wgrad128_min = v;
    if (const char* q = strstr(t, "pipe=")) if (sscanf(q + 5, "%d", &v) == 1) h->use_pipeline = v != 0;
    if (const char* q = strstr(t, "fd2=")) if (sscanf(q + 4, "%d", &v) == 1) h->fd_two_streams = v != 0;
  }
  plan(h);
  *out = h;
  return BETTY_OK;
}

void betty_destroy(betty_handle h) {
  if (!h) return;
  drop_graphs(h);
  release_side_stream(h);
  for (auto& r : h->ctx.recs) { (void)hipEventDestroy(r.e0); (void)hipEventDestroy(r.e1); }
  delete h;
}

const char* betty_last_error(betty_handle h) { return h ? h->err.c_str() : "null handle"; }
size_t betty_num_params(betty_handle h) { return h ? h->d : 0; }
size_t betty_num_hyper(betty_handle h) { return h ? h->n_hyper : 0; }
size_t betty_workspace_bytes(betty_handle h) { return h ? h->ws_need : 0; }

betty_status betty_bind(betty_handle h, void* workspace, size_t bytes, void* hip_stream) {
  if (!h) return BETTY_ENULL;
  if (!workspace) return fail(h, BETTY_ENULL, "workspace is NULL");
  if (((uintptr_t)workspace) & 255) return fail(h, BETTY_EALIGN, "workspace is not 256-byte aligned");
  if (bytes < h->ws_need) return fail(h, BETTY_EWORKSPACE, "workspace has %zu bytes, %zu needed", bytes, h->ws_need);
  h->ws = (char*)workspace;
  h->ctx.stream = (hipStream_t)hip_stream;
  if (!h->side_stream && hip_stream != nullptr) {
    // second stream (default priority) and the events that order it against the bound stream
    bool ok = hipStreamCreateWithFlags(&h->side_stream, hipStreamNonBlocking) == hipSuccess;
    h->fork_events.assign(h->L, nullptr);
    for (int l = 0; ok && l < h->L; ++l)
      ok = hipEventCreateWithFlags(&h->fork_events[l], hipEventDisableTiming) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&h->join_event, hipEventDisableTiming) == hipSuccess;
    if (!ok) { (void)hipGetLastError(); release_side_stream(h); }
  }
  drop_graphs(h);
  h->epoch = next_epoch();
  h->bound = true;
  h->batches = false;
  init_workspace(h);
  return finish(h);
}

betty_status betty_set_batches(betty_handle h, betty_batch train, betty_batch val) {
  if (!h) return BETTY_ENULL;
  if (!h->bound) return fail(h, BETTY_EWORKSPACE, "no workspace bound (call betty_bind)");
  const betty_batch b[2] = {train, val};
  for (int s = 0; s < 2; ++s) {
    CHECK(check_vec(h, b[s].x, s ? "val.x" : "train.x"));
    if (h->desc.loss == BETTY_LOSS_SOFTMAX_CE) CHECK(check_vec(h, b[s].y, s ? "val.y" : "train.y"));
    else CHECK(check_vec(h, b[s].target, s ? "val.target" : "train.target"));
  }
  drop_graphs(h);
  h->epoch = next_epoch();
  h->batch[0] = train;
  h->batch[1] = val;
  const LayerInfo& l0 = h->layers[0];
  for (int k = 0; k < 2; ++k) {
    OperandSet& os = h->sets[k];
    if (!os.present) continue;
    for (int s = 0; s < 2; ++s) {
      SideBuf& sb = os.side[s];
      launch_convert_dual(h->ctx, os.elem, b[s].x, l0.n_in, 1.f, sb.B, l0.n_in, h->at<void>(sb.X), l0.n_in_p,
                          h->at<void>(sb.XT), sb.Bp);
    }
  }
  if (h->fd_minus.present) {
    SideBuf& sb = h->fd_minus.side[0];
    launch_convert_dual(h->ctx, ELEM_F32, b[0].x, l0.n_in, 1.f, sb.B, l0.n_in, h->at<void>(sb.X), l0.n_in_p,
                        h->at<void>(sb.XT), sb.Bp);
  }
  h->batches = true;
  return finish(h);
}

betty_status betty_lower_grad(betty_handle h, const float* w, const float* lambda, float* grad_w,
                              float* loss_or_null) {
  CHECK(check_ready(h));
  CHECK(check_vec(h, w, "w")); CHECK(check_vec(h, lambda, "lambda")); CHECK(check_vec(h, grad_w, "grad_w"));
  if (loss_or_null) CHECK(check_vec(h, loss_or_null, "loss"));
  if (overlaps(grad_w, h->d * 4, w, h->d * 4) || overlaps(grad_w, h->d * 4, lambda, h->n_hyper * 4))
    return fail(h, BETTY_EINVAL, "grad_w overlaps an input");
  OperandSet& os = h->sets[0];
  make_weight_operands(h, os, w);
  lower_grad_seq(h, os, w, lambda, grad_w, loss_or_null);
  return finish(h);
}

betty_status betty_upper_grad(betty_handle h, const float* w, float* grad_w, float* loss_or_null) {
  CHECK(check_ready(h));
  CHECK(check_vec(h, w, "w")); CHECK(check_vec(h, grad_w, "grad_w"));
  if (loss_or_null) CHECK(check_vec(h, loss_or_null, "loss"));
  if (overlaps(grad_w, h->d * 4, w, h->d * 4)) return fail(h, BETTY_EINVAL, "grad_w overlaps w");
  OperandSet& os = h->sets[0];
  make_weight_operands(h, os, w);
  WgradSink k{EPI_WGRAD, grad_w, nullptr, nullptr, nullptr, nullptr, 0.f, false};
  upper_grad_seq(h, os, w, nullptr, false, k, loss_or_null);
  return finish(h);
}

static betty_status check_hvp_args(betty_handle h, const float* w, const float* lambda, const float* v, float* Hv) {
  CHECK(check_vec(h, w, "w")); CHECK(check_vec(h, lambda, "lambda")); CHECK(check_vec(h, v, "v"));
  CHECK(check_vec(h, Hv, "Hv"));
  if (overlaps(Hv, h->d * 4, w, h->d * 4) || overlaps(Hv, h->d * 4, v, h->d * 4) ||
      overlaps(Hv, h->d * 4, lambda, h->n_hyper * 4))
    return fail(h, BETTY_EINVAL, "Hv overlaps an input");
  return BETTY_OK;
}

// one stand-alone Hessian-vector product: operand copies of w, the forward/backward cache of the
// train batch, operand copies of v, the forward-over-reverse passes
static void hvp_seq(betty_handle h, const float* w, const float* lambda, const float* v, float* Hv) {
  OperandSet& os = h->sets[0];
  make_weight_operands(h, os, w);
  prepare_lower(h, os, w, lambda);
  make_shadows(h, os, v, 1.f, &os.Vn, &os.Vt);
  const float* dl = diag_log(h, lambda);
  WgradSink k{EPI_WGRAD, Hv, dl, dl ? v : nullptr, nullptr, nullptr, 0.f, false};
  hvp_cached(h, os, v, k);
}

betty_status betty_hvp(betty_handle h, const float* w, const float* lambda, const float* v, float* Hv) {
  CHECK(check_ready(h));
  CHECK(check_hvp_args(h, w, lambda, v, Hv));
  hvp_seq(h, w, lambda, v, Hv);
  return finish(h);
}

// ---- the same product for callers that cannot allocate device memory ----------------------
// The workspace is a fixed array in the library's device image; every GPU the library runs on has
// its own copy at its own address, looked up once per device.
static __device__ __align__(256) unsigned char scratch[BETTY_STATIC_SCRATCH_BYTES];

static betty_status static_scratch(betty_handle h, char** out) {
  constexpr int MAX_DEVICES = 64;
  static std::mutex mu;
  static char* base[MAX_DEVICES] = {};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES)
    return fail(h, BETTY_EDEVICE, "no current HIP device (or its index is beyond %d)", MAX_DEVICES - 1);
  std::lock_guard<std::mutex> lock(mu);
  if (!base[dev]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return fail(h, BETTY_EDEVICE, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
    base[dev] = (char*)p;
  }
  *out = base[dev];
  return BETTY_OK;
}

size_t betty_static_scratch_bytes(void) { return BETTY_STATIC_SCRATCH_BYTES; }

betty_status betty_hvp_static(betty_handle h, betty_batch train, void* hip_stream, const float* w,
                              const float* lambda, const float* v, float* Hv) {
  if (!h) return BETTY_ENULL;
  CHECK(check_hvp_args(h, w, lambda, v, Hv));
  CHECK(check_vec(h, train.x, "train.x"));
  if (h->desc.loss == BETTY_LOSS_SOFTMAX_CE) CHECK(check_vec(h, train.y, "train.y"));
  else CHECK(check_vec(h, train.target, "train.target"));
  if (h->ws_need > BETTY_STATIC_SCRATCH_BYTES)
    return fail(h, BETTY_EWORKSPACE, "this problem needs %zu bytes of workspace, the library's fixed scratch array holds %zu: "
                "use betty_bind with a caller-owned workspace and betty_hvp", h->ws_need, (size_t)BETTY_STATIC_SCRATCH_BYTES);
  char* base = nullptr;
  CHECK(static_scratch(h, &base));
  // run on the scratch array and the given stream, with the handle's own binding set aside
  char* const ws0 = h->ws;
  const hipStream_t st0 = h->ctx.stream;
  const bool prof0 = h->ctx.profiling;
  const betty_batch b0 = h->batch[0], b1 = h->batch[1];
  h->ws = base;
  h->ctx.stream = (hipStream_t)hip_stream;
  h->ctx.profiling = false;                         // (event creation allocates)
  h->batch[0] = train;
  h->batch[1] = train;
  init_workspace(h);                                // the array keeps the last call's contents
  OperandSet& os = h->sets[0];
  const LayerInfo& l0 = h->layers[0];
  SideBuf& sb = os.side[0];
  launch_convert_dual(h->ctx, os.elem, train.x, l0.n_in, 1.f, sb.B, l0.n_in, h->at<void>(sb.X), l0.n_in_p,
                      h->at<void>(sb.XT), sb.Bp);
  if (hybrid_forward(h, os)) {                      // the fp32 forward of ReLU networks reads its own copy of X
    SideBuf& fb = h->sets[1].side[0];
    launch_convert_dual(h->ctx, ELEM_F32, train.x, l0.n_in, 1.f, fb.B, l0.n_in, h->at<void>(fb.X), l0.n_in_p,
                        h->at<void>(fb.XT), fb.Bp);
  }
  hvp_seq(h, w, lambda, v, Hv);
  h->ws = ws0;
  h->ctx.stream = st0;
  h->ctx.profiling = prof0;
  h->batch[0] = b0;
  h->batch[1] = b1;
  return finish(h);
}

betty_status betty_mixed_vjp(betty_handle h, const float* w, const float* lambda, const float* q, float* out) {
  CHECK(check_ready(h));
  CHECK(check_vec(h, w, "w")); CHECK(check_vec(h, lambda, "lambda")); CHECK(check_vec(h, q, "q"));
  CHECK(check_vec(h, out, "out"));
  if (overlaps(out, h->n_hyper * 4, w, h->d * 4) || overlaps(out, h->n_hyper * 4, q, h->d * 4) ||
      overlaps(out, h->n_hyper * 4, lambda, h->n_hyper * 4))
    return fail(h, BETTY_EINVAL, "out overlaps an input");
  if (h->desc.hp == BETTY_HP_L2_DECAY) {
    launch_mixed_l2(h->ctx, lambda, w, q, 1.f, out, h->d);
    return finish(h);
  }
  if (h->desc.hp == BETTY_HP_PROXIMAL) {
    launch_mixed_prox(h->ctx, h->f(h->logrho), q, 1.f, out, h->d);
    return finish(h);
  }
  OperandSet& os = h->sets[0];
  make_weight_operands(h, os, w);
  forward_and_loss(h, os, SIDE_TRAIN, w, lambda);
  mixed_reweight_seq(h, os, lambda, q, 1.f, out);
  return finish(h);
}

betty_status betty_hypergrad_neumann(betty_handle h, const float* w, const float* lambda, int K, float alpha,
                                     float* dlambda) {
  CHECK(check_hyper_args(h, w, lambda, K, alpha, dlambda));
  auto body = [=]() { neumann_seq(h, w, lambda, nullptr, K, alpha, dlambda); };
  return run_cached(h, h->graph_neumann, w, lambda, nullptr, dlambda, K, alpha, 0.f, body);
}

betty_status betty_best_response_neumann(betty_handle h, const float* w, const float* lambda, const float* u, int K,
                                         float alpha, float* out) {
  CHECK(check_hyper_args(h, w, lambda, K, alpha, out));
  CHECK(check_vec(h, u, "u"));
  if (overlaps(out, h->n_hyper * 4, u, h->d * 4)) return fail(h, BETTY_EINVAL, "out overlaps u");
  auto body = [=]() { neumann_seq(h, w, lambda, u, K, alpha, out); };
  return run_cached(h, h->graph_br, w, lambda, u, out, K, alpha, 0.f, body);
}

betty_status betty_hypergrad_chain3(betty_handle hp, betty_handle hf, const float* w, const float* theta,
                                    const float* v, int K_pre, float alpha_pre, int K_ft, float alpha_ft,
                                    float* dtheta) {
  if (!hp || !hf) return BETTY_ENULL;
  CHECK(check_hyper_args(hp, w, theta, K_pre, alpha_pre, dtheta));
  if (check_ready(hf) != BETTY_OK) return fail(hp, BETTY_EWORKSPACE, "finetune handle: %s", hf->err.c_str());
  if (hf->desc.hp != BETTY_HP_PROXIMAL) return fail(hp, BETTY_EINVAL, "the finetune handle must be BETTY_HP_PROXIMAL");
  if (hf->d != hp->d) return fail(hp, BETTY_ESHAPE, "finetune handle has %zu parameters, pretrain handle %zu", hf->d, hp->d);
  if (hf->ctx.stream != hp->ctx.stream) return fail(hp, BETTY_EINVAL, "both handles must be bound to the same stream");
  CHECK(check_vec(hp, v, "v"));
  if (K_ft < 0) return fail(hp, BETTY_EINVAL, "K_finetune must be >= 0 (got %d)", K_ft);
  if (!std::isfinite(alpha_ft)) return fail(hp, BETTY_EINVAL, "alpha_finetune must be finite");
  if (overlaps(dtheta, hp->n_hyper * 4, v, hp->d * 4)) return fail(hp, BETTY_EINVAL, "dtheta overlaps v");
  // rightmost factor first: u = (dv* / dw) grad_v L_U(v) on the finetuning problem (anchor w),
  // kept in that handle's workspace; then (dw* / dtheta) u on the pretraining problem
  if (hf->ctx.profiling) return fail(hp, BETTY_EINVAL, "switch per-launch timing off on the finetune handle first");
  auto body = [=]() {
    float* u = hf->f(hf->vec_g);
    neumann_seq(hf, v, w, nullptr, K_ft, alpha_ft, u);
    if (hf->ctx.first_error != hipSuccess) {          // reported through the pretrain handle
      if (hp->ctx.first_error == hipSuccess) hp->ctx.first_error = hf->ctx.first_error;
      hf->ctx.first_error = hipSuccess;
    }
    neumann_seq(hp, w, theta, u, K_pre, alpha_pre, dtheta);
  };
  // repeated identical calls replay one captured graph that spans both handles (same stream); the
  // finetune handle's workspace and batches are part of what the graph has recorded, so its stamp
  // is part of the key
  return run_cached(hp, hp->graph_chain, w, theta, v, dtheta, K_pre, alpha_pre, 0.f, body, K_ft, alpha_ft, hf,
                    hf->epoch);
}

betty_status betty_hypergrad_fd(betty_handle h, const float* w, const float* lambda, int K, float alpha,
                                float eps_scale, float* dlambda) {
  CHECK(check_hyper_args(h, w, lambda, K, alpha, dlambda));
  if (!std::isfinite(eps_scale) || eps_scale <= 0.f) return fail(h, BETTY_EINVAL, "eps_scale must be positive and finite");
  auto body = [=]() {
    OperandSet& os = fd_operands(h);
    SideBuf& sb = os.side[0];
    const bool l2 = h->desc.hp == BETTY_HP_L2_DECAY, rw = h->desc.hp == BETTY_HP_REWEIGHT_NET;
    float* v = h->f(h->vec_v); float* p = h->f(h->vec_p); float* Gp = h->f(h->vec_Hv);
    float* Gm = h->f(h->vec_Gm); float* wpm = h->f(h->vec_wpm); float* wpm2 = h->f(h->vec_wpm2);
    OperandSet& om = h->fd_minus;
    float* nrm2 = h->f(h->scalars); float* eps = h->f(h->scalars) + 1;
    make_weight_operands(h, os, w);
    WgradSink init{EPI_WGRAD_INIT, nullptr, nullptr, nullptr, v, p, 0.f, false};
    const float* omega_bar = nullptr;
    if (!rw) {
      upper_grad_seq(h, os, w, nullptr, false, init, nullptr);
    } else {
      // the reweighting cost holds its sample weights constant in w: evaluate them (and the loss fed
      // to the weight net) once at the unperturbed w and keep them for every perturbed pass
      forward_and_loss(h, os, SIDE_BOTH, w, lambda);
      backward_chain(h, os, SIDE_VAL);
      wgrad_batch(h, os, 1, false, init);
      launch_scale_copy(h->ctx, h->f(sb.ell), 1.f, h->f(sb.ell_bar), sb.B);
      launch_scale_copy(h->ctx, h->f(sb.omega), 1.f, h->f(sb.omega_bar), sb.B);
      launch_scale_copy(h->ctx, h->f(sb.dsig), 1.f, h->f(sb.dsig_bar), sb.B);
      omega_bar = h->f(sb.omega_bar);
    }
    for (int k = 0; k < K; ++k) {
      launch_sumsq(h->ctx, v, h->d, h->at<double>(h->partials), nrm2);
      launch_fd_eps(h->ctx, nrm2, eps_scale, 1.f, eps);
      // the evaluation at w - eps v goes to the second stream, with operands and scratch of its own
      hipStream_t main = h->ctx.stream;
      const bool two = h->fd_minus.present && h->side_stream != nullptr;
      if (two) {
        hipError_t e = hipEventRecord(h->fork_events[0], main);
        if (e == hipSuccess) e = hipStreamWaitEvent(h->side_stream, h->fork_events[0], 0);
        if (e != hipSuccess && h->ctx.first_error == hipSuccess) h->ctx.first_error = e;
        h->ctx.stream = h->side_stream;
        launch_fd_perturb(h->ctx, w, v, eps, -1.f, wpm2, h->d);
        make_weight_operands(h, om, wpm2);
        lower_grad_seq(h, om, wpm2, lambda, Gm, nullptr, omega_bar, h->vec_g2 ? h->f(h->vec_g2) : nullptr);
        h->ctx.stream = main;
      }
      launch_fd_perturb(h->ctx, w, v, eps, +1.f, wpm, h->d);
      make_weight_operands(h, os, wpm);
      lower_grad_seq(h, os, wpm, lambda, Gp, nullptr, omega_bar);
      if (two) {
        hipError_t e = hipEventRecord(h->join_event, h->side_stream);
        if (e == hipSuccess) e = hipStreamWaitEvent(main, h->join_event, 0);
        if (e != hipSuccess && h->ctx.first_error == hipSuccess) h->ctx.first_error = e;
      } else {
        launch_fd_perturb(h->ctx, w, v, eps, -1.f, wpm, h->d);
        make_weight_operands(h, os, wpm);
        lower_grad_seq(h, os, wpm, lambda, Gm, nullptr, omega_bar);
      }
      launch_fd_update(h->ctx, v, p, Gp, Gm, eps, alpha, h->d);
    }
    launch_sumsq(h->ctx, p, h->d, h->at<double>(h->partials), nrm2);
    launch_fd_eps(h->ctx, nrm2, eps_scale, alpha, eps);
    if (l2) {
      launch_mixed_l2_fd(h->ctx, lambda, w, p, alpha, eps, dlambda, h->d);
    } else if (!rw) {
      // grad_a of the proximal cost is linear in w, so its central difference along q is exact
      launch_mixed_prox(h->ctx, h->f(h->logrho), p, alpha, dlambda, h->d);
    } else {
      // grad_theta L_L(w') = (1/B) sum_i l_i(w') dR(lbar_i)/dtheta, so its central difference along
      // q = alpha p needs only the per-sample losses at w +- eps q
      launch_scale_copy(h->ctx, p, alpha, v, h->d);                       // v := q (v is no longer needed)
      launch_fd_perturb(h->ctx, w, v, eps, +1.f, wpm, h->d);
      make_weight_operands(h, os, wpm);
      forward_and_loss(h, os, SIDE_TRAIN, wpm, lambda, omega_bar);
      launch_scale_copy(h->ctx, h->f(sb.ell), 1.f, h->f(sb.ell_p), sb.B);
      launch_fd_perturb(h->ctx, w, v, eps, -1.f, wpm, h->d);
      make_weight_operands(h, os, wpm);
      forward_and_loss(h, os, SIDE_TRAIN, wpm, lambda, omega_bar);
      launch_fd_loss_diff(h->ctx, h->f(sb.ell_p), h->f(sb.ell), eps, sb.B, h->f(os.cvec));
      launch_wnet_theta_vjp(h->ctx, h->f(sb.ell_bar), h->f(sb.dsig_bar), h->f(os.cvec), lambda,
                            h->desc.wnet_hidden, sb.B, 1.0f / (float)sb.B, dlambda);
    }
  };
  return run_cached(h, h->graph_fd, w, lambda, nullptr, dlambda, K, alpha, eps_scale, body);
}

betty_status betty_hypergrad_cg(betty_handle h, const float* w, const float* lambda, int K, float* dlambda) {
  CHECK(check_hyper_args(h, w, lambda, K, 0.f, dlambda));
  auto body = [=]() {
    OperandSet& os = h->sets[0];
    const bool l2 = h->desc.hp == BETTY_HP_L2_DECAY, rw = h->desc.hp == BETTY_HP_REWEIGHT_NET;
    const float* dl = diag_log(h, lambda);
    float* r = h->f(h->vec_g); float* d = h->f(h->vec_v); float* q = h->f(h->vec_p); float* Hd = h->f(h->vec_Hv);
    float* sc = h->f(h->scalars);            // sc[0], sc[1]: r.r of the current / next iterate; sc[2]: d.Hd
    double* partials = h->at<double>(h->partials);
    make_weight_operands(h, os, w);
    WgradSink g_out{EPI_WGRAD, r, nullptr, nullptr, nullptr, nullptr, 0.f, false};
    upper_grad_seq(h, os, w, lambda, K > 0 || rw, g_out, nullptr);
    launch_cg_init(h->ctx, r, d, q, h->d);
    launch_sumsq(h->ctx, r, h->d, partials, sc);
    for (int k = 0; k < K; ++k) {
      float* rs = sc + (k & 1);
      float* rs_new = sc + ((k + 1) & 1);
      make_shadows(h, os, d, 1.f, &os.Vn, &os.Vt);
      WgradSink hd{EPI_WGRAD, Hd, dl, dl ? d : nullptr, nullptr, nullptr, 0.f, false};
      hvp_cached(h, os, d, hd);
      launch_dot(h->ctx, d, Hd, h->d, partials, sc + 2);
      launch_cg_step(h->ctx, q, r, d, Hd, rs, sc + 2, h->d, partials, rs_new);
      if (k + 1 < K) launch_cg_dir(h->ctx, d, r, rs, rs_new, h->d);
    }
    if (l2) launch_mixed_l2(h->ctx, lambda, w, q, 1.f, dlambda, h->d);
    else if (rw) mixed_reweight_seq(h, os, lambda, q, 1.f, dlambda);
    else launch_mixed_prox(h->ctx, h->f(h->logrho), q, 1.f, dlambda, h->d);
  };
  return run_cached(h, h->graph_cg, w, lambda, nullptr, dlambda, K, 0.f, -1.f, body);
}

betty_status betty_lower_sgd_step(betty_handle h, float* w, const float* lambda, float* momentum, float lr, float mu,
                                  float weight_decay, float* loss_or_null) {
  CHECK(check_ready(h));
  CHECK(check_vec(h, w, "w")); CHECK(check_vec(h, lambda, "lambda")); CHECK(check_vec(h, momentum, "momentum"));
  if (loss_or_null) CHECK(check_vec(h, loss_or_null, "loss"));
  if (!std::isfinite(lr) || !std::isfinite(mu) || !std::isfinite(weight_decay))
    return fail(h, BETTY_EINVAL, "lr, mu and weight_decay must be finite");
  if (overlaps(w, h->d * 4, momentum, h->d * 4) || overlaps(w, h->d * 4, lambda, h->n_hyper * 4) ||
      overlaps(momentum, h->d * 4, lambda, h->n_hyper * 4))
    return fail(h, BETTY_EINVAL, "w, momentum and lambda must not overlap");
  OperandSet& os = h->sets[0];
  const bool prox = h->desc.hp == BETTY_HP_PROXIMAL;
  const float* dl = diag_log(h, lambda);
  make_weight_operands(h, os, w);
  forward_backward(h, os, SIDE_TRAIN, w, wnet_theta(h, lambda));
  if (loss_or_null) {                      // the cost at the w before the step
    float* add = nullptr;
    if (dl) {
      const float* x = w;
      if (prox) {
        launch_diff(h->ctx, w, lambda, h->f(h->vec_g), h->d);
        x = h->f(h->vec_g);
      }
      add = h->f(h->scalars) + 8;
      launch_l2_cost(h->ctx, dl, x, h->d, h->at<double>(h->partials), add);
    }
    launch_weighted_loss_sum(h->ctx, h->f(os.side[0].s), h->f(os.side[0].ell), os.side[0].B, add, loss_or_null);
  }
  // momentum and parameters are updated in the epilogue of the weight-gradient launch
  // (the proximal term pulls towards the anchor: the epilogue subtracts it from w in that term)
  WgradSink k{EPI_WGRAD_SGD, nullptr, dl, prox ? lambda : nullptr, momentum, w, lr, false};
  k.beta = mu; k.gamma = weight_decay;
  wgrad_batch(h, os, 0, false, k);
  return finish(h);
}

betty_status betty_upper_adam_step(betty_handle h, float* lambda, const float* dlambda, float* m, float* v, int t,
                                   float lr, float beta1, float beta2, float eps) {
  if (!h) return BETTY_ENULL;
  CHECK(check_vec(h, lambda, "lambda")); CHECK(check_vec(h, dlambda, "dlambda")); CHECK(check_vec(h, m, "m"));
  CHECK(check_vec(h, v, "v"));
  if (t < 1) return fail(h, BETTY_EINVAL, "t must be >= 1 (got %d)", t);
  if (!std::isfinite(lr) || !(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f) || !(eps >= 0.f))
    return fail(h, BETTY_EINVAL, "need finite lr, 0 <= beta1, beta2 < 1, eps >= 0");
  const size_t nb = h->n_hyper * 4;
  if (overlaps(lambda, nb, dlambda, nb) || overlaps(lambda, nb, m, nb) || overlaps(lambda, nb, v, nb) ||
      overlaps(m, nb, v, nb) || overlaps(m, nb, dlambda, nb) || overlaps(v, nb, dlambda, nb))
    return fail(h, BETTY_EINVAL, "lambda, dlambda, m and v must not overlap");
  const float bias1 = 1.f - std::pow(beta1, (float)t), bias2 = 1.f - std::pow(beta2, (float)t);
  launch_adam(h->ctx, lambda, dlambda, m, v, lr, beta1, beta2, eps, bias1, bias2, h->n_hyper);
  return finish(h);
}

betty_status betty_apply_label_noise(betty_handle h, const int32_t* y, const uint32_t* words, const int32_t* alt,
                                     double p, int n, int32_t* y_out, uint8_t* mask_or_null) {
  if (!h) return BETTY_ENULL;
  if (n < 0) return fail(h, BETTY_EINVAL, "n must be >= 0");
  if (!(p >= 0.0 && p <= 1.0)) return fail(h, BETTY_EINVAL, "p must lie in [0, 1]");
  if (n == 0) return BETTY_OK;
  CHECK(check_vec(h, y, "y")); CHECK(check_vec(h, words, "words")); CHECK(check_vec(h, alt, "alt"));
  CHECK(check_vec(h, y_out, "y_out"));
  unsigned long long T = (unsigned long long)std::floor(p * 4294967296.0);
  if (T > 4294967296ULL) T = 4294967296ULL;
  launch_label_noise(h->ctx, y, words, alt, T, n, y_out, mask_or_null);
  return finish(h);
}

betty_status betty_profile_enable(betty_handle h, int on) {
  if (!h) return BETTY_ENULL;
  for (auto& r : h->ctx.recs) { (void)hipEventDestroy(r.e0); (void)hipEventDestroy(r.e1); }
  h->ctx.recs.clear();
  h->ctx.profiling = on != 0;
  return BETTY_OK;
}

int betty_profile_collect(betty_handle h) {
  if (!h) return 0;
  if (hipStreamSynchronize(h->ctx.stream) != hipSuccess) return 0;
  for (auto& r : h->ctx.recs)
    if (r.ms < 0.f && hipEventElapsedTime(&r.ms, r.e0, r.e1) != hipSuccess) r.ms = -1.f;
  return (int)h->ctx.recs.size();
}

betty_status betty_profile_get(betty_handle h, int i, betty_profile_rec* out) {
  if (!h || !out) return BETTY_ENULL;
  if (i < 0 || i >= (int)h->ctx.recs.size()) return fail(h, BETTY_EINVAL, "profile record %d out of range", i);
  const ProfRec& r = h->ctx.recs[i];
  out->kind = r.kind; out->ms = r.ms; out->flops = r.flops; out->bytes = r.bytes;
  return BETTY_OK;
}

}  // extern "C"

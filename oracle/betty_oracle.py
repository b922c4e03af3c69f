"""fp64 CPU oracle for the bilevel hypergradient path.  TEST INFRASTRUCTURE ONLY.

This file is the slow, plain reference that the GPU library is checked
against.  Nothing in the product path may import it; only the tests, the
smoke check and the benchmark's CPU-baseline leg do.  It shares no code with
the HIP implementation.

What it computes (paper Sec. 3.2, "Gradient Calculation with Best-Response
Jacobians", Eq. 3-4, specialised to two levels through Eq. 1): for a lower
problem  w*(lambda) = argmin_w L_L(w, lambda)  and an upper cost L_U(w*),

    dL_U/dlambda = dL_U/dlambda|direct  -  (d^2 L_L / dlambda dw) H^{-1} grad_w L_U,
    H = d^2 L_L / dw dw,

evaluated right-to-left with vectors only (Sec. 3.2: the rightmost factor is
a vector, so every step is a matrix-vector product and no Jacobian is ever
formed).  The paper names the approximate-implicit-differentiation variants
(AID with a Neumann series, AID with finite differences; Sec. 3.2 last
paragraph) without printing their formulas, so the recurrences below are this
project's stated reading of them:

  Neumann(K, alpha):  v_0 = p_0 = g;  v_k = v_{k-1} - alpha H v_{k-1};
                      p_k = p_{k-1} + v_k;  q = alpha p_K   (K products, K+1 terms)
  CG(K):              K conjugate-gradient iterations on H q = g from q = 0
  FD(K, alpha, s):    the same with  H v := [grad L_L(w + e v) - grad L_L(w - e v)] / (2 e),
                      e = s / ||v||_2, and the mixed term by the same central
                      difference of grad_lambda L_L along q.  K = 0 is the
                      paper's AID-FD (q = alpha g, first-order gradients only;
                      Sec. 5.4 and App. D.1).

Lower costs:
  "l2":       L_L = sum_i s_i l_i(w) + sum_j exp(lambda_j) w_j^2,  s_i = 1/B
              (per-parameter weight decay, App. D.1; lambda has the layout of w)
  "reweight": L_L = (1/B) sum_i R(l_i; theta) l_i(w), R a 1-H-1 MLP (ReLU hidden,
              sigmoid out) fed the *value* of l_i, i.e. treated as constant
              when differentiating in w (App. B Listing 3: the reweighting
              input is detached; App. C: 1-100-1 weight net)
  "proximal": L_L = (1/B) sum_i l_i(w) + sum_j rho_j (w_j - a_j)^2, the finetuning level of the
              three-level program of Sec. 4.3: its "hyperparameter" a is the optimum of the level
              below it in the chain (the pretraining weights).  rho_j = rho on every parameter,
              or 0 on the last layer's when prox_skip_last (App. B Listing 5 leaves the
              classifier head out of the proximal term).
Upper cost:   L_U = mean_i l_i(w) on the validation batch (Listing 3, level 2).

Three levels (Sec. 3.1 Eq. 2, Sec. 4.3): with theta -> w*(theta) -> v*(w*) -> L_U(v*) the
single path gives  dL_U/dtheta = (dw*/dtheta) (dv*/dw*) grad_v L_U, evaluated from the right:
each factor applied to a vector is the same base operation (Eq. 3-4) on one of the two lower
problems, `best_response_neumann`.

Parity status of each function against pins other than itself is listed in
tests/test_oracle_pins.py; no function here is "parity unpinned".
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np
from scipy.special import erf

F64 = np.float64


@dataclass
class Problem:
    dims: tuple
    act: str                 # "none" | "relu" | "gelu"
    loss: str                # "mse" | "ce"
    hp: str                  # "l2" | "reweight" | "proximal"
    has_bias: bool
    X_tr: np.ndarray
    X_val: np.ndarray
    y_tr: Optional[np.ndarray] = None    # integer labels (ce)
    y_val: Optional[np.ndarray] = None
    t_tr: Optional[np.ndarray] = None    # real targets (mse), (B, n_L)
    t_val: Optional[np.ndarray] = None
    wnet_hidden: int = 100
    prox_rho: float = 0.0                # "proximal": coefficient of ||w - a||^2
    prox_skip_last: bool = False         # "proximal": no proximal term on the last layer

    def __post_init__(self):
        self.X_tr = np.asarray(self.X_tr, dtype=F64)
        self.X_val = np.asarray(self.X_val, dtype=F64)
        if self.t_tr is not None:
            self.t_tr = np.asarray(self.t_tr, dtype=F64)
        if self.t_val is not None:
            self.t_val = np.asarray(self.t_val, dtype=F64)

    @property
    def n_layers(self):
        return len(self.dims) - 1

    @property
    def d(self):
        return sum(self.dims[l] * self.dims[l + 1] + (self.dims[l + 1] if self.has_bias else 0)
                   for l in range(self.n_layers))

    def batch(self, which):
        if which == "train":
            return self.X_tr, (self.y_tr if self.loss == "ce" else self.t_tr)
        return self.X_val, (self.y_val if self.loss == "ce" else self.t_val)


# ----------------------------------------------------------------------------
# parameter layout: one flat vector [W_1 (n_0 x n_1, row-major), b_1, ..., W_L, b_L]
# ----------------------------------------------------------------------------

def split_params(prob: Problem, w):
    """Views (W_l, b_l) of a flat vector; b_l is None without biases."""
    w = np.asarray(w, dtype=F64)
    assert w.shape == (prob.d,)
    out, o = [], 0
    for l in range(prob.n_layers):
        n_in, n_out = prob.dims[l], prob.dims[l + 1]
        W = w[o:o + n_in * n_out].reshape(n_in, n_out)
        o += n_in * n_out
        b = None
        if prob.has_bias:
            b = w[o:o + n_out]
            o += n_out
        out.append((W, b))
    return out


def join_params(prob: Problem, parts):
    flat = []
    for (GW, Gb) in parts:
        flat.append(np.asarray(GW, dtype=F64).ravel())
        if prob.has_bias:
            flat.append(np.asarray(Gb, dtype=F64).ravel())
    return np.concatenate(flat)


# ----------------------------------------------------------------------------
# activations (exact erf GELU; ReLU derivative at 0 is 0)
# ----------------------------------------------------------------------------

def activation(z, act):
    """phi(z), phi'(z), phi''(z)."""
    if act == "none":
        return z, np.ones_like(z), np.zeros_like(z)
    if act == "relu":
        pos = (z > 0).astype(F64)
        return z * pos, pos, np.zeros_like(z)
    if act == "gelu":
        Phi = 0.5 * (1.0 + erf(z / np.sqrt(2.0)))
        pdf = np.exp(-0.5 * z * z) / np.sqrt(2.0 * np.pi)
        return z * Phi, Phi + z * pdf, pdf * (2.0 - z * z)
    raise ValueError(act)


# ----------------------------------------------------------------------------
# forward pass and per-sample losses
# ----------------------------------------------------------------------------

def forward(prob: Problem, w, X):
    """a_0 = X; z_l = a_{l-1} W_l + b_l; a_l = phi(z_l) for l < L.  Returns (a list, z list)."""
    params = split_params(prob, w)
    a, zs = [np.asarray(X, dtype=F64)], []
    for l, (W, b) in enumerate(params):
        z = a[-1] @ W
        if b is not None:
            z = z + b
        zs.append(z)
        if l < prob.n_layers - 1:
            a.append(activation(z, prob.act)[0])
    return a, zs


def sample_losses(prob: Problem, zL, target):
    """Per-sample loss l_i and its derivative in the logits, dl_i/dz_L (B x C)."""
    if prob.loss == "ce":
        # a label outside [0, C) is read as the nearest class (the library's stated behaviour)
        y = np.clip(np.asarray(target).astype(np.int64), 0, zL.shape[1] - 1)
        m = zL.max(axis=1, keepdims=True)
        e = np.exp(zL - m)
        Z = e.sum(axis=1, keepdims=True)
        p = e / Z
        idx = np.arange(zL.shape[0])
        ell = (np.log(Z[:, 0]) + m[:, 0]) - zL[idx, y]
        dz = p.copy()
        dz[idx, y] -= 1.0
        return ell, dz
    if prob.loss == "mse":
        r = zL - target
        return (r * r).sum(axis=1), 2.0 * r
    raise ValueError(prob.loss)


def loss_hessian_vec(prob: Problem, zL, Rz):
    """(d^2 l_i / dz_L^2) applied to a logit direction Rz, per sample."""
    if prob.loss == "ce":
        m = zL.max(axis=1, keepdims=True)
        e = np.exp(zL - m)
        p = e / e.sum(axis=1, keepdims=True)
        return p * Rz - p * (p * Rz).sum(axis=1, keepdims=True)
    return 2.0 * Rz


# ----------------------------------------------------------------------------
# weight net R(l; theta) = sigmoid(u2 . relu(u1 l + b1) + b2)
# ----------------------------------------------------------------------------

def split_theta(theta, hidden):
    theta = np.asarray(theta, dtype=F64)
    assert theta.shape == (3 * hidden + 1,)
    return theta[:hidden], theta[hidden:2 * hidden], theta[2 * hidden:3 * hidden], theta[3 * hidden]


def weight_net(ell, theta, hidden):
    """Per-sample weight omega_i = R(l_i; theta)."""
    u1, b1, u2, b2 = split_theta(theta, hidden)
    pre = np.outer(ell, u1) + b1
    h = np.maximum(pre, 0.0)
    s = h @ u2 + b2
    return 1.0 / (1.0 + np.exp(-s))


def weight_net_theta_vjp(ell, theta, hidden, c):
    """sum_i c_i * dR(l_i; theta)/dtheta, by backpropagation through the 1-H-1 net."""
    u1, b1, u2, b2 = split_theta(theta, hidden)
    pre = np.outer(ell, u1) + b1
    mask = (pre > 0).astype(F64)
    h = pre * mask
    s = h @ u2 + b2
    om = 1.0 / (1.0 + np.exp(-s))
    ds = c * om * (1.0 - om)                  # (B,)
    g_u2 = h.T @ ds
    g_b2 = ds.sum()
    dpre = np.outer(ds, u2) * mask            # (B, H)
    g_u1 = dpre.T @ ell
    g_b1 = dpre.sum(axis=0)
    return np.concatenate([g_u1, g_b1, g_u2, [g_b2]])


def sample_scales(prob: Problem, ell, lam, lower: bool):
    """s_i such that the data part of the cost is sum_i s_i l_i (weights held constant)."""
    B = ell.shape[0]
    if lower and prob.hp == "reweight":
        return weight_net(ell, lam, prob.wnet_hidden) / B
    return np.full(B, 1.0 / B)


# ----------------------------------------------------------------------------
# first-order gradients
# ----------------------------------------------------------------------------

def backprop(prob: Problem, w, a, zs, deltaL):
    """Gradient of sum_i <deltaL_i, z_L,i>-style output sensitivities w.r.t. the flat w."""
    params = split_params(prob, w)
    grads = [None] * prob.n_layers
    delta = deltaL
    for l in range(prob.n_layers - 1, -1, -1):
        W, b = params[l]
        grads[l] = (a[l].T @ delta, delta.sum(axis=0))
        if l > 0:
            delta = (delta @ W.T) * activation(zs[l - 1], prob.act)[1]
    return join_params(prob, grads)


def data_cost_and_grad(prob: Problem, w, lam, which, ell_frozen=None):
    lower = which == "train"
    X, target = prob.batch(which)
    a, zs = forward(prob, w, X)
    ell, dz = sample_losses(prob, zs[-1], target)
    s = sample_scales(prob, ell if ell_frozen is None else ell_frozen, lam, lower)
    cost = float((s * ell).sum())
    grad = backprop(prob, w, a, zs, s[:, None] * dz)
    return cost, grad


def prox_coeff(prob: Problem):
    """rho_j of the proximal cost, one entry per parameter (weights and biases alike)."""
    c = np.full(prob.d, float(prob.prox_rho), dtype=F64)
    if prob.prox_skip_last:
        n_in, n_out = prob.dims[-2], prob.dims[-1]
        c[prob.d - (n_in * n_out + (n_out if prob.has_bias else 0)):] = 0.0
    return c


def lower_cost(prob: Problem, w, lam):
    """L_L(w, lambda): the training cost whose argmin defines w*(lambda) (Eq. 4)."""
    w = np.asarray(w, dtype=F64)
    X, target = prob.batch("train")
    _, zs = forward(prob, w, X)
    ell, _ = sample_losses(prob, zs[-1], target)
    s = sample_scales(prob, ell, lam, True)
    cost = float((s * ell).sum())
    if prob.hp == "l2":
        cost += float((np.exp(np.asarray(lam, dtype=F64)) * w * w).sum())
    if prob.hp == "proximal":
        diff = w - np.asarray(lam, dtype=F64)
        cost += float((prox_coeff(prob) * diff * diff).sum())
    return cost


def lower_grad(prob: Problem, w, lam, ell_frozen=None):
    """(L_L, grad_w L_L) on the train batch; the reweighting weights are constants in w.

    ell_frozen, if given, is the per-sample loss fed to the weight net instead of l_i(w)
    (used by the finite-difference products, which must keep the weights fixed)."""
    w = np.asarray(w, dtype=F64)
    cost, grad = data_cost_and_grad(prob, w, lam, "train", ell_frozen)
    if prob.hp == "l2":
        e = np.exp(np.asarray(lam, dtype=F64))
        cost += float((e * w * w).sum())
        grad = grad + 2.0 * e * w
    if prob.hp == "proximal":
        c = prox_coeff(prob)
        diff = w - np.asarray(lam, dtype=F64)
        cost += float((c * diff * diff).sum())
        grad = grad + 2.0 * c * diff
    return cost, grad


def upper_grad(prob: Problem, w):
    """(L_U, grad_w L_U): plain mean loss on the validation batch (the direct gradient of Eq. 1)."""
    return data_cost_and_grad(prob, np.asarray(w, dtype=F64), None, "val")


# ----------------------------------------------------------------------------
# Hessian-vector product by forward-over-reverse differentiation
# ----------------------------------------------------------------------------

def r_forward(prob: Problem, w, v, a, zs):
    """Directional derivative of every pre-activation along the parameter direction v."""
    params = split_params(prob, w)
    dirs = split_params(prob, v)
    Ra = np.zeros_like(a[0])
    Rzs, Ras = [], [Ra]
    for l in range(prob.n_layers):
        W, _ = params[l]
        V, c = dirs[l]
        Rz = Ra @ W + a[l] @ V
        if c is not None:
            Rz = Rz + c
        Rzs.append(Rz)
        if l < prob.n_layers - 1:
            Ra = activation(zs[l], prob.act)[1] * Rz
            Ras.append(Ra)
    return Ras, Rzs


def hvp(prob: Problem, w, lam, v):
    """H v with H = d^2 L_L / dw dw at (w, lambda), without forming H."""
    w = np.asarray(w, dtype=F64)
    v = np.asarray(v, dtype=F64)
    X, target = prob.batch("train")
    params = split_params(prob, w)
    dirs = split_params(prob, v)
    a, zs = forward(prob, w, X)
    ell, dz = sample_losses(prob, zs[-1], target)
    s = sample_scales(prob, ell, lam, True)
    Ras, Rzs = r_forward(prob, w, v, a, zs)

    delta = s[:, None] * dz
    Rdelta = s[:, None] * loss_hessian_vec(prob, zs[-1], Rzs[-1])
    out = [None] * prob.n_layers
    for l in range(prob.n_layers - 1, -1, -1):
        W, _ = params[l]
        V, _ = dirs[l]
        out[l] = (Ras[l].T @ delta + a[l].T @ Rdelta, Rdelta.sum(axis=0))
        if l > 0:
            _, d1, d2 = activation(zs[l - 1], prob.act)
            back = delta @ W.T
            Rdelta = (Rdelta @ W.T + delta @ V.T) * d1 + back * d2 * Rzs[l - 1]
            delta = back * d1
    Hv = join_params(prob, out)
    if prob.hp == "l2":
        Hv = Hv + 2.0 * np.exp(np.asarray(lam, dtype=F64)) * v
    if prob.hp == "proximal":
        Hv = Hv + 2.0 * prox_coeff(prob) * v
    return Hv


def train_losses(prob: Problem, w):
    """l_i(w) on the train batch."""
    X, target = prob.batch("train")
    _, zs = forward(prob, np.asarray(w, dtype=F64), X)
    return sample_losses(prob, zs[-1], target)[0]


def hvp_fd(prob: Problem, w, lam, v, eps_scale):
    """Central finite difference of the lower gradient along v, step eps_scale/||v||_2.

    For the reweighting cost the sample weights stay those of the unperturbed w (the cost treats
    them as constants in w), so that the difference approximates the same H as `hvp`."""
    w = np.asarray(w, dtype=F64)
    v = np.asarray(v, dtype=F64)
    nrm = float(np.sqrt((v * v).sum()))
    if nrm == 0.0:
        return np.zeros_like(v)
    eps = eps_scale / nrm
    frozen = train_losses(prob, w) if prob.hp == "reweight" else None
    gp = lower_grad(prob, w + eps * v, lam, frozen)[1]
    gm = lower_grad(prob, w - eps * v, lam, frozen)[1]
    return (gp - gm) / (2.0 * eps)


# ----------------------------------------------------------------------------
# mixed second-order vector-Jacobian product into lambda
# ----------------------------------------------------------------------------

def per_sample_directional(prob: Problem, w, q):
    """c_i = <grad_w l_i(w), q> for every train sample, and l_i."""
    w = np.asarray(w, dtype=F64)
    X, target = prob.batch("train")
    a, zs = forward(prob, w, X)
    ell, dz = sample_losses(prob, zs[-1], target)
    _, Rzs = r_forward(prob, w, np.asarray(q, dtype=F64), a, zs)
    return (dz * Rzs[-1]).sum(axis=1), ell


def mixed_vjp(prob: Problem, w, lam, q):
    """- grad_lambda < grad_w L_L(w, lambda), q >  with q held constant."""
    w = np.asarray(w, dtype=F64)
    q = np.asarray(q, dtype=F64)
    lam = np.asarray(lam, dtype=F64)
    if prob.hp == "l2":
        return -2.0 * np.exp(lam) * w * q
    if prob.hp == "proximal":
        # d/da of <2 rho (w - a), q> is -2 rho q
        return 2.0 * prox_coeff(prob) * q
    c, ell = per_sample_directional(prob, w, q)
    B = ell.shape[0]
    return -weight_net_theta_vjp(ell, lam, prob.wnet_hidden, c) / B


def lambda_grad(prob: Problem, w, lam, ell_frozen=None):
    """grad_lambda L_L(w, lambda) (first order; used by the finite-difference mixed term)."""
    w = np.asarray(w, dtype=F64)
    lam = np.asarray(lam, dtype=F64)
    if prob.hp == "l2":
        return np.exp(lam) * w * w
    if prob.hp == "proximal":
        return -2.0 * prox_coeff(prob) * (w - lam)
    X, target = prob.batch("train")
    _, zs = forward(prob, w, X)
    ell, _ = sample_losses(prob, zs[-1], target)
    src = ell if ell_frozen is None else ell_frozen
    return weight_net_theta_vjp(src, lam, prob.wnet_hidden, ell) / ell.shape[0]


def mixed_vjp_fd(prob: Problem, w, lam, q, eps_scale):
    """Central difference of grad_lambda L_L along q (negated), step eps_scale/||q||_2.

    For the reweighting cost the weight-net *input* is frozen at l_i(w) during the
    two perturbed evaluations, so that the difference converges to the analytic
    mixed term of the detached cost.
    """
    w = np.asarray(w, dtype=F64)
    q = np.asarray(q, dtype=F64)
    nrm = float(np.sqrt((q * q).sum()))
    if nrm == 0.0:
        return np.zeros_like(np.asarray(lam, dtype=F64))
    eps = eps_scale / nrm
    frozen = None
    if prob.hp == "reweight":
        X, target = prob.batch("train")
        _, zs = forward(prob, w, X)
        frozen, _ = sample_losses(prob, zs[-1], target)
    gp = lambda_grad(prob, w + eps * q, lam, frozen)
    gm = lambda_grad(prob, w - eps * q, lam, frozen)
    return -(gp - gm) / (2.0 * eps)


# ----------------------------------------------------------------------------
# hypergradients
# ----------------------------------------------------------------------------

def neumann_q(prob: Problem, w, lam, g, K, alpha, product):
    v = np.array(g, dtype=F64)
    p = v.copy()
    for _ in range(K):
        v = v - alpha * product(v)
        p = p + v
    return alpha * p


def hypergrad_neumann(prob: Problem, w, lam, K, alpha):
    """dL_U/dlambda by the K-step Neumann approximation of H^{-1} g and the mixed VJP."""
    g = upper_grad(prob, w)[1]
    q = neumann_q(prob, w, lam, g, K, alpha, lambda v: hvp(prob, w, lam, v))
    return mixed_vjp(prob, w, lam, q)


def best_response_neumann(prob: Problem, w, lam, u, K, alpha):
    """The base operation of Sec. 3.2 (Eq. 3-4): (dw*/dlambda) applied to a vector u of the size
    of w, i.e. -(d^2 L_L/dlambda dw) H^{-1} u with the K-step Neumann approximation of H^{-1} u.
    `hypergrad_neumann` is this with u = grad_w L_U."""
    q = neumann_q(prob, w, lam, np.asarray(u, dtype=F64), K, alpha, lambda v: hvp(prob, w, lam, v))
    return mixed_vjp(prob, w, lam, q)


def hypergrad_chain3(pre: Problem, ft: Problem, w, theta, v, K_pre, alpha_pre, K_ft, alpha_ft):
    """dL_U/dtheta of the three-level chain theta -> w*(theta) -> v*(w*) -> L_U(v*) (Eq. 2 with
    its single path; Sec. 4.3), from the right:  u = (dv*/dw) grad_v L_U  on the finetuning
    problem `ft` (proximal cost anchored at w, parameters v, upper cost on ft's validation batch),
    then (dw*/dtheta) u on the pretraining problem `pre` (parameters w, hyperparameters theta)."""
    assert ft.hp == "proximal" and ft.d == pre.d
    g = upper_grad(ft, v)[1]
    u = best_response_neumann(ft, v, w, g, K_ft, alpha_ft)
    return best_response_neumann(pre, w, theta, u, K_pre, alpha_pre)


def hypergrad_fd(prob: Problem, w, lam, K, alpha, eps_scale):
    """Same, with every second-order product replaced by central differences."""
    g = upper_grad(prob, w)[1]
    q = neumann_q(prob, w, lam, g, K, alpha, lambda v: hvp_fd(prob, w, lam, v, eps_scale))
    return mixed_vjp_fd(prob, w, lam, q, eps_scale)


def cg_q(g, K, product):
    """K conjugate-gradient iterations on H q = g from q = 0 (AID-CG, Sec. 3.2)."""
    g = np.asarray(g, dtype=F64)
    q = np.zeros_like(g)
    r = g.copy()
    d = r.copy()
    rs = float(r @ r)
    for _ in range(K):
        if rs == 0.0:
            break
        Hd = product(d)
        dHd = float(d @ Hd)
        if dHd == 0.0:
            break
        a = rs / dHd
        q = q + a * d
        r = r - a * Hd
        rs_new = float(r @ r)
        d = r + (rs_new / rs) * d
        rs = rs_new
    return q


def hypergrad_cg(prob: Problem, w, lam, K):
    """dL_U/dlambda with H^{-1} g approximated by K conjugate-gradient iterations."""
    g = upper_grad(prob, w)[1]
    q = cg_q(g, K, lambda v: hvp(prob, w, lam, v))
    return mixed_vjp(prob, w, lam, q)


# ----------------------------------------------------------------------------
# the optimisation steps around the hypergradient (Sec. 3.3; optimisers as in App. C)
# ----------------------------------------------------------------------------

def lower_sgd_step(prob: Problem, w, lam, mom, lr, mu, weight_decay=0.0):
    """One step of the lower problem: SGD with momentum on L_L(w, lambda) (+ plain weight decay).

    g = grad_w L_L + weight_decay * w;  mom <- mu * mom + g;  w <- w - lr * mom."""
    w = np.asarray(w, dtype=F64)
    g = lower_grad(prob, w, lam)[1] + weight_decay * w
    mom = mu * np.asarray(mom, dtype=F64) + g
    return w - lr * mom, mom


def adam_step(x, grad, m, v, t, lr, beta1=0.9, beta2=0.999, eps=1e-8):
    """One Adam step (step counter t >= 1) on the upper parameters given their (hyper)gradient."""
    x = np.asarray(x, dtype=F64)
    grad = np.asarray(grad, dtype=F64)
    m = beta1 * np.asarray(m, dtype=F64) + (1.0 - beta1) * grad
    v = beta2 * np.asarray(v, dtype=F64) + (1.0 - beta2) * grad * grad
    mhat = m / (1.0 - beta1 ** t)
    vhat = v / (1.0 - beta2 ** t)
    return x - lr * mhat / (np.sqrt(vhat) + eps), m, v


def bilevel_step(prob: Problem, w, mom, lam, am, av, t, unroll, lr_w, mu, K, alpha, lr_lam,
                 weight_decay=0.0):
    """`unroll` lower SGD steps, then one Adam step on lambda along the Neumann hypergradient
    evaluated at the unrolled w (Sec. 3.3: the lower problem calls the upper one after its
    unrolling steps; the best-response Jacobian is taken at the unrolled weights)."""
    for _ in range(unroll):
        w, mom = lower_sgd_step(prob, w, lam, mom, lr_w, mu, weight_decay)
    dlam = hypergrad_neumann(prob, w, lam, K, alpha)
    lam, am, av = adam_step(lam, dlam, am, av, t, lr_lam)
    return w, mom, lam, am, av


# ----------------------------------------------------------------------------
# exact ridge lower solve (used to place w at w* for the ridge workload) and label noise
# ----------------------------------------------------------------------------

def ridge_solve(X, t, lam):
    """argmin_w ||X w - t||^2 / n + sum_j exp(lambda_j) w_j^2 by the normal equations."""
    X = np.asarray(X, dtype=F64)
    t = np.asarray(t, dtype=F64).reshape(-1)
    n = X.shape[0]
    A = X.T @ X / n + np.diag(np.exp(np.asarray(lam, dtype=F64)))
    return np.linalg.solve(A, X.T @ t / n)


def apply_label_noise(y, words, alt, p):
    """y'_i = alt_i if words_i < floor(p 2^32) else y_i, with the mask.  Pure integer work."""
    T = min(int(np.floor(p * 4294967296.0)), 4294967296)
    out = np.empty(len(y), dtype=np.int32)
    mask = np.empty(len(y), dtype=np.uint8)
    for i in range(len(y)):
        hit = int(words[i]) < T
        mask[i] = 1 if hit else 0
        out[i] = int(alt[i]) if hit else int(y[i])
    return out, mask

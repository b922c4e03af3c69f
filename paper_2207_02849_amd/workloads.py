"""Seeded synthetic inputs for the bilevel hypergradient workloads.

This module only *draws data*: design matrices, labels, label-noise words,
initial parameters and hyperparameters.  It contains none of the method's
arithmetic (no losses, gradients, Hessian products or solves) so that both
the CPU oracle's tests and the GPU path can be fed from it without sharing
any computation.

The workloads stand in for the paper's experiments (Sec. 5.1 data
reweighting with a 1-100-1 Meta-Weight-Net, App. C "Experiment Details";
App. D.1 per-parameter weight-decay hyperparameter optimisation), whose
datasets are not available here: Gaussian-mixture classification data and a
Gaussian linear-regression problem of the stated shapes.

Every array is drawn from numpy's Philox counter-based generator keyed by
the seed, in fp64, in a fixed order, and then cast.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Optional

import numpy as np


@dataclass
class Workload:
    """Plain container; fields mirror the C-ABI problem description."""
    name: str
    dims: tuple            # (n_0, ..., n_L): L linear layers
    act: str               # "none" | "relu" | "gelu"
    loss: str              # "mse" | "ce"
    hp: str                # "l2" (lambda has length d) | "reweight" (1-H-1 weight net) |
                           # "proximal" (lambda = anchor parameters, length d)
    prec: str              # "fp32" | "bf16"
    has_bias: bool
    K: int
    alpha: float
    eps_scale: float
    X_tr: np.ndarray       # (B_tr, n_0) float32
    X_val: np.ndarray      # (B_val, n_0) float32
    y_tr: Optional[np.ndarray] = None     # int32 labels (ce); None when they are to be derived from the
                                          # label-noise ingredients below (each consumer applies the rule itself)
    y_val: Optional[np.ndarray] = None
    t_tr: Optional[np.ndarray] = None     # float32 targets (mse), (B, n_L)
    t_val: Optional[np.ndarray] = None
    w: Optional[np.ndarray] = None        # float32 flat [W_1, b_1, ..., W_L, b_L]
    lam: Optional[np.ndarray] = None      # float32: length d (l2) or 3H+1 (reweight)
    wnet_hidden: int = 100
    # label-noise ingredients (reweighting workloads): the train labels follow from these
    y_clean: Optional[np.ndarray] = None  # int32
    noise_words: Optional[np.ndarray] = None   # uint32, one per train sample
    noise_alt: Optional[np.ndarray] = None     # int32 replacement class per sample
    noise_p: float = 0.0
    prox_rho: float = 0.0                 # "proximal": coefficient of the squared distance to the anchor
    prox_skip_last: bool = False          # "proximal": last layer left out of the proximal term
    extra: dict = field(default_factory=dict)

    @property
    def d(self) -> int:
        return n_params(self.dims, self.has_bias)


def n_params(dims, has_bias=True) -> int:
    return sum(dims[l] * dims[l + 1] + (dims[l + 1] if has_bias else 0)
               for l in range(len(dims) - 1))


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=int(seed)))


def _mixture(rng, n_classes, n_in, batches, sigma):
    """Gaussian mixture: class means ~ N(0, I), isotropic noise sigma."""
    means = rng.standard_normal((n_classes, n_in))
    out = []
    for b in batches:
        y = rng.integers(0, n_classes, size=b, dtype=np.int64)
        x = means[y] + sigma * rng.standard_normal((b, n_in))
        out.append((x.astype(np.float32), y.astype(np.int32)))
    return out


def _init_mlp(rng, dims, has_bias=True):
    """W_l ~ N(0, 1/n_{l-1}), b_l ~ 0.01 N(0,1), flat [W_1, b_1, ...]."""
    parts = []
    for l in range(len(dims) - 1):
        n_in, n_out = dims[l], dims[l + 1]
        parts.append((rng.standard_normal((n_in, n_out)) / math.sqrt(n_in)).ravel())
        if has_bias:
            parts.append(0.01 * rng.standard_normal(n_out))
    return np.concatenate(parts).astype(np.float32)


def _init_l2_lambda(rng, d):
    """log-decay hyperparameters around log(5e-4), jittered per parameter."""
    return (math.log(5e-4) + 0.1 * rng.standard_normal(d)).astype(np.float32)


def _init_wnet(rng, hidden):
    """theta = [u1(H), b1(H), u2(H), b2(1)] of the 1-H-1 weight net."""
    u1 = rng.uniform(-1.0, 1.0, hidden)
    b1 = rng.uniform(-1.0, 1.0, hidden)
    u2 = rng.uniform(-0.1, 0.1, hidden)
    b2 = np.zeros(1)
    return np.concatenate([u1, b1, u2, b2]).astype(np.float32)


def ridge(seed=0, n_tr=512, n_val=256, n_feat=64, K=20, alpha=0.05):
    """Ridge-regression bilevel problem (linear 64->1, no bias, MSE).

    The lower-level solution w* is *not* computed here (that is the method's
    arithmetic); `w` is left as None and `extra["w_true"]` holds the planted
    coefficients.
    """
    rng = _rng(seed)
    w_true = rng.standard_normal(n_feat)
    X_tr = rng.standard_normal((n_tr, n_feat))
    t_tr = X_tr @ w_true + 0.1 * rng.standard_normal(n_tr)
    X_val = rng.standard_normal((n_val, n_feat))
    t_val = X_val @ w_true + 0.1 * rng.standard_normal(n_val)
    lam = np.full(n_feat, math.log(0.1), dtype=np.float32)
    return Workload(
        name="ridge", dims=(n_feat, 1), act="none", loss="mse", hp="l2", prec="fp32",
        has_bias=False, K=K, alpha=alpha, eps_scale=0.01,
        X_tr=X_tr.astype(np.float32), X_val=X_val.astype(np.float32),
        t_tr=t_tr.astype(np.float32).reshape(-1, 1), t_val=t_val.astype(np.float32).reshape(-1, 1),
        w=None, lam=lam, extra={"w_true": w_true})


def l2_mlp(name, seed, dims, act, prec, batch_tr, batch_val, K, alpha,
           n_classes=10, sigma=2.0, eps_scale=0.01):
    """Per-parameter L2-decay hyperparameters on an MLP classifier."""
    rng = _rng(seed)
    (X_tr, y_tr), (X_val, y_val) = _mixture(rng, n_classes, dims[0], (batch_tr, batch_val), sigma)
    w = _init_mlp(rng, dims)
    lam = _init_l2_lambda(rng, w.size)
    return Workload(name=name, dims=tuple(dims), act=act, loss="ce", hp="l2", prec=prec,
                    has_bias=True, K=K, alpha=alpha, eps_scale=eps_scale,
                    X_tr=X_tr, X_val=X_val, y_tr=y_tr, y_val=y_val, w=w, lam=lam)


def reweight_mlp(name, seed, dims, act, prec, batch_tr, batch_val, K, alpha,
                 noise_p, n_classes=10, sigma=2.0, hidden=100):
    """Meta-Weight-Net style reweighting with uniform label noise on the train batch.

    Only the ingredients are drawn here: clean labels, one 32-bit word and one replacement
    class per train sample, and the noise probability.  Turning them into the noisy train labels
    is part of the method (the integer threshold rule), so `y_tr` stays None and every consumer
    applies its own implementation of the rule.
    """
    rng = _rng(seed)
    (X_tr, y_clean), (X_val, y_val) = _mixture(rng, n_classes, dims[0], (batch_tr, batch_val), sigma)
    words = rng.integers(0, 2 ** 32, size=batch_tr, dtype=np.uint64).astype(np.uint32)
    alt = rng.integers(0, n_classes, size=batch_tr, dtype=np.int64).astype(np.int32)
    w = _init_mlp(rng, dims)
    theta = _init_wnet(rng, hidden)
    return Workload(name=name, dims=tuple(dims), act=act, loss="ce", hp="reweight", prec=prec,
                    has_bias=True, K=K, alpha=alpha, eps_scale=0.01,
                    X_tr=X_tr, X_val=X_val, y_tr=None, y_val=y_val, w=w, lam=theta,
                    wnet_hidden=hidden, y_clean=y_clean, noise_words=words, noise_alt=alt,
                    noise_p=noise_p)


def config(index: int, seed: int = 0) -> Workload:
    """The five benchmark configurations (1-based): ridge, two small MLPs, the 5M-parameter L2-decay
    MLP the headline rate is quoted on, and the 121M-parameter reweighting MLP."""
    if index == 1:
        return ridge(seed)
    if index == 2:
        return l2_mlp("l2_mlp_784_256_10_relu_fp32", seed, (784, 256, 10), "relu", "fp32",
                      128, 128, K=5, alpha=0.01)
    if index == 3:
        return reweight_mlp("reweight_mlp_1024_512_512_10_relu_bf16", seed, (1024, 512, 512, 10),
                            "relu", "bf16", 256, 256, K=3, alpha=0.01, noise_p=0.4)
    if index == 4:
        return l2_mlp("l2_mlp_3072_1024x3_10_gelu_bf16", seed, (3072, 1024, 1024, 1024, 10),
                      "gelu", "bf16", 256, 256, K=5, alpha=0.01)
    if index == 5:
        dims = (4096,) * 8 + (1000,)
        return reweight_mlp("reweight_mlp_4096x8_1000_gelu_bf16", seed, dims, "gelu", "bf16",
                            512, 512, K=3, alpha=0.005, noise_p=0.3, n_classes=1000)
    raise ValueError("config index must be 1..5")


def tiny(kind="l2", act="gelu", seed=0, dims=(5, 4, 3, 3), batch=7, has_bias=True,
         loss="ce", noise_p=0.3, hidden=6, prec="fp32", prox_rho=0.05, prox_skip_last=False):
    """Small ragged problems for unit tests (odd sizes on purpose)."""
    rng = _rng(seed + 1000)
    C = dims[-1]
    if loss == "ce":
        (X_tr, y_tr), (X_val, y_val) = _mixture(rng, C, dims[0], (batch, batch + 2), 1.0)
        t_tr = t_val = None
    else:
        X_tr = rng.standard_normal((batch, dims[0])).astype(np.float32)
        X_val = rng.standard_normal((batch + 2, dims[0])).astype(np.float32)
        t_tr = rng.standard_normal((batch, C)).astype(np.float32)
        t_val = rng.standard_normal((batch + 2, C)).astype(np.float32)
        y_tr = y_val = None
    parts = []
    for l in range(len(dims) - 1):
        parts.append((rng.standard_normal((dims[l], dims[l + 1])) / math.sqrt(dims[l])).ravel())
        if has_bias:
            parts.append(0.1 * rng.standard_normal(dims[l + 1]))
    w = np.concatenate(parts).astype(np.float32)
    if kind == "l2":
        lam = (math.log(0.05) + 0.3 * rng.standard_normal(w.size)).astype(np.float32)
    elif kind == "proximal":
        lam = (w + 0.2 * rng.standard_normal(w.size)).astype(np.float32)     # the anchor
    else:
        lam = _init_wnet(rng, hidden)
    return Workload(name=f"tiny_{kind}_{act}_{loss}", dims=tuple(dims), act=act, loss=loss,
                    hp=kind, prec=prec, has_bias=has_bias, K=3, alpha=0.05, eps_scale=0.01,
                    X_tr=X_tr, X_val=X_val, y_tr=y_tr, y_val=y_val, t_tr=t_tr, t_val=t_val,
                    w=w, lam=lam, wnet_hidden=hidden, prox_rho=prox_rho,
                    prox_skip_last=prox_skip_last)


def chain3(seed=0, dims=(6, 5, 4), act="gelu", prec="fp32", batch=9, has_bias=True, hidden=6,
           noise_p=0.3, rho=0.05, skip_last=True, K=3, alpha=0.05, sigma=1.0, name="chain3"):
    """The two lower problems of the three-level program of Sec. 4.3 on one MLP architecture.

    Returns (pre, ft).  `pre` is a reweighting problem on "source-domain" data (its own mixture,
    label-noise ingredients, train labels left to the consumer); its parameters `pre.w` are the pretraining weights and `pre.lam` the weight-net
    parameters theta.  `ft` is the finetuning problem on "target-domain" data (the source class
    means shifted by a random offset), with the proximal cost anchored at the pretraining weights:
    `ft.lam` is `pre.w`, `ft.w` the finetuned parameters v; ft's validation batch carries the
    top-level cost.
    """
    rng = _rng(seed + 77000)
    C = dims[-1]
    means = rng.standard_normal((C, dims[0]))
    shift = 0.5 * rng.standard_normal((C, dims[0]))

    def draw(m, b):
        y = rng.integers(0, C, size=b, dtype=np.int64)
        x = m[y] + sigma * rng.standard_normal((b, dims[0]))
        return x.astype(np.float32), y.astype(np.int32)

    Xs, ys_clean = draw(means, batch)
    Xs_val, ys_val = draw(means, batch)               # unused by the chain; fills pre's validation slot
    Xt, yt = draw(means + shift, batch + 1)
    Xt_val, yt_val = draw(means + shift, batch + 3)
    words = rng.integers(0, 2 ** 32, size=batch, dtype=np.uint64).astype(np.uint32)
    alt = rng.integers(0, C, size=batch, dtype=np.int64).astype(np.int32)
    w = _init_mlp(rng, dims, has_bias)
    v = (w + 0.1 * _init_mlp(rng, dims, has_bias)).astype(np.float32)
    theta = _init_wnet(rng, hidden)
    pre = Workload(name=name + "_pretrain", dims=tuple(dims), act=act, loss="ce", hp="reweight", prec=prec,
                   has_bias=has_bias, K=K, alpha=alpha, eps_scale=0.01, X_tr=Xs, X_val=Xs_val, y_tr=None,
                   y_val=ys_val, w=w, lam=theta, wnet_hidden=hidden, y_clean=ys_clean, noise_words=words,
                   noise_alt=alt, noise_p=noise_p)
    ft = Workload(name=name + "_finetune", dims=tuple(dims), act=act, loss="ce", hp="proximal", prec=prec,
                  has_bias=has_bias, K=K, alpha=alpha, eps_scale=0.01, X_tr=Xt, X_val=Xt_val, y_tr=yt,
                  y_val=yt_val, w=v, lam=w.copy(), prox_rho=rho, prox_skip_last=skip_last)
    return pre, ft

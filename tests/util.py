"""Test helpers: build an oracle Problem from a seeded workload; error metric."""
import numpy as np

from oracle import betty_oracle as orc


def train_labels(wl):
    """The train labels of a workload: as drawn, or (reweighting workloads with label noise) made from
    the noise ingredients by the oracle's own statement of the integer rule."""
    if wl.y_tr is None and wl.y_clean is not None:
        return orc.apply_label_noise(wl.y_clean, wl.noise_words, wl.noise_alt, wl.noise_p)[0]
    return wl.y_tr


def oracle_problem(wl) -> "orc.Problem":
    return orc.Problem(dims=wl.dims, act=wl.act, loss=wl.loss, hp=wl.hp, has_bias=wl.has_bias,
                       X_tr=wl.X_tr, X_val=wl.X_val, y_tr=train_labels(wl), y_val=wl.y_val,
                       t_tr=wl.t_tr, t_val=wl.t_val, wnet_hidden=wl.wnet_hidden,
                       prox_rho=wl.prox_rho, prox_skip_last=wl.prox_skip_last)


def rel_l2(x, ref):
    x = np.asarray(x, dtype=np.float64).ravel()
    ref = np.asarray(ref, dtype=np.float64).ravel()
    den = np.linalg.norm(ref)
    if den == 0.0:
        return float(np.linalg.norm(x))
    return float(np.linalg.norm(x - ref) / den)


def param_slices(dims, has_bias=True):
    """(name, start, stop) of every weight matrix and bias vector inside the flat parameter layout."""
    out, o = [], 0
    for l in range(len(dims) - 1):
        n = dims[l] * dims[l + 1]
        out.append((f"W{l + 1}", o, o + n))
        o += n
        if has_bias:
            out.append((f"b{l + 1}", o, o + dims[l + 1]))
            o += dims[l + 1]
    return out


def worst_slice(x, ref, dims, has_bias=True):
    """Largest relative L2 error over the tensors of a parameter-shaped vector, with its name."""
    x = np.asarray(x, dtype=np.float64).ravel()
    ref = np.asarray(ref, dtype=np.float64).ravel()
    worst = (0.0, "")
    for name, a, b in param_slices(dims, has_bias):
        e = rel_l2(x[a:b], ref[a:b])
        if e > worst[0]:
            worst = (e, name)
    return worst


def spectral_alpha(prob, w, lam, iters=8, seed=0):
    """1 / |lambda|_max of the lower Hessian, by a few power iterations with the oracle's product:
    the step size at which alpha * H has unit norm, so that the H term of the series carries full weight."""
    v = np.random.default_rng(seed).standard_normal(prob.d)
    v /= np.linalg.norm(v)
    top = 1.0
    for _ in range(iters):
        Hv = orc.hvp(prob, w, lam, v)
        top = np.linalg.norm(Hv)
        v = Hv / top
    return 1.0 / top

"""Test helpers: build an oracle Problem from a seeded workload; error metric."""
import numpy as np

from oracle import betty_oracle as orc


def oracle_problem(wl) -> "orc.Problem":
    return orc.Problem(dims=wl.dims, act=wl.act, loss=wl.loss, hp=wl.hp, has_bias=wl.has_bias,
                       X_tr=wl.X_tr, X_val=wl.X_val, y_tr=wl.y_tr, y_val=wl.y_val,
                       t_tr=wl.t_tr, t_val=wl.t_val, wnet_hidden=wl.wnet_hidden,
                       prox_rho=wl.prox_rho, prox_skip_last=wl.prox_skip_last)


def rel_l2(x, ref):
    x = np.asarray(x, dtype=np.float64).ravel()
    ref = np.asarray(ref, dtype=np.float64).ravel()
    den = np.linalg.norm(ref)
    if den == 0.0:
        return float(np.linalg.norm(x))
    return float(np.linalg.norm(x - ref) / den)

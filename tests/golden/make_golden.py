"""Writes tests/golden/tiny_hypergradients.json from the fp64 oracle alone.

The paper prints no hypergradient value (its tables are accuracies, memory and wall time), so
there is no paper-quoted fixture to store.  This file freezes the oracle's own results on a few
seeded tiny problems instead: a regression guard for the oracle's arithmetic (a change to it must
be deliberate and regenerate this file) and a stored expectation for the GPU tests that does not
depend on the oracle code of the day.  Run from the repository root:

    python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from oracle import betty_oracle as orc                     # noqa: E402
from paper_2207_02849_amd import workloads as wk           # noqa: E402
from tests.util import oracle_problem                      # noqa: E402

CASES = [
    dict(kind="l2", act="gelu", loss="ce"),
    dict(kind="l2", act="gelu", loss="mse", dims=(4, 5, 2)),
    dict(kind="reweight", act="gelu", loss="ce"),
    dict(kind="proximal", act="gelu", loss="ce", prox_rho=0.3),
]


def compute(cfg):
    wl = wk.tiny(**cfg)
    prob = oracle_problem(wl)
    w, lam = wl.w.astype(np.float64), wl.lam.astype(np.float64)
    return {
        "cfg": {k: (list(v) if isinstance(v, tuple) else v) for k, v in cfg.items()},
        "K": wl.K, "alpha": wl.alpha, "eps_scale": wl.eps_scale,
        "neumann": orc.hypergrad_neumann(prob, w, lam, wl.K, wl.alpha).tolist(),
        "fd": orc.hypergrad_fd(prob, w, lam, wl.K, wl.alpha, wl.eps_scale).tolist(),
        "cg": orc.hypergrad_cg(prob, w, lam, 3).tolist(),
    }


def chain_case():
    pre_wl, ft_wl = wk.chain3(seed=3, act="gelu", skip_last=True)
    pre, ft = oracle_problem(pre_wl), oracle_problem(ft_wl)
    w, th, v = (x.astype(np.float64) for x in (pre_wl.w, pre_wl.lam, ft_wl.w))
    return {"seed": 3, "K_pre": 4, "alpha_pre": 0.06, "K_ft": 3, "alpha_ft": 0.09,
            "chain3": orc.hypergrad_chain3(pre, ft, w, th, v, 4, 0.06, 3, 0.09).tolist()}


def main():
    out = {"source": "oracle/betty_oracle.py (fp64), seeded inputs from paper_2207_02849_amd/workloads.py",
           "cases": [compute(c) for c in CASES], "chain3": chain_case()}
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_hypergradients.json")
    with open(path, "w") as f:
        json.dump(out, f, indent=1)
    print("wrote", path)


if __name__ == "__main__":
    main()

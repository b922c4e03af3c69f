"""Config 5 (8 x 4096-wide layers, 1000 classes, ~1.2e8 parameters): full-size parity.

The oracle needs on the order of a minute per hypergradient at this size, so the whole
comparison is one test."""
import numpy as np
import pytest
import torch

from oracle import betty_oracle as orc
from paper_2207_02849_amd import binding
from paper_2207_02849_amd import workloads as wk
from tests.util import oracle_problem, rel_l2, worst_slice

pytestmark = pytest.mark.gpu


def test_config5_reweight_gelu_bf16():
    wl = wk.config(5)
    assert wl.d == 121566184
    prob = oracle_problem(wl)
    b = binding.from_workload(wl)
    w, lam = torch.as_tensor(wl.w).cuda(), torch.as_tensor(wl.lam).cuda()
    print("config5: GPU neumann", flush=True)
    hg = b.betty_hypergrad_neumann(w, lam, wl.K, wl.alpha)
    torch.cuda.synchronize()
    got = hg.cpu().numpy()
    print("config5: GPU hvp", flush=True)
    v = np.random.default_rng(5).standard_normal(wl.d).astype(np.float32)
    Hv = b.betty_hvp(w, lam, torch.as_tensor(v).cuda())
    torch.cuda.synchronize()
    Hv_host = Hv.cpu().numpy()
    del Hv
    print("config5: GPU lower gradient", flush=True)
    g = b.betty_lower_grad(w, lam)
    torch.cuda.synchronize()
    g_host = g.cpu().numpy()
    del g
    b.close()
    print("config5: oracle hvp", flush=True)
    ref_Hv = orc.hvp(prob, wl.w, wl.lam, v)
    e_hvp = rel_l2(Hv_host, ref_Hv)
    # every weight matrix and every bias on its own as well: the layers take different paths (full
    # tiles, the ragged 1000-column layer, the bias rows), and one wrong small slice would vanish
    # in the norm of 1.2e8 entries
    es_hvp, where_hvp = worst_slice(Hv_host, ref_Hv, wl.dims, wl.has_bias)
    del ref_Hv
    print("config5: oracle lower gradient", flush=True)
    ref_g = orc.lower_grad(prob, wl.w, wl.lam)[1]
    e_g = rel_l2(g_host, ref_g)
    es_g, where_g = worst_slice(g_host, ref_g, wl.dims, wl.has_bias)
    del ref_g
    print(f"config5 hvp {e_hvp:.2e} (worst tensor {where_hvp} {es_hvp:.2e}) lower gradient {e_g:.2e} "
          f"(worst tensor {where_g} {es_g:.2e})", flush=True)
    assert e_g < 2e-2 and es_g < 2e-2, (e_g, where_g, es_g)
    assert es_hvp < 2e-2, (where_hvp, es_hvp)
    print("config5: oracle neumann", flush=True)
    ref = orc.hypergrad_neumann(prob, wl.w, wl.lam, wl.K, wl.alpha)
    e_hg = rel_l2(got, ref)
    print(f"config5 hvp {e_hvp:.2e} neumann {e_hg:.2e}", flush=True)
    assert e_hvp < 2e-2 and e_hg < 2e-2

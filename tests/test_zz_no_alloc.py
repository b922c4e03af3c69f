"""The entry point for callers that cannot allocate device memory: betty_hvp_static runs the
Hessian-vector product on the library's fixed scratch array and must reproduce betty_hvp (same
kernels on the same data: bit for bit) and agree with the oracle, on two calls in a row of which the
second is a smaller problem (the array still holds the first call's contents)."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import betty_oracle as orc
from paper_2207_02849_amd import binding
from paper_2207_02849_amd import workloads as wk
from tests.util import oracle_problem, rel_l2

pytestmark = pytest.mark.gpu

TOL = {"fp32": 1e-4, "bf16": 2e-2}


def dev(a, dt=torch.float32):
    return torch.as_tensor(np.ascontiguousarray(a)).to(dt).contiguous().cuda()


def one_call(cfg):
    wl = wk.tiny(**cfg)
    prob = oracle_problem(wl)
    v = np.random.default_rng(7).standard_normal(wl.d).astype(np.float32)
    w, lam, vd = dev(wl.w), dev(wl.lam), dev(v)
    X = dev(wl.X_tr)
    y = dev(wl.y_tr, torch.int32) if wl.y_tr is not None else None
    t = dev(wl.t_tr) if wl.t_tr is not None else None
    # the new entry point through the C ABI, on a handle that was never bound to a workspace
    free = binding.Betty(wl.dims, act=wl.act, loss=wl.loss, hp=wl.hp, prec=wl.prec, has_bias=wl.has_bias,
                         batch_train=wl.X_tr.shape[0], batch_val=wl.X_val.shape[0], wnet_hidden=wl.wnet_hidden,
                         prox_rho=wl.prox_rho, prox_skip_last=wl.prox_skip_last, bind=False)
    assert free.workspace is None
    before = torch.cuda.memory_allocated()
    got = torch.empty(wl.d, device="cuda")
    during = torch.cuda.memory_allocated()
    free.betty_hvp_static(X, w, lam, vd, y_tr=y, t_tr=t, out=got)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == during and during - before <= got.numel() * 4 + 512
    # the existing entry point on a bound workspace
    b = binding.from_workload(wl)
    ref = b.betty_hvp(w, lam, vd)
    torch.cuda.synchronize()
    assert torch.equal(got, ref), cfg
    e = rel_l2(got.cpu().numpy(), orc.hvp(prob, wl.w.astype(np.float64), wl.lam.astype(np.float64), v.astype(np.float64)))
    print(wl.name, wl.dims, wl.prec, f"static hvp vs oracle {e:.2e}", flush=True)
    assert e < TOL[wl.prec]
    b.close()
    free.close()


def test_static_scratch_hvp_two_calls_the_second_smaller():
    assert binding.load_library().betty_static_scratch_bytes() == 64 << 20
    one_call(dict(kind="l2", act="gelu", loss="ce", dims=(300, 200, 150, 10), batch=130, prec="bf16"))
    one_call(dict(kind="reweight", act="relu", loss="ce", dims=(70, 50, 24), batch=37, prec="bf16", hidden=9))
    one_call(dict(kind="proximal", act="gelu", loss="mse", dims=(20, 30, 7), batch=6, prec="fp32", prox_rho=0.2,
                  prox_skip_last=True))


def test_static_scratch_rejects_problems_beyond_its_size():
    wl = wk.tiny(kind="l2", act="gelu", dims=(3072, 1024, 1024, 10), batch=16, prec="bf16")
    free = binding.Betty(wl.dims, act=wl.act, loss=wl.loss, hp=wl.hp, prec=wl.prec, batch_train=16, batch_val=18, bind=False)
    assert free.lib.betty_workspace_bytes(free.h) > (64 << 20)
    w, lam = dev(wl.w), dev(wl.lam)
    out = torch.full((wl.d,), 7.0, device="cuda")
    with pytest.raises(binding.BettyError) as e:
        free.betty_hvp_static(dev(wl.X_tr), w, lam, w, y_tr=dev(wl.y_tr, torch.int32), out=out)
    assert e.value.status == binding.EWORKSPACE and "scratch" in str(e.value)
    torch.cuda.synchronize()
    assert (out == 7.0).all()
    free.close()

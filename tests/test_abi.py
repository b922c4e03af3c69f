"""CPU-only checks of the C ABI: the library loads, exports every declared symbol, and
rejects bad problem descriptions on the host without touching a device."""
import ctypes as C
import os
import re

import pytest

from paper_2207_02849_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "betty_hip.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(betty_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = binding.load_library()
    names = declared_functions()
    assert {"betty_lower_grad", "betty_hvp", "betty_hypergrad_neumann", "betty_hypergrad_fd",
            "betty_mixed_vjp"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def _create(dims, **kw):
    lib = binding.load_library()
    arr = (C.c_int * len(dims))(*dims)
    args = dict(n_layers=len(dims) - 1, has_bias=1, act=1, loss=1, hp=0, prec=0, batch_train=4, batch_val=4,
                wnet_hidden=100, prox_rho=0.0, prox_skip_last=0)
    args.update(kw)
    desc = binding.ProblemDesc(args["n_layers"], arr, args["has_bias"], args["act"], args["loss"], args["hp"],
                               args["prec"], args["batch_train"], args["batch_val"], args["wnet_hidden"],
                               args["prox_rho"], args["prox_skip_last"])
    h = C.c_void_p()
    st = lib.betty_create(C.byref(desc), C.byref(h))
    return lib, st, h


def test_create_plans_sizes_on_the_host():
    lib, st, h = _create([784, 256, 10])
    assert st == binding.OK
    assert lib.betty_num_params(h) == 203530 and lib.betty_num_hyper(h) == 203530
    assert lib.betty_workspace_bytes(h) > 6 * 4 * 203530
    lib.betty_destroy(h)
    lib, st, h = _create([1024, 512, 512, 10], hp=1, prec=1, wnet_hidden=100)
    assert st == binding.OK and lib.betty_num_params(h) == 792586 and lib.betty_num_hyper(h) == 301
    lib.betty_destroy(h)
    lib, st, h = _create([12, 7, 3], hp=2, prox_rho=0.01, prox_skip_last=1)        # anchor has the layout of w
    assert st == binding.OK and lib.betty_num_params(h) == lib.betty_num_hyper(h) == 12 * 7 + 7 + 7 * 3 + 3
    lib.betty_destroy(h)


@pytest.mark.parametrize("kw,expect", [
    (dict(n_layers=0), binding.ESHAPE),
    (dict(batch_train=0), binding.ESHAPE),
    (dict(act=7), binding.EINVAL),
    (dict(loss=5), binding.EINVAL),
    (dict(hp=3), binding.EINVAL),
    (dict(prec=2), binding.EINVAL),
    (dict(hp=1, wnet_hidden=0), binding.ESHAPE),
    (dict(hp=2, prox_rho=-1.0), binding.EINVAL),
    (dict(hp=2, prox_rho=float("nan")), binding.EINVAL),
])
def test_create_rejects_bad_descriptions(kw, expect):
    _, st, h = _create([8, 4, 3], **kw)
    assert st == expect and not h.value


def test_create_rejects_bad_dims_and_nulls():
    _, st, _ = _create([8, 0, 3])
    assert st == binding.ESHAPE
    _, st, _ = _create([65536, 32768, 3])                 # a 2^31-element layer: beyond 32-bit offsets
    assert st == binding.ESHAPE
    _, st, _ = _create([1 << 20, 4, 3], batch_train=4096, batch_val=4)   # activation of 2^32 elements
    assert st == binding.ESHAPE
    lib = binding.load_library()
    assert lib.betty_create(None, None) == binding.ENULL


def test_calls_before_bind_fail_cleanly():
    lib, st, h = _create([8, 4, 3])
    assert st == binding.OK
    assert lib.betty_lower_grad(h, None, None, None, None) == binding.EWORKSPACE
    assert b"workspace" in lib.betty_last_error(h)
    assert lib.betty_bind(h, None, 0, None) == binding.ENULL
    assert lib.betty_bind(h, C.c_void_p(256 + 4), 1 << 40, None) == binding.EALIGN
    assert lib.betty_bind(h, C.c_void_p(4096), 16, None) == binding.EWORKSPACE
    assert lib.betty_apply_label_noise(h, None, None, None, 1.5, 4, None, None) == binding.EINVAL
    assert lib.betty_apply_label_noise(h, None, None, None, 0.5, -1, None, None) == binding.EINVAL
    lib.betty_destroy(h)

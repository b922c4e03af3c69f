"""ctypes binding of libbetty_hip.so: argument marshalling only.

Every step of the hypergradient path runs inside the library's HIP kernels; this
module only turns torch tensors into device pointers and forwards the calls of
include/betty_hip.h under the same names.  PyTorch provides device memory and the
stream handle, nothing else.  There is no fallback: a missing library is an error.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# BETTY_HIP_LIBRARY overrides the in-tree build (e.g. to try another build of the same ABI)
LIB_PATH = os.environ.get("BETTY_HIP_LIBRARY") or os.path.join(_HERE, "libbetty_hip.so")

ACT = {"none": 0, "relu": 1, "gelu": 2}
LOSS = {"mse": 0, "ce": 1}
HP = {"l2": 0, "reweight": 1, "proximal": 2}
PREC = {"fp32": 0, "bf16": 1}

OK, EINVAL, ENULL, ESHAPE, EWORKSPACE, EALIGN, EUNSUPPORTED, EDEVICE = 0, -1, -2, -3, -4, -5, -6, -7
KIND_NAMES = ["gemm", "epilogue", "loss", "shadow", "vector", "reduce", "wnet", "other", "gemm_update",
              "gemm_update_final", "last_layer", "gemm_rfwd", "gemm_rbwd"]


class ProblemDesc(C.Structure):
    _fields_ = [("n_layers", C.c_int), ("dims", C.POINTER(C.c_int)), ("has_bias", C.c_int),
                ("act", C.c_int), ("loss", C.c_int), ("hp", C.c_int), ("prec", C.c_int),
                ("batch_train", C.c_int), ("batch_val", C.c_int), ("wnet_hidden", C.c_int),
                ("prox_rho", C.c_float), ("prox_skip_last", C.c_int)]


class Batch(C.Structure):
    _fields_ = [("x", C.c_void_p), ("y", C.c_void_p), ("target", C.c_void_p)]


class ProfileRec(C.Structure):
    _fields_ = [("kind", C.c_int), ("ms", C.c_float), ("flops", C.c_double), ("bytes", C.c_double)]


class BettyError(RuntimeError):
    def __init__(self, status, text):
        super().__init__(f"betty status {status}: {text}")
        self.status = status


_lib = None


def load_library():
    """Loads the shared library built by paper_2207_02849_amd.build; raises if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} not found: build it first (python -m paper_2207_02849_amd.build); "
            "there is no CPU or PyTorch fallback")
    lib = C.CDLL(LIB_PATH)
    vp, f32p = C.c_void_p, C.c_void_p
    lib.betty_create.argtypes = [C.POINTER(ProblemDesc), C.POINTER(vp)]
    lib.betty_create.restype = C.c_int
    lib.betty_destroy.argtypes = [vp]
    lib.betty_destroy.restype = None
    lib.betty_last_error.argtypes = [vp]
    lib.betty_last_error.restype = C.c_char_p
    for name in ("betty_num_params", "betty_num_hyper", "betty_workspace_bytes"):
        getattr(lib, name).argtypes = [vp]
        getattr(lib, name).restype = C.c_size_t
    lib.betty_bind.argtypes = [vp, vp, C.c_size_t, vp]
    lib.betty_bind.restype = C.c_int
    lib.betty_set_batches.argtypes = [vp, Batch, Batch]
    lib.betty_set_batches.restype = C.c_int
    lib.betty_lower_grad.argtypes = [vp, f32p, f32p, f32p, f32p]
    lib.betty_upper_grad.argtypes = [vp, f32p, f32p, f32p]
    lib.betty_hvp.argtypes = [vp, f32p, f32p, f32p, f32p]
    lib.betty_mixed_vjp.argtypes = [vp, f32p, f32p, f32p, f32p]
    lib.betty_hvp_static.argtypes = [vp, Batch, vp, f32p, f32p, f32p, f32p]
    lib.betty_hvp_static.restype = C.c_int
    lib.betty_static_scratch_bytes.argtypes = []
    lib.betty_static_scratch_bytes.restype = C.c_size_t
    lib.betty_hypergrad_neumann.argtypes = [vp, f32p, f32p, C.c_int, C.c_float, f32p]
    lib.betty_hypergrad_fd.argtypes = [vp, f32p, f32p, C.c_int, C.c_float, C.c_float, f32p]
    lib.betty_hypergrad_cg.argtypes = [vp, f32p, f32p, C.c_int, f32p]
    lib.betty_best_response_neumann.argtypes = [vp, f32p, f32p, f32p, C.c_int, C.c_float, f32p]
    lib.betty_hypergrad_chain3.argtypes = [vp, vp, f32p, f32p, f32p, C.c_int, C.c_float, C.c_int, C.c_float, f32p]
    lib.betty_lower_sgd_step.argtypes = [vp, f32p, f32p, f32p, C.c_float, C.c_float, C.c_float, f32p]
    lib.betty_upper_adam_step.argtypes = [vp, f32p, f32p, f32p, f32p, C.c_int, C.c_float, C.c_float, C.c_float, C.c_float]
    lib.betty_apply_label_noise.argtypes = [vp, vp, vp, vp, C.c_double, C.c_int, vp, vp]
    lib.betty_profile_enable.argtypes = [vp, C.c_int]
    lib.betty_profile_collect.argtypes = [vp]
    lib.betty_profile_get.argtypes = [vp, C.c_int, C.POINTER(ProfileRec)]
    for name in ("betty_lower_grad", "betty_upper_grad", "betty_hvp", "betty_mixed_vjp",
                 "betty_hypergrad_neumann", "betty_hypergrad_fd", "betty_hypergrad_cg", "betty_best_response_neumann",
                 "betty_hypergrad_chain3", "betty_lower_sgd_step", "betty_upper_adam_step", "betty_apply_label_noise",
                 "betty_profile_enable", "betty_profile_collect", "betty_profile_get"):
        getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def _ptr(t: Optional[torch.Tensor], dtype=None, n=None):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected dtype {dtype}, got {t.dtype}")
    if n is not None and t.numel() != n:
        raise ValueError(f"expected {n} elements, got {t.numel()}")
    return t.data_ptr()


class Betty:
    """One problem description bound to a workspace and the current torch stream."""

    def __init__(self, dims: Sequence[int], act="relu", loss="ce", hp="l2", prec="fp32", has_bias=True,
                 batch_train=1, batch_val=1, wnet_hidden=100, prox_rho=0.0, prox_skip_last=False,
                 device="cuda:0", stream=None, bind=True):
        """bind=False leaves the handle without a workspace (none is allocated): only the calls that
        take no bound workspace work on it (betty_hvp_static)."""
        self.lib = load_library()
        self._dims = (C.c_int * len(dims))(*dims)
        desc = ProblemDesc(len(dims) - 1, self._dims, int(has_bias), ACT[act], LOSS[loss], HP[hp], PREC[prec],
                           batch_train, batch_val, wnet_hidden, float(prox_rho), int(bool(prox_skip_last)))
        self.h = C.c_void_p()
        st = self.lib.betty_create(C.byref(desc), C.byref(self.h))
        if st != OK:
            raise BettyError(st, "betty_create rejected the problem description")
        self.device = torch.device(device)
        self.d = self.lib.betty_num_params(self.h)
        self.n_hyper = self.lib.betty_num_hyper(self.h)
        self.dims, self.loss, self.hp = tuple(dims), loss, hp
        self.batch_train, self.batch_val = batch_train, batch_val
        nbytes = self.lib.betty_workspace_bytes(self.h)
        self._keep = []
        if not bind:
            self.workspace = None
            self.stream = torch.cuda.current_stream(self.device) if stream is None else stream
            return
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        # The library captures repeated calls into HIP graphs and overlaps launches on a second stream;
        # neither is possible on the legacy default stream, so without an explicit stream the handle
        # gets one of its own (default priority).  Whenever the handle's stream is not the caller's
        # current torch stream, every call is ordered against that stream with events, before and after.
        # Handles that work together (betty_hypergrad_chain3) must share a stream: pass the first one's.
        self.stream = torch.cuda.Stream(self.device) if stream is None else stream
        cur = torch.cuda.current_stream(self.device)
        if cur.cuda_stream != self.stream.cuda_stream:
            self.stream.wait_stream(cur)
        self._check(self.lib.betty_bind(self.h, self.workspace.data_ptr(), nbytes, self.stream.cuda_stream))
        self._keep = []

    def _check(self, st):
        if st != OK:
            raise BettyError(st, self.lib.betty_last_error(self.h).decode())

    def _call(self, fn, *args):
        cur = torch.cuda.current_stream(self.device)
        foreign = cur.cuda_stream != self.stream.cuda_stream
        if foreign:
            self.stream.wait_stream(cur)
        st = fn(self.h, *args)
        if foreign:
            cur.wait_stream(self.stream)
        self._check(st)

    def close(self):
        if getattr(self, "h", None) is not None and self.h.value:
            self.lib.betty_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- marshalling helpers
    def _vec(self, n):
        return torch.empty(n, dtype=torch.float32, device=self.device)

    def set_batches(self, X_tr, X_val, y_tr=None, y_val=None, t_tr=None, t_val=None):
        n0, nL = self.dims[0], self.dims[-1]
        tr = Batch(_ptr(X_tr, torch.float32, self.batch_train * n0), _ptr(y_tr, torch.int32, self.batch_train) if y_tr is not None else None,
                   _ptr(t_tr, torch.float32, self.batch_train * nL) if t_tr is not None else None)
        va = Batch(_ptr(X_val, torch.float32, self.batch_val * n0), _ptr(y_val, torch.int32, self.batch_val) if y_val is not None else None,
                   _ptr(t_val, torch.float32, self.batch_val * nL) if t_val is not None else None)
        self._keep = [X_tr, X_val, y_tr, y_val, t_tr, t_val]
        self._call(self.lib.betty_set_batches, tr, va)

    # ---- the calls of include/betty_hip.h, same names
    def betty_lower_grad(self, w, lam, want_loss=False):
        g = self._vec(self.d)
        loss = self._vec(1) if want_loss else None
        self._call(self.lib.betty_lower_grad, _ptr(w, torch.float32, self.d), _ptr(lam, torch.float32, self.n_hyper),
                                              g.data_ptr(), _ptr(loss))
        return (g, loss) if want_loss else g

    def betty_upper_grad(self, w, want_loss=False):
        g = self._vec(self.d)
        loss = self._vec(1) if want_loss else None
        self._call(self.lib.betty_upper_grad, _ptr(w, torch.float32, self.d), g.data_ptr(), _ptr(loss))
        return (g, loss) if want_loss else g

    def betty_hvp(self, w, lam, v, out=None):
        Hv = out if out is not None else self._vec(self.d)
        self._call(self.lib.betty_hvp, _ptr(w, torch.float32, self.d), _ptr(lam, torch.float32, self.n_hyper),
                                       _ptr(v, torch.float32, self.d), _ptr(Hv, torch.float32, self.d))
        return Hv

    def betty_hvp_static(self, X_tr, w, lam, v, y_tr=None, t_tr=None, out=None):
        """betty_hvp on the library's fixed scratch array: allocates nothing on the device inside the
        library (the output tensor is the caller's, or made here before the call)."""
        n0, nL = self.dims[0], self.dims[-1]
        Hv = out if out is not None else self._vec(self.d)
        self._keep = [X_tr, y_tr, t_tr]
        tr = Batch(_ptr(X_tr, torch.float32, self.batch_train * n0),
                   _ptr(y_tr, torch.int32, self.batch_train) if y_tr is not None else None,
                   _ptr(t_tr, torch.float32, self.batch_train * nL) if t_tr is not None else None)
        self._call(lambda h, *a: self.lib.betty_hvp_static(h, tr, self.stream.cuda_stream, *a),
                   _ptr(w, torch.float32, self.d), _ptr(lam, torch.float32, self.n_hyper),
                   _ptr(v, torch.float32, self.d), _ptr(Hv, torch.float32, self.d))
        return Hv

    def betty_mixed_vjp(self, w, lam, q, out=None):
        o = out if out is not None else self._vec(self.n_hyper)
        self._call(self.lib.betty_mixed_vjp, _ptr(w, torch.float32, self.d), _ptr(lam, torch.float32, self.n_hyper),
                                             _ptr(q, torch.float32, self.d), _ptr(o, torch.float32, self.n_hyper))
        return o

    def betty_hypergrad_neumann(self, w, lam, K, alpha, out=None):
        o = out if out is not None else self._vec(self.n_hyper)
        self._call(self.lib.betty_hypergrad_neumann, _ptr(w, torch.float32, self.d),
                                                     _ptr(lam, torch.float32, self.n_hyper), int(K), float(alpha),
                                                     _ptr(o, torch.float32, self.n_hyper))
        return o

    def betty_hypergrad_fd(self, w, lam, K, alpha, eps_scale=0.01, out=None):
        o = out if out is not None else self._vec(self.n_hyper)
        self._call(self.lib.betty_hypergrad_fd, _ptr(w, torch.float32, self.d),
                                                _ptr(lam, torch.float32, self.n_hyper), int(K), float(alpha),
                                                float(eps_scale), _ptr(o, torch.float32, self.n_hyper))
        return o

    def betty_hypergrad_cg(self, w, lam, K, out=None):
        o = out if out is not None else self._vec(self.n_hyper)
        self._call(self.lib.betty_hypergrad_cg, _ptr(w, torch.float32, self.d),
                                                _ptr(lam, torch.float32, self.n_hyper), int(K),
                                                _ptr(o, torch.float32, self.n_hyper))
        return o

    def betty_best_response_neumann(self, w, lam, u, K, alpha, out=None):
        o = out if out is not None else self._vec(self.n_hyper)
        self._call(self.lib.betty_best_response_neumann, _ptr(w, torch.float32, self.d),
                                                         _ptr(lam, torch.float32, self.n_hyper),
                                                         _ptr(u, torch.float32, self.d), int(K), float(alpha),
                                                         _ptr(o, torch.float32, self.n_hyper))
        return o

    def betty_hypergrad_chain3(self, finetune: "Betty", w, theta, v, K_pretrain, alpha_pretrain, K_finetune,
                               alpha_finetune, out=None):
        """self is the pretraining problem's handle, `finetune` the proximal one."""
        o = out if out is not None else self._vec(self.n_hyper)
        self._call(self.lib.betty_hypergrad_chain3, finetune.h, _ptr(w, torch.float32, self.d),
                                                    _ptr(theta, torch.float32, self.n_hyper),
                                                    _ptr(v, torch.float32, self.d), int(K_pretrain),
                                                    float(alpha_pretrain), int(K_finetune), float(alpha_finetune),
                                                    _ptr(o, torch.float32, self.n_hyper))
        return o

    def betty_lower_sgd_step(self, w, lam, momentum, lr, mu, weight_decay=0.0, want_loss=False):
        loss = self._vec(1) if want_loss else None
        self._call(self.lib.betty_lower_sgd_step, _ptr(w, torch.float32, self.d),
                                                  _ptr(lam, torch.float32, self.n_hyper),
                                                  _ptr(momentum, torch.float32, self.d), float(lr), float(mu),
                                                  float(weight_decay), _ptr(loss))
        return loss

    def betty_upper_adam_step(self, lam, dlam, m, v, t, lr, beta1=0.9, beta2=0.999, eps=1e-8):
        self._call(self.lib.betty_upper_adam_step, _ptr(lam, torch.float32, self.n_hyper),
                                                   _ptr(dlam, torch.float32, self.n_hyper),
                                                   _ptr(m, torch.float32, self.n_hyper),
                                                   _ptr(v, torch.float32, self.n_hyper), int(t), float(lr),
                                                   float(beta1), float(beta2), float(eps))

    def betty_apply_label_noise(self, y, words, alt, p, want_mask=True):
        n = y.numel()
        if words.element_size() != 4:
            raise ValueError("words must hold 32-bit values")
        out = torch.empty(n, dtype=torch.int32, device=self.device)
        mask = torch.empty(n, dtype=torch.uint8, device=self.device) if want_mask else None
        self._call(self.lib.betty_apply_label_noise, _ptr(y, torch.int32), _ptr(words, None, n),
                                                     _ptr(alt, torch.int32, n), float(p), n, out.data_ptr(), _ptr(mask))
        return out, mask

    # ---- per-kernel timing
    def profile(self, on: bool):
        self._check(self.lib.betty_profile_enable(self.h, int(on)))

    def profile_records(self):
        n = self.lib.betty_profile_collect(self.h)
        rec, out = ProfileRec(), []
        for i in range(n):
            self._check(self.lib.betty_profile_get(self.h, i, C.byref(rec)))
            out.append((KIND_NAMES[rec.kind], rec.ms, rec.flops, rec.bytes))
        return out


def from_workload(wl, device="cuda:0", stream=None) -> "Betty":
    """Creates a handle for a seeded workload and uploads its batches."""
    b = Betty(wl.dims, act=wl.act, loss=wl.loss, hp=wl.hp, prec=wl.prec, has_bias=wl.has_bias,
              batch_train=wl.X_tr.shape[0], batch_val=wl.X_val.shape[0], wnet_hidden=wl.wnet_hidden,
              prox_rho=wl.prox_rho, prox_skip_last=wl.prox_skip_last, device=device, stream=stream)
    dev = b.device

    def up(a, dt):
        return None if a is None else torch.as_tensor(a).to(dt).contiguous().to(dev)
    y_tr = up(wl.y_tr, torch.int32)
    if y_tr is None and wl.y_clean is not None:
        # label noise: the train labels are made on the device from the drawn ingredients
        import numpy as np
        words = torch.as_tensor(np.ascontiguousarray(wl.noise_words).view(np.int32)).to(dev)
        y_tr, _ = b.betty_apply_label_noise(up(wl.y_clean, torch.int32), words, up(wl.noise_alt, torch.int32),
                                            wl.noise_p, want_mask=False)
    b.set_batches(up(wl.X_tr, torch.float32), up(wl.X_val, torch.float32), y_tr,
                  up(wl.y_val, torch.int32), up(wl.t_tr, torch.float32), up(wl.t_val, torch.float32))
    return b

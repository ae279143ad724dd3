"""Thin ctypes binding over libbagel.so (C ABI in include/bagel.h).

Argument marshalling only: every function below checks shapes / dtypes / device of the torch
tensors it is given and passes their device pointers through.  PyTorch supplies device memory
and the stream; all computation happens inside the library's HIP kernels.  There is no
fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbagel.so")

OK, EINVAL, ENOTPREPARED, ENOMEM, ENOTPD, EHIP = 0, -1, -2, -3, -4, -5
_NAMES = {EINVAL: "BAGEL_EINVAL", ENOTPREPARED: "BAGEL_ENOTPREPARED", ENOMEM: "BAGEL_ENOMEM",
          ENOTPD: "BAGEL_ENOTPD", EHIP: "BAGEL_EHIP"}

EXPORTS = ["bagel_num_params", "bagel_create", "bagel_destroy", "bagel_workspace_bytes",
           "bagel_prepare_samples", "bagel_set_samples", "bagel_rollout_loss",
           "bagel_rollout_loss_grad", "bagel_sample_eval", "bagel_last_error", "bagel_adam_step", "bagel_optimize",
           "bagel_hyper_lml_grad", "bagel_hyper_fit", "bagel_prepare_posterior", "bagel_posterior_rollout_loss", "bagel_posterior_rollout_loss_grad",
           "bagel_profile_enable", "bagel_profile_read", "bagel_sample_eval_static"]


class BagelError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{_NAMES.get(code, code)}: {msg}")
        self.code = code


class Dims(C.Structure):
    _fields_ = [
        ("d_s", C.c_int32), ("d_a", C.c_int32), ("d_g", C.c_int32),
        ("N", C.c_int32), ("L", C.c_int32), ("S", C.c_int32), ("B", C.c_int32), ("H", C.c_int32),
        ("n_hidden", C.c_int32), ("hidden", C.c_int32 * 2),
        ("act_bound", C.c_float),
        ("tracked", C.c_int32 * 8), ("q", C.c_float * 8),
        ("ckpt_interval", C.c_int32), ("cost_kind", C.c_int32), ("sigma_r", C.c_float),
    ]


def make_dims(*, d_s, d_a, d_g, N, L, S, B, H, hidden: Sequence[int], act_bound=0.0, tracked=None,
              q=None, ckpt_interval=0, cost_kind=0, sigma_r=1.0) -> Dims:
    dm = Dims()
    dm.d_s, dm.d_a, dm.d_g = d_s, d_a, d_g
    dm.N, dm.L, dm.S, dm.B, dm.H = N, L, S, B, H
    dm.n_hidden = len(hidden)
    for i, h in enumerate(list(hidden)[:2]):
        dm.hidden[i] = h
    dm.act_bound = float(act_bound)
    tracked = list(range(d_g)) if tracked is None else list(tracked)
    q = [1.0] * d_g if q is None else list(q)
    for j in range(min(d_g, 8)):
        dm.tracked[j] = tracked[j]
        dm.q[j] = q[j]
    dm.ckpt_interval, dm.cost_kind, dm.sigma_r = ckpt_interval, cost_kind, float(sigma_r)
    return dm


def dims_from_config(cfg, S: Optional[int] = None, **kw) -> Dims:
    kw.setdefault("ckpt_interval", cfg.ckpt_interval)
    return make_dims(d_s=cfg.d_s, d_a=cfg.d_a, d_g=cfg.d_g, N=cfg.N, L=cfg.L,
                     S=cfg.B if S is None else S, B=cfg.B, H=cfg.H, hidden=cfg.hidden,
                     act_bound=cfg.act_bound, tracked=cfg.tracked, q=cfg.q, **kw)


_lib = None


def load():
    """Load libbagel.so; raises if it has not been built (python -m paper_2202_13638_amd.build)."""
    global _lib
    if _lib is None:
        # torch first: the library must bind to the HIP runtime that torch has already loaded, so
        # that device pointers and streams handed over belong to the same runtime instance
        import torch  # noqa: F401
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2202_13638_amd.build`")
        L = C.CDLL(LIB_PATH)
        fp, vp = C.c_void_p, C.c_void_p
        L.bagel_num_params.restype = C.c_int
        L.bagel_num_params.argtypes = [C.POINTER(Dims)]
        L.bagel_create.restype = C.c_int
        L.bagel_create.argtypes = [C.POINTER(vp), C.POINTER(Dims), vp]
        L.bagel_destroy.restype = C.c_int
        L.bagel_destroy.argtypes = [vp]
        L.bagel_workspace_bytes.restype = C.c_int64
        L.bagel_workspace_bytes.argtypes = [vp]
        L.bagel_prepare_samples.restype = C.c_int
        L.bagel_prepare_samples.argtypes = [vp] + [fp] * 10
        L.bagel_set_samples.restype = C.c_int
        L.bagel_set_samples.argtypes = [vp] + [fp] * 7
        L.bagel_rollout_loss.restype = C.c_int
        L.bagel_rollout_loss.argtypes = [vp] + [fp] * 6
        L.bagel_rollout_loss_grad.restype = C.c_int
        L.bagel_rollout_loss_grad.argtypes = [vp] + [fp] * 8
        L.bagel_sample_eval.restype = C.c_int
        L.bagel_sample_eval.argtypes = [vp] + [fp] * 3
        L.bagel_profile_enable.restype = C.c_int
        L.bagel_profile_enable.argtypes = [vp, C.c_int]
        L.bagel_profile_read.restype = C.c_int
        L.bagel_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_int)]
        L.bagel_prepare_posterior.restype = C.c_int
        L.bagel_prepare_posterior.argtypes = [vp] + [fp] * 5
        L.bagel_posterior_rollout_loss.restype = C.c_int
        L.bagel_posterior_rollout_loss.argtypes = [vp] + [fp] * 7
        L.bagel_posterior_rollout_loss_grad.restype = C.c_int
        L.bagel_posterior_rollout_loss_grad.argtypes = [vp] + [fp] * 9
        L.bagel_hyper_lml_grad.restype = C.c_int
        L.bagel_hyper_lml_grad.argtypes = [vp] + [fp] * 5
        L.bagel_hyper_fit.restype = C.c_int
        L.bagel_hyper_fit.argtypes = [vp] + [fp] * 5 + [C.c_int] * 2 + [C.c_float] * 4 + [fp]
        L.bagel_adam_step.restype = C.c_int
        L.bagel_adam_step.argtypes = [vp] + [fp] * 4 + [C.c_int] + [C.c_float] * 4
        L.bagel_optimize.restype = C.c_int
        L.bagel_optimize.argtypes = [vp] + [fp] * 5 + [C.c_int] * 3 + [C.c_float] * 4 + [fp]
        L.bagel_sample_eval_static.restype = C.c_int
        L.bagel_sample_eval_static.argtypes = [C.POINTER(Dims), vp] + [fp] * 10
        L.bagel_last_error.restype = C.c_char_p
        L.bagel_last_error.argtypes = [vp]
        _lib = L
    return _lib


def bagel_num_params(dims: Dims) -> int:
    return int(load().bagel_num_params(C.byref(dims)))


def _ptr(t, shape, name, optional=False):
    import torch
    if t is None:
        if optional:
            return None
        raise ValueError(f"{name} is required")
    if not isinstance(t, torch.Tensor) or not t.is_cuda or t.dtype != torch.float32 or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous float32 tensor on the GPU")
    if tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} has shape {tuple(t.shape)}, expected {tuple(shape)}")
    return C.c_void_p(t.data_ptr())


def bagel_sample_eval_static(dims: Dims, X, lengthscale, signal_var, omega, phase, w, v, x, f, jac=None, stream=None):
    """The context-free, allocation-free sample evaluation (see include/bagel.h)."""
    import torch
    lib = load()
    M, D = dims.d_s, dims.d_s + dims.d_a
    if stream is None:
        stream = torch.cuda.current_stream()
    rc = lib.bagel_sample_eval_static(
        C.byref(dims), C.c_void_p(stream.cuda_stream), _ptr(X, (dims.N, D), "X"),
        _ptr(lengthscale, (M, D), "lengthscale"), _ptr(signal_var, (M,), "signal_var"),
        _ptr(omega, (M, dims.L, D), "omega"), _ptr(phase, (M, dims.L), "phase"), _ptr(w, (dims.S, M, dims.L), "w"),
        _ptr(v, (dims.S, M, dims.N), "v"), _ptr(x, (dims.B, D), "x"), _ptr(f, (dims.B, M), "f"),
        _ptr(jac, (dims.B, M, D), "jac", optional=True))
    if rc != OK:
        raise BagelError(rc, lib.bagel_last_error(None).decode())


class Bagel:
    """One context = one set of dims on the current device and stream."""

    def __init__(self, dims: Dims, stream=None):
        import torch
        self._lib = load()
        self.dims = dims
        self._h = C.c_void_p()
        if stream is None:
            stream = torch.cuda.current_stream()
        self.stream = stream
        rc = self._lib.bagel_create(C.byref(self._h), C.byref(dims), C.c_void_p(stream.cuda_stream))
        if rc != OK:
            msg = self._lib.bagel_last_error(None).decode()
            self._h = C.c_void_p()
            raise BagelError(rc, msg)
        self.P = bagel_num_params(dims)
        self.M = dims.d_s
        self.D = dims.d_s + dims.d_a

    # -- helpers -------------------------------------------------------------------------
    def _check(self, rc: int):
        if rc != OK:
            raise BagelError(rc, self._lib.bagel_last_error(self._h).decode())

    def workspace_bytes(self) -> int:
        return int(self._lib.bagel_workspace_bytes(self._h))

    def close(self):
        if self._h:
            self._lib.bagel_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the entry points, same names as the C ABI --------------------------------------------
    def bagel_prepare_samples(self, X, y, lengthscale, signal_var, noise_var, omega, phase, w, eps, v_out=None):
        d, M, D = self.dims, self.M, self.D
        self._check(self._lib.bagel_prepare_samples(
            self._h, _ptr(X, (d.N, D), "X"), _ptr(y, (M, d.N), "y"), _ptr(lengthscale, (M, D), "lengthscale"),
            _ptr(signal_var, (M,), "signal_var"), _ptr(noise_var, (M,), "noise_var"),
            _ptr(omega, (M, d.L, D), "omega"), _ptr(phase, (M, d.L), "phase"), _ptr(w, (d.S, M, d.L), "w"),
            _ptr(eps, (d.S, M, d.N), "eps"), _ptr(v_out, (d.S, M, d.N), "v_out", optional=True)))

    def bagel_set_samples(self, X, lengthscale, signal_var, omega, phase, w, v):
        d, M, D = self.dims, self.M, self.D
        self._check(self._lib.bagel_set_samples(
            self._h, _ptr(X, (d.N, D), "X"), _ptr(lengthscale, (M, D), "lengthscale"),
            _ptr(signal_var, (M,), "signal_var"), _ptr(omega, (M, d.L, D), "omega"),
            _ptr(phase, (M, d.L), "phase"), _ptr(w, (d.S, M, d.L), "w"), _ptr(v, (d.S, M, d.N), "v")))

    def bagel_rollout_loss(self, theta, s0, goals, loss, loss_per_traj=None, states=None):
        d = self.dims
        self._check(self._lib.bagel_rollout_loss(
            self._h, _ptr(theta, (self.P,), "theta"), _ptr(s0, (d.B, d.d_s), "s0"),
            _ptr(goals, (d.H, d.B, d.d_g), "goals"), _ptr(loss, (1,), "loss"),
            _ptr(loss_per_traj, (d.B,), "loss_per_traj", optional=True),
            _ptr(states, (d.H + 1, d.B, d.d_s), "states", optional=True)))

    def bagel_rollout_loss_grad(self, theta, s0, goals, loss, grad_theta, loss_per_traj=None, states=None,
                                grad_s0=None):
        d = self.dims
        self._check(self._lib.bagel_rollout_loss_grad(
            self._h, _ptr(theta, (self.P,), "theta"), _ptr(s0, (d.B, d.d_s), "s0"),
            _ptr(goals, (d.H, d.B, d.d_g), "goals"), _ptr(loss, (1,), "loss"),
            _ptr(grad_theta, (self.P,), "grad_theta"),
            _ptr(loss_per_traj, (d.B,), "loss_per_traj", optional=True),
            _ptr(states, (d.H + 1, d.B, d.d_s), "states", optional=True),
            _ptr(grad_s0, (d.B, d.d_s), "grad_s0", optional=True)))

    def bagel_prepare_posterior(self, X, y, lengthscale, signal_var, noise_var):
        d, M, D = self.dims, self.M, self.D
        self._check(self._lib.bagel_prepare_posterior(
            self._h, _ptr(X, (d.N, D), "X"), _ptr(y, (M, d.N), "y"), _ptr(lengthscale, (M, D), "lengthscale"),
            _ptr(signal_var, (M,), "signal_var"), _ptr(noise_var, (M,), "noise_var")))

    def bagel_posterior_rollout_loss(self, theta, s0, goals, xi, loss, loss_per_traj=None, states=None):
        d = self.dims
        self._check(self._lib.bagel_posterior_rollout_loss(
            self._h, _ptr(theta, (self.P,), "theta"), _ptr(s0, (d.B, d.d_s), "s0"),
            _ptr(goals, (d.H, d.B, d.d_g), "goals"), _ptr(xi, (d.H, d.B, self.M), "xi"), _ptr(loss, (1,), "loss"),
            _ptr(loss_per_traj, (d.B,), "loss_per_traj", optional=True),
            _ptr(states, (d.H + 1, d.B, d.d_s), "states", optional=True)))

    def bagel_posterior_rollout_loss_grad(self, theta, s0, goals, xi, loss, grad_theta, loss_per_traj=None,
                                          states=None, grad_s0=None):
        d = self.dims
        self._check(self._lib.bagel_posterior_rollout_loss_grad(
            self._h, _ptr(theta, (self.P,), "theta"), _ptr(s0, (d.B, d.d_s), "s0"),
            _ptr(goals, (d.H, d.B, d.d_g), "goals"), _ptr(xi, (d.H, d.B, self.M), "xi"), _ptr(loss, (1,), "loss"),
            _ptr(grad_theta, (self.P,), "grad_theta"),
            _ptr(loss_per_traj, (d.B,), "loss_per_traj", optional=True),
            _ptr(states, (d.H + 1, d.B, d.d_s), "states", optional=True),
            _ptr(grad_s0, (d.B, d.d_s), "grad_s0", optional=True)))

    def bagel_hyper_lml_grad(self, X, y, log_hyp, lml, grad=None):
        d, M, D = self.dims, self.M, self.D
        self._check(self._lib.bagel_hyper_lml_grad(
            self._h, _ptr(X, (d.N, D), "X"), _ptr(y, (M, d.N), "y"), _ptr(log_hyp, (M, D + 2), "log_hyp"),
            _ptr(lml, (M,), "lml"), _ptr(grad, (M, D + 2), "grad", optional=True)))

    def bagel_hyper_fit(self, X, y, log_hyp, adam_m, adam_v, n_iters, lml_history, first_step=1, lr=1e-2, beta1=0.9,
                        beta2=0.999, eps=1e-8):
        d, M, D = self.dims, self.M, self.D
        self._check(self._lib.bagel_hyper_fit(
            self._h, _ptr(X, (d.N, D), "X"), _ptr(y, (M, d.N), "y"), _ptr(log_hyp, (M, D + 2), "log_hyp"),
            _ptr(adam_m, (M, D + 2), "adam_m"), _ptr(adam_v, (M, D + 2), "adam_v"), int(n_iters), int(first_step),
            lr, beta1, beta2, eps, _ptr(lml_history, (int(n_iters), M), "lml_history")))

    def bagel_adam_step(self, theta, grad, adam_m, adam_v, step, lr=1e-2, beta1=0.9, beta2=0.999, eps=1e-8):
        P = (self.P,)
        self._check(self._lib.bagel_adam_step(
            self._h, _ptr(theta, P, "theta"), _ptr(grad, P, "grad"), _ptr(adam_m, P, "adam_m"),
            _ptr(adam_v, P, "adam_v"), int(step), lr, beta1, beta2, eps))

    def bagel_optimize(self, theta, adam_m, adam_v, s0_sets, goal_sets, n_iters, loss_history, first_step=1,
                       lr=1e-2, beta1=0.9, beta2=0.999, eps=1e-8):
        d, P = self.dims, (self.P,)
        n_sets = int(s0_sets.shape[0]) if hasattr(s0_sets, "shape") and len(s0_sets.shape) == 3 else 0
        self._check(self._lib.bagel_optimize(
            self._h, _ptr(theta, P, "theta"), _ptr(adam_m, P, "adam_m"), _ptr(adam_v, P, "adam_v"),
            _ptr(s0_sets, (n_sets, d.B, d.d_s), "s0_sets"), _ptr(goal_sets, (n_sets, d.H, d.B, d.d_g), "goal_sets"),
            n_sets, int(n_iters), int(first_step), lr, beta1, beta2, eps,
            _ptr(loss_history, (int(n_iters),), "loss_history")))

    def bagel_profile_enable(self, every: int):
        self._check(self._lib.bagel_profile_enable(self._h, int(every)))

    def bagel_profile_read(self):
        ms, n = C.c_double(), C.c_int()
        self._check(self._lib.bagel_profile_read(self._h, C.byref(ms), C.byref(n)))
        return ms.value, n.value

    def bagel_sample_eval(self, x, f, jac=None):
        d = self.dims
        self._check(self._lib.bagel_sample_eval(
            self._h, _ptr(x, (d.B, self.D), "x"), _ptr(f, (d.B, self.M), "f"),
            _ptr(jac, (d.B, self.M, self.D), "jac", optional=True)))

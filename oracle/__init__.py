"""ctypes loader for the float64 CPU oracle (``bagel_oracle.c``).

TEST INFRASTRUCTURE: only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this package.  It shares nothing
with the HIP path.  Every array handed in is promoted to float64; the float32
inputs of a workload are therefore used at exactly the values the GPU sees.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bagel_oracle.c")
_LIB = os.path.join(_HERE, "libbagel_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no arch-specific flags: the library travels between hosts)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class Dims(C.Structure):
    _fields_ = [
        ("d_s", C.c_int32), ("d_a", C.c_int32), ("d_g", C.c_int32),
        ("N", C.c_int32), ("L", C.c_int32), ("S", C.c_int32), ("B", C.c_int32), ("H", C.c_int32),
        ("n_hidden", C.c_int32), ("hidden", C.c_int32 * 2),
        ("act_bound", C.c_double),
        ("tracked", C.c_int32 * 8), ("q", C.c_double * 8),
        ("cost_kind", C.c_int32), ("sigma_r", C.c_double),
    ]


def make_dims(*, d_s, d_a, d_g, N, L, S, B, H, hidden, act_bound=0.0, tracked=None, q=None,
              cost_kind=0, sigma_r=1.0) -> Dims:
    dm = Dims()
    dm.d_s, dm.d_a, dm.d_g = d_s, d_a, d_g
    dm.N, dm.L, dm.S, dm.B, dm.H = N, L, S, B, H
    dm.n_hidden = len(hidden)
    for i, h in enumerate(hidden):
        dm.hidden[i] = h
    dm.act_bound = float(act_bound)
    tracked = list(range(d_g)) if tracked is None else list(tracked)
    q = [1.0] * d_g if q is None else list(q)
    for j in range(d_g):
        dm.tracked[j] = tracked[j]
        dm.q[j] = q[j]
    dm.cost_kind = cost_kind
    dm.sigma_r = float(sigma_r)
    return dm


def dims_from_config(cfg, S: Optional[int] = None, **kw) -> Dims:
    return make_dims(d_s=cfg.d_s, d_a=cfg.d_a, d_g=cfg.d_g, N=cfg.N, L=cfg.L,
                     S=cfg.B if S is None else S, B=cfg.B, H=cfg.H, hidden=cfg.hidden,
                     act_bound=cfg.act_bound, tracked=cfg.tracked, q=cfg.q, **kw)


_DP = C.POINTER(C.c_double)


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        L.oracle_num_threads.restype = C.c_int
        L.oracle_kernel.restype = C.c_double
        L.oracle_kernel.argtypes = [C.c_int, _DP, C.c_double, _DP, _DP]
        L.oracle_features.restype = None
        L.oracle_features.argtypes = [C.c_int, C.c_int, C.c_double, _DP, _DP, _DP, _DP]
        L.oracle_prepare_samples.restype = C.c_int
        L.oracle_prepare_samples.argtypes = [C.POINTER(Dims)] + [_DP] * 10
        L.oracle_sample_eval.restype = None
        L.oracle_sample_eval.argtypes = [C.POINTER(Dims)] + [_DP] * 10
        L.oracle_num_params.restype = C.c_int
        L.oracle_num_params.argtypes = [C.POINTER(Dims)]
        L.oracle_policy.restype = None
        L.oracle_policy.argtypes = [C.POINTER(Dims), _DP, _DP, _DP]
        L.oracle_rollout.restype = C.c_int
        L.oracle_rollout.argtypes = [C.POINTER(Dims)] + [_DP] * 15
        L.oracle_posterior_prepare.restype = C.c_int
        L.oracle_posterior_prepare.argtypes = [C.POINTER(Dims)] + [_DP] * 7
        L.oracle_posterior_moments.restype = None
        L.oracle_posterior_moments.argtypes = [C.POINTER(Dims)] + [_DP] * 11
        L.oracle_posterior_rollout.restype = C.c_int
        L.oracle_posterior_rollout.argtypes = [C.POINTER(Dims)] + [_DP] * 14
        L.oracle_adam_step.restype = None
        L.oracle_adam_step.argtypes = [C.c_int, _DP, _DP, _DP, _DP, C.c_int] + [C.c_double] * 4
        _lib = L
    return _lib


def _d(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(_DP)


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def kernel(ell, sf2, xa, xb) -> float:
    ell, xa, xb = _d(ell), _d(xa), _d(xb)
    return float(lib().oracle_kernel(len(ell), _p(ell), float(sf2), _p(xa), _p(xb)))


def features(sf2, omega, phase, x) -> np.ndarray:
    omega, phase, x = _d(omega), _d(phase), _d(x)
    L, D = omega.shape
    out = np.empty(L)
    lib().oracle_features(D, L, float(sf2), _p(omega), _p(phase), _p(x), _p(out))
    return out


def prepare_samples(dm: Dims, m: Dict[str, np.ndarray]) -> np.ndarray:
    """v[S,M,N] from the model arrays X y lengthscale signal_var noise_var omega phase w eps."""
    a = {k: _d(m[k]) for k in ("X", "y", "lengthscale", "signal_var", "noise_var", "omega", "phase", "w", "eps")}
    M = dm.d_s
    assert a["w"].shape == (dm.S, M, dm.L) and a["eps"].shape == (dm.S, M, dm.N)
    v = np.empty((dm.S, M, dm.N))
    rc = lib().oracle_prepare_samples(C.byref(dm), _p(a["X"]), _p(a["y"]), _p(a["lengthscale"]),
                                      _p(a["signal_var"]), _p(a["noise_var"]), _p(a["omega"]),
                                      _p(a["phase"]), _p(a["w"]), _p(a["eps"]), _p(v))
    if rc != 0:
        raise FloatingPointError(f"oracle_prepare_samples failed with code {rc}")
    return v


def sample_eval(dm: Dims, m: Dict[str, np.ndarray], w_s, v_s, x, jac: bool = True):
    a = {k: _d(m[k]) for k in ("X", "lengthscale", "signal_var", "omega", "phase")}
    w_s, v_s, x = _d(w_s), _d(v_s), _d(x)
    M, D = dm.d_s, dm.d_s + dm.d_a
    f = np.empty(M)
    J = np.empty((M, D)) if jac else None
    lib().oracle_sample_eval(C.byref(dm), _p(a["X"]), _p(a["lengthscale"]), _p(a["signal_var"]),
                             _p(a["omega"]), _p(a["phase"]), _p(w_s), _p(v_s), _p(x), _p(f), _p(J))
    return (f, J) if jac else f


def num_params(dm: Dims) -> int:
    return int(lib().oracle_num_params(C.byref(dm)))


def policy(dm: Dims, theta, h0) -> np.ndarray:
    theta, h0 = _d(theta), _d(h0)
    a = np.empty(dm.d_a)
    lib().oracle_policy(C.byref(dm), _p(theta), _p(h0), _p(a))
    return a


def rollout(dm: Dims, m: Dict[str, np.ndarray], v, theta=None, s0=None, goals=None, *,
            grad: bool = True, want_states: bool = True):
    """Returns dict(loss, loss_per_traj, states, grad_theta, grad_s0) (float64)."""
    a = {k: _d(m[k]) for k in ("X", "lengthscale", "signal_var", "omega", "phase", "w")}
    v = _d(v)
    theta = _d(m["theta"] if theta is None else theta)
    s0 = _d(m["s0"] if s0 is None else s0)
    goals = _d(m["goals"] if goals is None else goals)
    M = dm.d_s
    assert v.shape == (dm.S, M, dm.N) and a["w"].shape == (dm.S, M, dm.L)
    assert s0.shape == (dm.B, dm.d_s) and goals.shape == (dm.H, dm.B, dm.d_g)
    P = num_params(dm)
    assert theta.shape == (P,)
    loss = np.zeros(1)
    lpt = np.empty(dm.B)
    states = np.empty((dm.H + 1, dm.B, dm.d_s)) if want_states else None
    g = np.zeros(P) if grad else None
    gs0 = np.zeros((dm.B, dm.d_s)) if grad else None
    rc = lib().oracle_rollout(C.byref(dm), _p(a["X"]), _p(a["lengthscale"]), _p(a["signal_var"]),
                              _p(a["omega"]), _p(a["phase"]), _p(a["w"]), _p(v), _p(theta), _p(s0),
                              _p(goals), _p(loss), _p(lpt), _p(states), _p(g), _p(gs0))
    if rc != 0:
        raise RuntimeError(f"oracle_rollout failed with code {rc}")
    return {"loss": float(loss[0]), "loss_per_traj": lpt, "states": states, "grad_theta": g, "grad_s0": gs0}


ADAM_DEFAULTS = dict(lr=1e-2, beta1=0.9, beta2=0.999, eps=1e-8)   # lr: Sec. IV-A; the rest: Adam's own defaults


def adam_step(theta, grad, m, v, t: int, *, lr=1e-2, beta1=0.9, beta2=0.999, eps=1e-8) -> None:
    """In-place Adam update of float64 arrays theta, m, v (step counter t >= 1)."""
    for a in (theta, m, v):
        assert a.dtype == np.float64 and a.flags.c_contiguous
    grad = _d(grad)
    lib().oracle_adam_step(len(theta), _p(theta), _p(grad), _p(m), _p(v), int(t), float(lr), float(beta1),
                           float(beta2), float(eps))


def optimize(dm: Dims, m: Dict[str, np.ndarray], v, theta0, s0_sets, goal_sets, n_iters: int, *,
             first_step: int = 1, adam_m=None, adam_v=None, **adam):
    """Inner loop of Algorithm 1: iteration i rolls out from s0_sets[i % n_sets] towards goal_sets[i % n_sets],
    takes the gradient of the loss and updates theta with Adam.  Returns (theta, adam_m, adam_v, losses)."""
    theta = _d(theta0).copy()
    am = np.zeros_like(theta) if adam_m is None else _d(adam_m).copy()
    av = np.zeros_like(theta) if adam_v is None else _d(adam_v).copy()
    losses = np.empty(n_iters)
    n_sets = len(s0_sets)
    for i in range(n_iters):
        r = rollout(dm, m, v, theta=theta, s0=s0_sets[i % n_sets], goals=goal_sets[i % n_sets], want_states=False)
        losses[i] = r["loss"]
        adam_step(theta, r["grad_theta"], am, av, first_step + i, **adam)
    return theta, am, av, losses


def posterior_prepare(dm: Dims, m: Dict[str, np.ndarray]):
    """alpha[M,N] = K_hat^-1 y and Kinv[M,N,N] = K_hat^-1 (eq. (2), (3)) from X y lengthscale signal_var noise_var."""
    a = {k: _d(m[k]) for k in ("X", "y", "lengthscale", "signal_var", "noise_var")}
    M = dm.d_s
    alpha = np.empty((M, dm.N))
    Kinv = np.empty((M, dm.N, dm.N))
    rc = lib().oracle_posterior_prepare(C.byref(dm), _p(a["X"]), _p(a["y"]), _p(a["lengthscale"]), _p(a["signal_var"]),
                                        _p(a["noise_var"]), _p(alpha), _p(Kinv))
    if rc != 0:
        raise FloatingPointError(f"oracle_posterior_prepare failed with code {rc}")
    return alpha, Kinv


def posterior_moments(dm: Dims, m: Dict[str, np.ndarray], alpha, Kinv, x, jac: bool = True):
    """mu[M], var[M] (and dmu[M,D], dvar[M,D]) of the predictive posterior at x[D]."""
    a = {k: _d(m[k]) for k in ("X", "lengthscale", "signal_var")}
    alpha, Kinv, x = _d(alpha), _d(Kinv), _d(x)
    M, D = dm.d_s, dm.d_s + dm.d_a
    mu, var = np.empty(M), np.empty(M)
    dmu = np.empty((M, D)) if jac else None
    dvar = np.empty((M, D))
    work = np.empty(2 * dm.N)
    lib().oracle_posterior_moments(C.byref(dm), _p(a["X"]), _p(a["lengthscale"]), _p(a["signal_var"]), _p(alpha),
                                   _p(Kinv), _p(x), _p(mu), _p(var), _p(dmu), _p(dvar), _p(work))
    return (mu, var, dmu, dvar) if jac else (mu, var)


def posterior_rollout(dm: Dims, m: Dict[str, np.ndarray], alpha, Kinv, xi, theta=None, s0=None, goals=None, *,
                      grad: bool = True, want_states: bool = True):
    """Algorithm 1 with per-step posterior draws f = mu + sqrt(var) xi, xi[H,B,M].  Returns the dict of rollout()."""
    a = {k: _d(m[k]) for k in ("X", "lengthscale", "signal_var")}
    alpha, Kinv, xi = _d(alpha), _d(Kinv), _d(xi)
    theta = _d(m["theta"] if theta is None else theta)
    s0 = _d(m["s0"] if s0 is None else s0)
    goals = _d(m["goals"] if goals is None else goals)
    M = dm.d_s
    assert alpha.shape == (M, dm.N) and Kinv.shape == (M, dm.N, dm.N) and xi.shape == (dm.H, dm.B, M)
    assert s0.shape == (dm.B, dm.d_s) and goals.shape == (dm.H, dm.B, dm.d_g)
    P = num_params(dm)
    assert theta.shape == (P,)
    loss = np.zeros(1)
    lpt = np.empty(dm.B)
    states = np.empty((dm.H + 1, dm.B, dm.d_s)) if want_states else None
    g = np.zeros(P) if grad else None
    gs0 = np.zeros((dm.B, dm.d_s)) if grad else None
    rc = lib().oracle_posterior_rollout(C.byref(dm), _p(a["X"]), _p(a["lengthscale"]), _p(a["signal_var"]), _p(alpha),
                                        _p(Kinv), _p(xi), _p(theta), _p(s0), _p(goals), _p(loss), _p(lpt), _p(states),
                                        _p(g), _p(gs0))
    if rc != 0:
        raise RuntimeError(f"oracle_posterior_rollout failed with code {rc}")
    return {"loss": float(loss[0]), "loss_per_traj": lpt, "states": states, "grad_theta": g, "grad_s0": gs0}


# ---------------------------------------------------------------------------------------------
# GP hyper-parameter learning (the step before the rollouts in Algorithm 1: "learn GP transition
# dynamics").  Plain numpy, float64.

def hyper_lml_grad(X, y_m, log_hyp_m):
    """Log marginal likelihood of one output's GP and its gradient (eq. (5), (6); eq. (6) as printed has
    K_hat and its inverse exchanged, the standard form is used):
        lml = -1/2 y^T K_hat^-1 y - 1/2 log|K_hat| - n/2 log(2 pi),
        d lml / d phi = 1/2 tr((a a^T - K_hat^-1) dK_hat/dphi),  a = K_hat^-1 y,
    with the kernel of eq. (4), K_hat = K + sigma_n^2 I, and phi = log_hyp_m = (log l_1 .. log l_D,
    log alpha^2, log sigma_n^2).  Returns (lml, grad[D+2])."""
    X, y_m, lh = _d(X), _d(y_m), _d(log_hyp_m)
    n, D = X.shape
    ell, sf2, sn2 = np.exp(lh[:D]), np.exp(lh[D]), np.exp(lh[D + 1])
    diff2 = ((X[:, None, :] - X[None, :, :]) / ell) ** 2               # [n, n, D]
    K = sf2 * np.exp(-0.5 * diff2.sum(-1))
    Khat = K + sn2 * np.eye(n)
    Lc = np.linalg.cholesky(Khat)
    Kinv = np.linalg.inv(Khat)
    a = Kinv @ y_m
    lml = -0.5 * y_m @ a - np.log(np.diag(Lc)).sum() - 0.5 * n * np.log(2.0 * np.pi)
    W = np.outer(a, a) - Kinv
    grad = np.empty(D + 2)
    for d in range(D):
        grad[d] = 0.5 * np.sum(W * K * diff2[:, :, d])                  # dK/d log l_d = K (x_d - x'_d)^2 / l_d^2
    grad[D] = 0.5 * np.sum(W * K)                                        # dK/d log alpha^2 = K
    grad[D + 1] = 0.5 * sn2 * np.trace(W)                                # dK_hat/d log sigma_n^2 = sigma_n^2 I
    return float(lml), grad


def hyper_fit(X, y, log_hyp0, n_iters: int, *, first_step: int = 1, adam_m=None, adam_v=None, lr=1e-2, beta1=0.9,
              beta2=0.999, eps=1e-8):
    """Adam on -lml / n of every output (hyper-parameters, moments and the Adam constants held in float32
    between iterations, as the device interface holds them; arithmetic in float64).  y[M, n],
    log_hyp0[M, D+2].  Returns (log_hyp, adam_m, adam_v, lml_history[n_iters, M])."""
    X, y = _d(X), _d(y)
    n = X.shape[0]
    lh = np.asarray(log_hyp0, dtype=np.float32).copy()
    am = np.zeros_like(lh) if adam_m is None else np.asarray(adam_m, dtype=np.float32).copy()
    av = np.zeros_like(lh) if adam_v is None else np.asarray(adam_v, dtype=np.float32).copy()
    hp = [float(np.float32(v)) for v in (lr, beta1, beta2, eps)]
    hist = np.empty((n_iters, lh.shape[0]))
    for it in range(n_iters):
        g = np.empty(lh.shape)
        for m in range(lh.shape[0]):
            hist[it, m], gm = hyper_lml_grad(X, y[m], lh[m])
            g[m] = -gm / n
        th, mm, vv = (a.astype(np.float64).ravel().copy() for a in (lh, am, av))
        adam_step(th, g.ravel(), mm, vv, first_step + it, lr=hp[0], beta1=hp[1], beta2=hp[2], eps=hp[3])
        lh, am, av = (a.reshape(lh.shape).astype(np.float32) for a in (th, mm, vv))
    return lh, am, av, hist

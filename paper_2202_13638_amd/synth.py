"""Seeded synthetic workloads shaped like the paper's boom-tracking tasks.

This module only *draws inputs*: training inputs X, training targets y, kernel
hyper-parameters, random-feature frequencies and phases, the standard-normal
weights w and noise draws eps that define each function sample, policy
parameters theta, initial states and goals.  It contains none of the method's
arithmetic (no kernel, no features, no solve, no rollout); both the HIP path
and the CPU oracle are fed from here and nothing else is shared between them.

The paper's data (a hydraulic boom driven by hand for 110 s, Sec. IV-A) is not
public, so every configuration below is a synthetic stand-in with the same
structure: a few states plus one or two actions, hundreds to thousands of
training transitions whose targets are small state increments (the
"discrete difference" targets of Sec. III-A), a goal-conditioned tanh MLP
policy (Sec. IV-B) and hundreds of rollout steps for up to ~10^4 trajectories
(the axes of the scalability study, Sec. IV-C).

All draws use numpy's PCG64 through ``default_rng``; everything is drawn in
float64 and rounded once to float32, which is what both sides consume.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, Optional, Tuple

import numpy as np


@dataclasses.dataclass(frozen=True)
class Config:
    name: str
    index: int
    d_s: int            # states
    d_a: int            # actions
    d_g: int            # tracked states = goal dimension
    N: int              # training points
    L: int              # random Fourier features
    B: int              # trajectories (S = B function samples by default)
    H: int              # horizon
    hidden: Tuple[int, ...]
    act_bound: float    # <= 0: linear policy output; > 0: a = act_bound * tanh(z)
    recipe: str         # "tiny" or "sinusoid"
    goals: str          # "const" or "steps"
    ckpt_interval: int  # 0 = keep the full tape
    signal_var: float
    noise_var: float = 1e-4

    @property
    def D(self) -> int:
        return self.d_s + self.d_a

    @property
    def M(self) -> int:
        return self.d_s

    @property
    def d_in(self) -> int:
        return self.d_s + self.d_g

    @property
    def layer_shapes(self):
        """[(out, in), ...] for every policy layer, input layer first."""
        widths = [self.d_in, *self.hidden, self.d_a]
        return [(widths[i + 1], widths[i]) for i in range(len(widths) - 1)]

    @property
    def P(self) -> int:
        return sum(o * i + o for o, i in self.layer_shapes)

    @property
    def tracked(self) -> Tuple[int, ...]:
        return tuple(range(self.d_g))

    @property
    def q(self) -> Tuple[float, ...]:
        return tuple(1.0 for _ in range(self.d_g))


CONFIGS: Dict[str, Config] = {
    c.name: c
    for c in [
        Config("tiny", 0, 2, 1, 1, 64, 256, 16, 20, (16,), 0.0, "tiny", "const", 0, 1.0),
        Config("small", 1, 4, 1, 1, 512, 1024, 256, 100, (64, 64), 0.0, "sinusoid", "const", 0, 1.0),
        Config("medium", 2, 4, 1, 1, 2048, 2048, 1024, 200, (64, 64), 0.0, "sinusoid", "steps", 0, 1.0),
        Config("large_policy", 3, 4, 1, 1, 4096, 2048, 4096, 500, (256, 256), 0.0, "sinusoid", "steps", 50, 1.0),
        Config("stress", 4, 6, 2, 2, 8192, 4096, 8192, 1000, (256, 256), 1.0, "sinusoid", "steps", 0, 0.01),
        # not one of the five benchmark configurations: the shape of the paper's own Exp. 1 (Sec. IV-A:
        # two states, one bounded action, 2200 training points, 100 trajectories of 300 steps, policy
        # with two hidden layers of 8), on the synthetic recipe, for a timing to set beside the paper's
        Config("paper_exp1", 5, 2, 1, 2, 2200, 1024, 100, 300, (8, 8), 1.0, "sinusoid", "const", 0, 1.0),
    ]
}


def scaled(cfg: Config, **kw) -> Config:
    """A copy of ``cfg`` with some sizes replaced (reduced parity cases)."""
    return dataclasses.replace(cfg, **kw)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64).astype(np.float32))


def _tiny_map(X: np.ndarray) -> np.ndarray:
    # the target map the Tiny configuration states: two states and one action
    return 0.1 * np.sin(3.0 * X[:, 0]) + 0.05 * X[:, 1] * X[:, 2]


def _sinusoid_map(cfg: Config, rng: np.random.Generator):
    """Per output: a restoring term, an actuation term and six small random sinusoids."""
    M, D = cfg.M, cfg.D
    amp = np.zeros((M, 8))
    freq = np.zeros((M, 8, D))
    phs = np.zeros((M, 8))
    for m in range(M):
        amp[m, 0] = 0.1 * 2.0 / math.pi          # -a sin(pi/2 x_m): pulls state m back to 0
        freq[m, 0, m] = math.pi / 2.0
        phs[m, 0] = math.pi
        amp[m, 1] = 0.05 * 2.0 / math.pi         # +a sin(pi/2 u): actuation
        freq[m, 1, cfg.d_s + (m % cfg.d_a)] = math.pi / 2.0
        phs[m, 1] = 0.0
        amp[m, 2:] = rng.uniform(0.0, 0.03 / math.sqrt(6.0), size=6)
        freq[m, 2:, :] = rng.standard_normal((6, D))
        phs[m, 2:] = rng.uniform(0.0, 2.0 * math.pi, size=6)
    return amp, freq, phs


def _eval_sinusoids(X, amp, freq, phs):
    # X [N,D] -> [M,N]
    arg = np.einsum("mjd,nd->mjn", freq, X) + phs[:, :, None]
    return np.einsum("mj,mjn->mn", amp, np.sin(arg))


def make_goals(cfg: Config, rng: np.random.Generator, B: int, H: int) -> np.ndarray:
    """goals[H,B,d_g]: constant per trajectory, or piecewise constant with 4 random steps."""
    if cfg.goals == "const":
        g = rng.uniform(-1.0, 1.0, size=(B, cfg.d_g))
        return np.broadcast_to(g[None], (H, B, cfg.d_g)).copy()
    levels = rng.uniform(-1.0, 1.0, size=(B, 5, cfg.d_g))
    lo, hi = 1, max(2, H)                      # change times ~ U{1..H-1}
    times = np.sort(rng.integers(lo, hi, size=(B, 4)), axis=1)
    t = np.arange(H)[:, None, None]            # [H,1,1]
    seg = (t >= times[None, :, :]).sum(axis=2)  # [H,B] in 0..4
    return np.take_along_axis(levels[None].repeat(H, 0), seg[:, :, None, None], axis=2)[:, :, 0, :]


def make_inputs(cfg: Config, trial: int = 0, S: Optional[int] = None) -> Dict[str, np.ndarray]:
    """Draw every input of one workload.  Returns float32 C-contiguous arrays.

    Keys: X[N,D] y[M,N] lengthscale[M,D] signal_var[M] noise_var[M]
          omega[M,L,D] phase[M,L] w[S,M,L] eps[S,M,N] theta[P]
          s0[B,d_s] goals[H,B,d_g]
    omega is already divided by the lengthscales (it is drawn from the kernel's
    spectral density N(0, diag(1/l^2))), phase ~ U[0, 2pi), w ~ N(0, I),
    eps ~ N(0, noise_var I).
    """
    S = cfg.B if S is None else S
    N, L, D, M, B, H = cfg.N, cfg.L, cfg.D, cfg.M, cfg.B, cfg.H
    root = np.random.default_rng(1000 * cfg.index + trial)
    (r_X, r_map, r_noise, r_ell, r_om, r_ph, r_w, r_eps, r_th, r_s0, r_g) = root.spawn(11)

    X = r_X.uniform(-1.0, 1.0, size=(N, D))
    if cfg.recipe == "tiny":
        # output 0 as stated; output 1 "same recipe, seed+1": same map, fresh noise stream
        clean = np.stack([_tiny_map(X) for _ in range(M)])
        noise = np.stack([np.random.default_rng(1000 * cfg.index + trial + 1 + m)
                          .standard_normal(N) for m in range(M)]) * 0.01
        ell = np.ones((M, D))
    else:
        amp, freq, phs = _sinusoid_map(cfg, r_map)
        clean = _eval_sinusoids(X, amp, freq, phs)
        noise = r_noise.standard_normal((M, N)) * 0.01
        ell = r_ell.uniform(0.5, 2.0, size=(M, D))
    y = clean + noise

    omega = r_om.standard_normal((M, L, D)) / ell[:, None, :]
    phase = r_ph.uniform(0.0, 2.0 * math.pi, size=(M, L))
    w = r_w.standard_normal((S, M, L), dtype=np.float32)
    eps = r_eps.standard_normal((S, M, N), dtype=np.float32) * np.float32(math.sqrt(cfg.noise_var))
    theta = r_th.standard_normal(cfg.P) * 0.1
    s0 = r_s0.uniform(-0.5, 0.5, size=(B, cfg.d_s))
    goals = make_goals(cfg, r_g, B, H)

    return {
        "X": _f32(X), "y": _f32(y), "lengthscale": _f32(ell),
        "signal_var": _f32(np.full(M, cfg.signal_var)), "noise_var": _f32(np.full(M, cfg.noise_var)),
        "omega": _f32(omega), "phase": _f32(phase),
        "w": np.ascontiguousarray(w), "eps": np.ascontiguousarray(eps),
        "theta": _f32(theta), "s0": _f32(s0), "goals": _f32(goals),
    }


def subset_trajectories(cfg: Config, inp: Dict[str, np.ndarray], idx) -> Tuple[Config, Dict[str, np.ndarray]]:
    """Keep only trajectories ``idx`` (and their function samples; requires S == B)."""
    idx = np.asarray(idx)
    out = dict(inp)
    assert inp["w"].shape[0] == inp["s0"].shape[0], "subsetting needs one sample per trajectory"
    for k in ("w", "eps", "s0"):
        out[k] = np.ascontiguousarray(inp[k][idx])
    out["goals"] = np.ascontiguousarray(inp["goals"][:, idx])
    return scaled(cfg, B=len(idx)), out


def make_normal_draws(cfg: Config, trial: int = 0) -> np.ndarray:
    """xi[H, B, M] ~ N(0, 1), float32: the draws of the per-step posterior sampler (its own stream,
    independent of make_inputs)."""
    rng = np.random.default_rng([1000 * cfg.index + trial, 77])
    return rng.standard_normal((cfg.H, cfg.B, cfg.M)).astype(np.float32)

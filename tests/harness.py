"""Shared plumbing of the GPU parity tests: run the oracle and the HIP path on the same seeded
float32 inputs and measure the deviations the way the tolerances are defined.

Tolerances (float32 interface, float64 oracle):
  states   max|delta| / max|s_oracle| over the whole [H+1,B,d_s] tensor   <= 1e-4
  loss     |delta| / |loss|                                               <= 1e-4
  gradient ||delta||_2 / ||g||_2  and  max|delta| / max|g|                <= 1e-3
"""
from __future__ import annotations

import numpy as np

import oracle
from paper_2202_13638_amd import synth

TOL_STATE = 1e-4
TOL_LOSS = 1e-4
TOL_GRAD = 1e-3


def progress(msg):
    """One line on the real stderr (pytest's capture suspended for it), flushed: the long tests say which
    of their steps has finished, so that a run whose output is piped is never silent for minutes."""
    import contextlib
    import sys
    import pytest
    capman = getattr(pytest, "bagel_capture_manager", None)      # set by conftest.py
    cm = capman.global_and_fixture_disabled() if capman is not None else contextlib.nullcontext()
    with cm:
        sys.stderr.write(f"[step] {msg}\n")
        sys.stderr.flush()


def oracle_reference(cfg, inp, S=None, grad=True, chunks=1, **dims_kw):
    """Oracle prepare (float64) -> v rounded once to float32 -> oracle rollout on that v.

    chunks > 1 (needs one sample per trajectory): the rollout is taken in that many consecutive groups of
    trajectories, one oracle call each, and put together here: trajectories are independent and the loss
    is their mean (eq. (10)), so the states and per-trajectory losses are concatenated and the loss and
    its gradients are the means of the groups' weighted by their sizes.  Only the order of the last
    float64 additions differs from a single call."""
    dm = oracle.dims_from_config(cfg, S=S, **dims_kw)
    v64 = oracle.prepare_samples(dm, inp)
    v32 = v64.astype(np.float32)
    progress(f"oracle prepare done ({cfg.name}, N={cfg.N}, S={dm.S})")
    if chunks <= 1:
        out = oracle.rollout(dm, inp, v32, grad=grad)
    else:
        assert S is None or S == cfg.B
        parts, sizes = [], []
        for idx in np.array_split(np.arange(cfg.B), chunks):
            sub_cfg, sub_inp = synth.subset_trajectories(cfg, inp, idx)
            sub_dm = oracle.dims_from_config(sub_cfg, **dims_kw)
            parts.append(oracle.rollout(sub_dm, sub_inp, v32[idx], grad=grad))
            sizes.append(len(idx))
            progress(f"oracle rollout: {sum(sizes)} of {cfg.B} trajectories done")
        wts = np.asarray(sizes, dtype=np.float64) / cfg.B
        out = {"states": np.concatenate([q["states"] for q in parts], axis=1),
               "loss_per_traj": np.concatenate([q["loss_per_traj"] for q in parts]),
               "loss": float(sum(w * q["loss"] for w, q in zip(wts, parts))),
               "grad_theta": None, "grad_s0": None}
        if grad:
            out["grad_theta"] = sum(w * q["grad_theta"] for w, q in zip(wts, parts))
            out["grad_s0"] = np.concatenate([w * q["grad_s0"] for w, q in zip(wts, parts)], axis=0)
    out["v32"] = v32
    out["v64"] = v64
    return out


def to_gpu(inp, keys=None):
    import torch
    return {k: torch.from_numpy(np.ascontiguousarray(a)).cuda() for k, a in inp.items() if keys is None or k in keys}


def gpu_rollout(cfg, inp, v32, S=None, grad=True, with_prepare=False, want_v=False, **dims_kw):
    """Run the HIP path through the C ABI binding; returns numpy arrays."""
    import torch
    from paper_2202_13638_amd import binding
    dims = binding.dims_from_config(cfg, S=S, **dims_kw)
    ctx = binding.Bagel(dims)
    g = to_gpu(inp)
    out = {}
    if with_prepare:
        v_out = torch.empty((dims.S, cfg.M, cfg.N), dtype=torch.float32, device="cuda") if want_v else None
        ctx.bagel_prepare_samples(g["X"], g["y"], g["lengthscale"], g["signal_var"], g["noise_var"], g["omega"],
                                  g["phase"], g["w"], g["eps"], v_out)
        if want_v:
            out["v"] = v_out.cpu().numpy()
    else:
        v = torch.from_numpy(np.ascontiguousarray(v32, dtype=np.float32)).cuda()
        ctx.bagel_set_samples(g["X"], g["lengthscale"], g["signal_var"], g["omega"], g["phase"], g["w"], v)
    B, H, ds = cfg.B, cfg.H, cfg.d_s
    loss = torch.full((1,), float("nan"), device="cuda")
    lpt = torch.full((B,), float("nan"), device="cuda")
    states = torch.full((H + 1, B, ds), float("nan"), device="cuda")
    if grad:
        gth = torch.full((ctx.P,), float("nan"), device="cuda")
        gs0 = torch.full((B, ds), float("nan"), device="cuda")
        ctx.bagel_rollout_loss_grad(g["theta"], g["s0"], g["goals"], loss, gth, lpt, states, gs0)
        torch.cuda.synchronize()
        out.update(grad_theta=gth.cpu().numpy().astype(np.float64), grad_s0=gs0.cpu().numpy().astype(np.float64))
    else:
        ctx.bagel_rollout_loss(g["theta"], g["s0"], g["goals"], loss, lpt, states)
        torch.cuda.synchronize()
    out.update(loss=float(loss.item()), loss_per_traj=lpt.cpu().numpy().astype(np.float64),
               states=states.cpu().numpy().astype(np.float64))
    ctx.close()
    return out


def deviations(ref, got, grad=True):
    d = {
        "state": np.abs(got["states"] - ref["states"]).max() / np.abs(ref["states"]).max(),
        "loss": abs(got["loss"] - ref["loss"]) / abs(ref["loss"]),
        "loss_per_traj": np.abs(got["loss_per_traj"] - ref["loss_per_traj"]).max() / np.abs(ref["loss_per_traj"]).max(),
    }
    if grad:
        g, h = ref["grad_theta"], got["grad_theta"]
        d["grad_l2"] = np.linalg.norm(h - g) / np.linalg.norm(g)
        d["grad_max"] = np.abs(h - g).max() / np.abs(g).max()
        gs, hs = ref["grad_s0"], got["grad_s0"]
        d["grad_s0"] = np.abs(hs - gs).max() / np.abs(gs).max()
    return d


def assert_parity(ref, got, grad=True, label=""):
    d = deviations(ref, got, grad)
    print(f"[parity {label}] " + " ".join(f"{k}={v:.3e}" for k, v in d.items()), flush=True)
    assert np.isfinite(got["states"]).all() and np.isfinite(got["loss"])
    assert d["state"] <= TOL_STATE, d
    assert d["loss"] <= TOL_LOSS, d
    assert d["loss_per_traj"] <= TOL_LOSS, d
    if grad:
        assert np.isfinite(got["grad_theta"]).all()
        assert d["grad_l2"] <= TOL_GRAD and d["grad_max"] <= TOL_GRAD, d
        assert d["grad_s0"] <= TOL_GRAD, d
    return d

"""Conditioning of the rollouts on the five synthetic workloads, measured with the oracle alone (CPU).

For each workload (whole batch on Tiny / Small / Medium, 64 strided trajectories at full N, L, H and
policy on Large policy / Stress) the float64 oracle is run three times:
  base   float32 inputs, v = float64 solve rounded once to float32 (what the parity tests compare with)
  s0+    the same with every initial state moved by one float32 unit in the last place
  v64    the same with v NOT rounded (the unrounded float64 solve of K_hat v = y - Phi w - eps)
and the table gives, relative to max|state| / |loss| / ||grad||:
  cond_s0  how far a 1-ulp change of s0 moves the states           (parity cannot be tighter than this)
  cond_v   how far rounding v to float32 moves states / loss / grad (the distance between a rollout
           driven from any float32 v and the unrounded one: the floor of the prepare -> rollout check)

Run:  python tests/conditioning.py [workload ...]      (prints one markdown table row per workload)
"""
import sys
import os
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2202_13638_amd import synth  # noqa: E402

SUBSET = {"large_policy": 64, "stress": 64}


def measure(name):
    cfg = synth.CONFIGS[name]
    inp = synth.make_inputs(cfg)
    if name in SUBSET:
        n = SUBSET[name]
        idx = np.arange(n) * (cfg.B // n) + 3
        cfg, inp = synth.subset_trajectories(cfg, inp, idx)
    dm = oracle.dims_from_config(cfg)
    v64 = oracle.prepare_samples(dm, inp)
    v32 = v64.astype(np.float32)
    base = oracle.rollout(dm, inp, v32, grad=True)
    moved = dict(inp)
    moved["s0"] = np.nextafter(inp["s0"], np.float32(np.inf), dtype=np.float32)
    s0p = oracle.rollout(dm, moved, v32, grad=True)
    unr = oracle.rollout(dm, inp, v64, grad=True)

    def dev(a, b):
        smax = np.abs(b["states"]).max()
        return (np.abs(a["states"] - b["states"]).max() / smax, abs(a["loss"] - b["loss"]) / abs(b["loss"]),
                np.linalg.norm(a["grad_theta"] - b["grad_theta"]) / np.linalg.norm(b["grad_theta"]))

    d_s0 = dev(s0p, base)
    d_v = dev(base, unr)
    return cfg, np.abs(base["states"]).max(), d_s0, d_v


if __name__ == "__main__":
    names = sys.argv[1:] or ["tiny", "small", "medium", "large_policy", "stress"]
    print("| workload | trajectories | max abs state | cond_s0 state | cond_v state | cond_v loss | cond_v grad |")
    print("|---|---|---|---|---|---|---|")
    for name in names:
        t0 = time.time()
        cfg, smax, d_s0, d_v = measure(name)
        print(f"| {name} | {cfg.B} | {smax:.2f} | {d_s0[0]:.1e} | {d_v[0]:.1e} | {d_v[1]:.1e} | {d_v[2]:.1e} |"
              f"   <!-- {time.time() - t0:.0f} s -->", flush=True)

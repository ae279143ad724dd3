#!/usr/bin/env python3
"""Throughput of the rollout + policy-gradient hot path on one MI355X.

A "step" is one call of bagel_rollout_loss_grad over the whole batch: B trajectories x H rollout
steps forward (policy, sampled GP transition with Jacobian, cost) and the backward sweep to the
policy gradient.  The metric is trajectory-steps per second (forward + backward) on the largest
single-GPU workload ("stress": N=8192, D=8, M=6, L=4096, B=S=8192, H=1000, policy 8-256-256-2).
Inputs are seeded synthetic data (paper_2202_13638_amd/synth.py), resident in HBM before the
timed region; the sample-set precompute (bagel_prepare_samples) runs before it, untimed.

Prints ONE JSON line, with
  value        B*H*steps / wall time of the timed steps (synchronised before and after);
               median_ms_per_call is the median over the same calls, each timed with HIP events on the
               library's stream.
  roofline     the dominant kernel (sample evaluation with Jacobian, one launch per rollout step):
               algorithmic flops per launch / average launch duration measured with HIP events on
               the library's stream during the timed steps, against the float64 vector peak; hbm_frac is
               the algorithmic bytes of the same launch against 8 TB/s; traffic is the counter reading
               stored in profiles/ if that profile was taken from the kernel sources as they are now,
               else null.
  cpu_baseline the float64 oracle timed on this host's cores on a bounded sample of the workload, on all
               threads and on one.
  forward_only, inner_loop   one bagel_rollout_loss call, and two iterations of bagel_optimize (rollout,
               gradient, Adam update), both outside the timed region.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2202_13638_amd import synth  # noqa: E402

PEAK_FP64_VECTOR_TFLOPS = 78.6   # MI355X vector float64 (= unpacked float32) peak
PEAK_HBM_TBS = 8.0
PMC_PROFILE = os.path.join("profiles", "gp_step_stress_pmc.md")
KERNEL_SOURCES = ["gp_step.hip", "model.hip"]    # kernel, its work decomposition and its tables: what fixes the launch the counters were read on


def kernel_source_digest():
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2202_13638_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def measured_traffic(cfg, S, horizon_override):
    """HBM bytes per launch of the sample-evaluation kernel from the rocprofv3 --pmc passes recorded in
    profiles/ (FETCH_SIZE and WRITE_SIZE, scaled by a plain copy of known size) - only if that profile
    names this workload and was taken from the kernel sources as they are now; otherwise None."""
    try:
        text = open(os.path.join(ROOT, PMC_PROFILE)).read()
    except OSError:
        return None
    m = re.search(r"traffic_bytes_per_launch=([0-9.eE+]+)\s+workload=(\w+)\s+S=(\d+)\s+sources=([0-9a-f]+)", text)
    if not m:
        return None
    if m.group(2) != cfg.name or int(m.group(3)) != S or m.group(4) != kernel_source_digest():
        return None
    return float(m.group(1))


def algorithmic_flops_per_traj_step(cfg, jac=True):
    """Sample evaluation only: FMA = 2 flops, each exp / sin / cos = 1 flop."""
    M, N, L, D = cfg.M, cfg.N, cfg.L, cfg.D
    fma = (2 if jac else 1) * M * (N + L) * (D + 1)
    return 2 * fma + M * N + (2 if jac else 1) * M * L


def algorithmic_bytes_per_launch(cfg, S):
    """Sample evaluation: the per-sample streams v and w, read once per launch (4 M (N + L) bytes per
    sample; trajectories that share a sample share its stream)."""
    return 4.0 * cfg.M * (cfg.N + cfg.L) * S


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(cfg, inp, seconds_target=12.0):
    """Time the oracle's loss+gradient on a bounded sample: min(B, 16*cores) trajectories, full N, L,
    policy; horizon chosen so the run takes about `seconds_target`; then once more on ONE thread, on a
    sample sized for about a third of that.  v is a random stand-in of the right scale (the oracle's own
    prepare at N=8192 would take minutes and its values do not change the work)."""
    import ctypes
    import oracle
    cores = oracle.num_threads()
    rng = np.random.default_rng(7)

    def run(Bc, H):
        idx = np.arange(Bc) * (cfg.B // Bc)
        v = (100.0 * rng.standard_normal((Bc, cfg.M, cfg.N))).astype(np.float32)
        sub = synth.scaled(cfg, B=Bc, H=H)
        m = dict(inp)
        m["w"] = np.ascontiguousarray(inp["w"][idx])
        m["s0"] = np.ascontiguousarray(inp["s0"][idx])
        m["goals"] = np.ascontiguousarray(inp["goals"][:H, idx])
        dm = oracle.dims_from_config(sub)
        t0 = time.perf_counter()
        oracle.rollout(dm, m, v, grad=True, want_states=False)
        return time.perf_counter() - t0

    Bc = min(cfg.B, 16 * cores)
    t_probe = run(Bc, 2)
    H = int(max(2, min(cfg.H, round(2 * seconds_target / max(t_probe, 1e-3)))))
    t = run(Bc, H)
    out = {"value": Bc * H / t, "unit": "trajectory-steps/s", "cores": cores, "kind": "oracle",
           "cpu": cpu_model(),
           "sample": f"{Bc} trajectories x {H} steps at full N={cfg.N}, L={cfg.L}, policy {cfg.hidden}; "
                     f"random v of the workload's scale; {t:.1f} s"}
    # one thread: the OpenMP runtime the oracle is linked against takes the thread count
    try:
        gomp = ctypes.CDLL("libgomp.so.1")
        gomp.omp_set_num_threads(1)
        B1 = min(cfg.B, 4)
        t_probe = run(B1, 2)
        H1 = int(max(2, min(cfg.H, round(2 * (seconds_target / 3) / max(t_probe, 1e-3)))))
        t1 = run(B1, H1)
        gomp.omp_set_num_threads(cores)
        out["single_thread"] = {"value": B1 * H1 / t1, "unit": "trajectory-steps/s",
                                "sample": f"{B1} trajectories x {H1} steps; {t1:.1f} s"}
    except OSError:
        out["single_thread"] = None
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="stress", choices=list(synth.CONFIGS))
    ap.add_argument("--sampler", default="pathwise", choices=["pathwise", "posterior"],
                    help="pathwise: one function sample per trajectory (the headline path); posterior: per-step "
                         "draws from the exact predictive posterior (2 N^2 flop per trajectory, step and output)")
    ap.add_argument("--hyper-iters", type=int, default=0,
                    help="also time this many iterations of bagel_hyper_fit (marginal-likelihood learning of the GP "
                         "hyper-parameters) on the workload's training set, outside the timed region")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the forward-only and inner-loop figures")
    ap.add_argument("--profile-every", type=int, default=8, help="time every n-th sample-evaluation launch")
    ap.add_argument("--ckpt", type=int, default=None, help="override ckpt_interval")
    ap.add_argument("--trajectories-per-sample", type=int, default=1,
                    help="supplementary runs: G trajectories share one function sample (S = B / G)")
    ap.add_argument("--horizon", type=int, default=None,
                    help="profiling runs only: shorter horizon (per-launch figures do not depend on it)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="profiling runs only: also run one plain 1 GiB device copy, whose FETCH_SIZE / WRITE_SIZE "
                         "readings calibrate the counters")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)")

    import torch
    from paper_2202_13638_amd import binding

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    cfg = synth.CONFIGS[args.workload]
    if args.horizon is not None:
        cfg = synth.scaled(cfg, H=args.horizon)
    t0 = time.perf_counter()
    S = cfg.B // args.trajectories_per_sample
    inp = synth.make_inputs(cfg, S=S)
    t_gen = time.perf_counter() - t0

    kw = {} if args.ckpt is None else {"ckpt_interval": args.ckpt}
    dims = binding.dims_from_config(cfg, S=S, **kw)
    ctx = binding.Bagel(dims)
    g = {k: torch.from_numpy(a).cuda() for k, a in inp.items()}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    posterior = args.sampler == "posterior"
    if posterior:
        ctx.bagel_prepare_posterior(g["X"], g["y"], g["lengthscale"], g["signal_var"], g["noise_var"])
        g["xi"] = torch.from_numpy(synth.make_normal_draws(cfg)).cuda()
    else:
        ctx.bagel_prepare_samples(g["X"], g["y"], g["lengthscale"], g["signal_var"], g["noise_var"], g["omega"],
                                  g["phase"], g["w"], g["eps"], None)
    torch.cuda.synchronize()
    t_prep = time.perf_counter() - t0
    for k in ("w", "eps", "y"):
        del g[k]
    torch.cuda.empty_cache()

    loss = torch.zeros(1, device="cuda")
    grad = torch.zeros(ctx.P, device="cuda")
    if args.pmc_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")      # 1 GiB
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    def step():
        if posterior:
            ctx.bagel_posterior_rollout_loss_grad(g["theta"], g["s0"], g["goals"], g["xi"], loss, grad)
        else:
            ctx.bagel_rollout_loss_grad(g["theta"], g["s0"], g["goals"], loss, grad)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ctx.bagel_profile_enable(args.profile_every)
    # every call between two events on the stream the library launches on (torch's current stream)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    ev[0].record()
    for i in range(args.steps):
        step()
        ev[i + 1].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    call_ms = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(args.steps))
    median_ms = call_ms[len(call_ms) // 2] if len(call_ms) % 2 else 0.5 * (call_ms[len(call_ms) // 2 - 1] + call_ms[len(call_ms) // 2])
    k_ms, k_n = ctx.bagel_profile_read()
    ctx.bagel_profile_enable(0)
    if not os.environ.get("BAGEL_BENCH_TIMING_ONLY"):      # timing experiments with deliberately wrong operands
        assert np.isfinite(loss.item()) and bool(torch.isfinite(grad).all())

    traj_steps = cfg.B * cfg.H
    value = traj_steps * args.steps / elapsed
    ckpt = dims.ckpt_interval if 0 < dims.ckpt_interval < cfg.H else 0
    if posterior:
        # per step: the float64 GEMM with K_hat^-1 (2 N^2 flop per trajectory and output) plus kernel rows and
        # the moment / derivative sums (about 2 N (3 D + 8))
        flops_launch = cfg.M * cfg.B * (2 * cfg.N * cfg.N + 2 * cfg.N * (3 * cfg.D + 8))
    else:
        flops_launch = algorithmic_flops_per_traj_step(cfg, jac=True) * cfg.B
    avg_ms = k_ms / max(k_n, 1)
    achieved = flops_launch / (avg_ms * 1e-3) / 1e12 if k_n else float("nan")
    out = {
        "metric": "trajectory-steps/sec (fwd+bwd)",
        "value": value,
        "unit": "trajectory-steps/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": 1e3 * elapsed / args.steps,
        "median_ms_per_call": median_ms,
        "min_ms_per_call": call_ms[0],
        "max_ms_per_call": call_ms[-1],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f64",
        "data": "synthetic",
        "config": {"workload": cfg.name, "sampler": args.sampler, "N": cfg.N, "D": cfg.D, "M": cfg.M, "L": cfg.L, "B": cfg.B, "S": S,
                   "H": cfg.H, "policy": [cfg.d_in, *cfg.hidden, cfg.d_a], "ckpt_interval": ckpt,
                   "arithmetic": "kernel row and feature phase in f64, policy and sin/cos in f32, f32 interface",
                   "prepare_s": round(t_prep, 3), "input_generation_s": round(t_gen, 1),
                   "workspace_GB": round(ctx.workspace_bytes() / 1e9, 2)},
        "roofline": {"bound": "alu", "kernel": "posterior step: rows + dgemm_kernel + reduce, all outputs" if posterior
                     else "gp_step_kernel<D,jac>", "achieved": achieved,
                     "peak": PEAK_FP64_VECTOR_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_FP64_VECTOR_TFLOPS,
                     "traffic": None if posterior else measured_traffic(cfg, S, args.horizon),
                     "traffic_source": PMC_PROFILE,
                     "hbm_frac": None if posterior else
                     algorithmic_bytes_per_launch(cfg, S) / (avg_ms * 1e-3) / (PEAK_HBM_TBS * 1e12) if k_n else None,
                     "algorithmic_bytes_per_launch": None if posterior else algorithmic_bytes_per_launch(cfg, S),
                     "avg_launch_ms": avg_ms, "timed_launches": k_n,
                     "flops_per_launch": flops_launch,
                     "share_of_step": (avg_ms * cfg.H) / (1e3 * elapsed / args.steps)},
    }
    r = out["roofline"]
    # the kernel's lower bound is the larger of its arithmetic time and its streaming time
    r["frac_of_max_bound"] = None if r["hbm_frac"] is None else max(r["frac"], r["hbm_frac"])
    if not args.no_extras and not posterior:
        # reported alongside, outside the timed region: the forward pass alone, and the inner loop of
        # Algorithm 1 (rollout, gradient, Adam update per iteration) on fixed initial states and goals
        def timed(fn):
            torch.cuda.synchronize()
            t = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            return time.perf_counter() - t
        t_fwd = timed(lambda: ctx.bagel_rollout_loss(g["theta"], g["s0"], g["goals"], loss))
        out["forward_only"] = {"value": traj_steps / t_fwd, "unit": "trajectory-steps/s", "ms_per_call": 1e3 * t_fwd}
        n_it = 2
        theta = g["theta"].clone()
        am, av = torch.zeros_like(theta), torch.zeros_like(theta)
        hist = torch.zeros(n_it, device="cuda")
        t_opt = timed(lambda: ctx.bagel_optimize(theta, am, av, g["s0"][None], g["goals"][None], n_it, hist))
        out["inner_loop"] = {"value": traj_steps * n_it / t_opt, "unit": "trajectory-steps/s", "iterations": n_it,
                             "ms_per_iteration": 1e3 * t_opt / n_it, "loss": [float(x) for x in hist.cpu()]}
    if args.hyper_iters > 0:
        lh = torch.cat([g["lengthscale"].log(), g["signal_var"].log()[:, None], g["noise_var"].log()[:, None]], dim=1).contiguous()
        am, av = torch.zeros_like(lh), torch.zeros_like(lh)
        hist = torch.zeros((args.hyper_iters, cfg.M), device="cuda")
        yy = torch.from_numpy(inp["y"]).cuda()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ctx.bagel_hyper_fit(g["X"], yy, lh, am, av, args.hyper_iters, hist)
        torch.cuda.synchronize()
        t_h = time.perf_counter() - t0
        Np = (cfg.N + 63) // 64 * 64
        # algorithmic work per output: Cholesky, inverse of the triangular factor and the symmetric product
        # Z^T Z, Np^3/6 FMA each (the library's structured substitution spends Np^3/4 on the middle one)
        flop = 2.0 * cfg.M * args.hyper_iters * (float(Np) ** 3 / 2)
        out["hyper_fit"] = {"iterations": args.hyper_iters, "ms_per_iteration": 1e3 * t_h / args.hyper_iters,
                            "TFLOP/s": flop / t_h / 1e12, "frac_of_f64_peak": flop / t_h / 1e12 / PEAK_FP64_VECTOR_TFLOPS,
                            "lml_first": [float(x) for x in hist[0].cpu()], "lml_last": [float(x) for x in hist[-1].cpu()]}
    if not args.no_cpu_baseline and args.trajectories_per_sample == 1 and not posterior:
        out["cpu_baseline"] = cpu_baseline(cfg, inp)
    ctx.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()

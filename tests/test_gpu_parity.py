"""GPU parity: the HIP path (through the C ABI) against the float64 CPU oracle on identical
seeded float32 inputs.  Tolerances are defined in tests/harness.py.

Rollout parity is driven from exactly the float32 representer weights v the oracle used
(oracle prepare in float64 -> rounded once -> bagel_set_samples), because v is an ill-conditioned
intermediate: rounding it to float32 differently already moves a rollout by more than the
tolerance.  bagel_prepare_samples is checked on its own against the oracle's float64 v."""
import numpy as np
import pytest

import harness
import oracle
from paper_2202_13638_amd import synth

pytestmark = pytest.mark.gpu


def _cfg(name, **kw):
    return synth.scaled(synth.CONFIGS[name], **kw) if kw else synth.CONFIGS[name]


# ------------------------------------------------------------------ the five configurations
@pytest.mark.parametrize("name", ["tiny", "small"])
def test_full_config_forward_and_gradient(name):
    cfg = _cfg(name)
    inp = synth.make_inputs(cfg)
    ref = harness.oracle_reference(cfg, inp)
    harness.assert_parity(ref, harness.gpu_rollout(cfg, inp, ref["v32"], grad=False), grad=False, label=f"{name}/fwd")
    harness.assert_parity(ref, harness.gpu_rollout(cfg, inp, ref["v32"], grad=True), label=f"{name}/grad")


@pytest.mark.timeout(600)
def test_medium_full_config():
    cfg = _cfg("medium")
    inp = synth.make_inputs(cfg)
    ref = harness.oracle_reference(cfg, inp)
    harness.assert_parity(ref, harness.gpu_rollout(cfg, inp, ref["v32"]), label="medium/grad")


N_SAMPLED = 256     # trajectories the oracle follows inside the two largest workloads


def _sampled_indices(cfg):
    """Strided sample of N_SAMPLED trajectories: every (B / N_SAMPLED)-th one, starting at 3."""
    return np.arange(N_SAMPLED) * (cfg.B // N_SAMPLED) + 3


def _run_full_batch(cfg, inp, v_rows=None, idx=None):
    """The configuration at its full sizes through bagel_prepare_samples (the library's own v for
    every sample; rows `idx` replaced by `v_rows`, the float32 v the oracle used) and one
    bagel_rollout_loss_grad call in the launch configuration bench.py times.  Returns numpy results and
    the library's v of the rows idx."""
    import torch
    from paper_2202_13638_amd import binding
    ctx = binding.Bagel(binding.dims_from_config(cfg))
    g = harness.to_gpu(inp)
    v_all = torch.empty((cfg.B, cfg.M, cfg.N), dtype=torch.float32, device="cuda")
    ctx.bagel_prepare_samples(g["X"], g["y"], g["lengthscale"], g["signal_var"], g["noise_var"], g["omega"],
                              g["phase"], g["w"], g["eps"], v_all)
    torch.cuda.synchronize()
    v_lib = None
    if idx is not None:
        ti = torch.from_numpy(idx).cuda()
        v_lib = v_all[ti].cpu().numpy().astype(np.float64)
        v_all[ti] = torch.from_numpy(np.ascontiguousarray(v_rows, dtype=np.float32)).cuda()
    ctx.bagel_set_samples(g["X"], g["lengthscale"], g["signal_var"], g["omega"], g["phase"], g["w"], v_all)
    B, H, ds = cfg.B, cfg.H, cfg.d_s
    loss = torch.full((1,), float("nan"), device="cuda")
    lpt = torch.full((B,), float("nan"), device="cuda")
    states = torch.full((H + 1, B, ds), float("nan"), device="cuda")
    gth = torch.full((ctx.P,), float("nan"), device="cuda")
    gs0 = torch.full((B, ds), float("nan"), device="cuda")
    ctx.bagel_rollout_loss_grad(g["theta"], g["s0"], g["goals"], loss, gth, lpt, states, gs0)
    torch.cuda.synchronize()
    out = dict(loss=float(loss.item()), loss_per_traj=lpt.cpu().numpy().astype(np.float64),
               states=states.cpu().numpy().astype(np.float64), grad_theta=gth.cpu().numpy().astype(np.float64),
               grad_s0=gs0.cpu().numpy().astype(np.float64))
    ctx.close()
    return out, v_lib, v_all


def _check_sampled_inside_full(name, cfg, full, ref, alone, idx):
    """The sampled trajectories inside the full batch against the oracle: states, per-trajectory loss and
    d loss / d s0 (a per-trajectory quantity that exercises the whole backward sweep)."""
    st = full["states"][:, idx]
    d_state = np.abs(st - ref["states"]).max() / np.abs(ref["states"]).max()
    d_lpt = np.abs(full["loss_per_traj"][idx] - ref["loss_per_traj"]).max() / np.abs(ref["loss_per_traj"]).max()
    gs = full["grad_s0"][idx] * (cfg.B / len(idx))                         # 1/B normalisation of the loss
    d_gs0 = np.abs(gs - ref["grad_s0"]).max() / np.abs(ref["grad_s0"]).max()
    print(f"[parity {name}/sampled inside the full batch] state={d_state:.3e} loss_per_traj={d_lpt:.3e} "
          f"grad_s0={d_gs0:.3e}", flush=True)
    assert d_state <= harness.TOL_STATE and d_lpt <= harness.TOL_LOSS and d_gs0 <= harness.TOL_GRAD
    # the same trajectories give (up to the summation order of a different work split) the same numbers
    # whether they run alone or inside the full batch
    np.testing.assert_allclose(st, alone["states"], rtol=0, atol=2e-5 * np.abs(alone["states"]).max())


@pytest.mark.timeout(1500)
def test_large_policy_full_batch_against_the_oracle():
    """N=4096, L=2048, B=S=4096, H=500, policy 5-256-256-1, ckpt_interval=50: the whole batch through
    the oracle (prepare in float64, v rounded once, rollout and gradient of all 4096 trajectories) and
    through bagel_set_samples + bagel_rollout_loss_grad at full size: loss, every state, every
    per-trajectory loss, grad_theta and grad_s0.  Then the library's own prepare at full size against the
    oracle's float64 v, and checkpointing against the full tape on a sampled batch."""
    cfg = _cfg("large_policy")
    inp = synth.make_inputs(cfg)
    ref = harness.oracle_reference(cfg, inp, chunks=8)
    got = harness.gpu_rollout(cfg, inp, ref["v32"])
    harness.assert_parity(ref, got, label="large_policy/full batch")
    harness.progress("large_policy: full batch compared with the oracle")
    _, v_lib, v_all = _run_full_batch(cfg, inp, ref["v32"][:8], np.arange(8))
    del v_all
    err = np.abs(v_lib - ref["v64"][:8]).max() / np.abs(ref["v64"]).max()
    print(f"[prepare large_policy full size] max|dv|/max|v| = {err:.3e}", flush=True)
    assert err <= 5e-7
    # a sampled batch with and without checkpointing: identical states, same gradient
    idx = _sampled_indices(cfg)[:64]
    sub_cfg, sub_inp = synth.subset_trajectories(cfg, inp, idx)
    ck = harness.gpu_rollout(sub_cfg, sub_inp, ref["v32"][idx])
    plain = harness.gpu_rollout(sub_cfg, sub_inp, ref["v32"][idx], ckpt_interval=0)
    np.testing.assert_array_equal(plain["states"], ck["states"])
    np.testing.assert_allclose(plain["grad_theta"], ck["grad_theta"], rtol=1e-5,
                               atol=1e-6 * np.abs(ck["grad_theta"]).max())


@pytest.mark.timeout(1500)
def test_stress_full_size():
    """N=8192, D=8, M=6, L=4096, B=S=8192, H=1000, policy 8-256-256-2 with bounded actions: the workload
    bench.py times.  The oracle cannot afford the whole batch (8.2e6 trajectory-steps), so:
      (a) 256 strided trajectories as a batch of their own (S = B = 256, full N, L, H, policy) against the
          oracle: everything, grad_theta included;
      (b) the same 256 inside the full batch: states, per-trajectory losses, d loss / d s0 against the oracle;
      (c) loss and grad_theta of the full batch against the 32 disjoint 256-trajectory sub-batches it is
          made of, each run on its own (same v): the mean of the sub-batch losses and gradients must give
          the full-batch values to summation-order accuracy, and one of the 32 is the oracle-checked
          batch of (a).  Trajectories are independent (eq. (10): the loss is a mean over them), so (a) and
          (c) together tie the full-batch loss and gradient to the oracle."""
    import torch
    name = "stress"
    cfg = _cfg(name)
    inp = synth.make_inputs(cfg)
    stride = cfg.B // N_SAMPLED
    idx = _sampled_indices(cfg)
    sub_cfg, sub_inp = synth.subset_trajectories(cfg, inp, idx)
    ref = harness.oracle_reference(sub_cfg, sub_inp)                      # oracle prepare + rollout on the sample
    alone = harness.gpu_rollout(sub_cfg, sub_inp, ref["v32"])
    harness.assert_parity(ref, alone, label=f"{name}/sampled batch of {N_SAMPLED}")
    harness.progress("stress: sampled batch compared with the oracle")

    full, v_lib, v_all = _run_full_batch(cfg, inp, ref["v32"], idx)
    harness.progress("stress: full batch done on the GPU")
    err = np.abs(v_lib - ref["v64"]).max() / np.abs(ref["v64"]).max()
    print(f"[prepare {name} full size] max|dv|/max|v| on the sampled rows = {err:.3e}", flush=True)
    assert err <= 5e-7
    _check_sampled_inside_full(name, cfg, full, ref, alone, idx)
    assert np.isfinite(full["grad_theta"]).all() and np.isfinite(full["states"]).all()
    assert abs(full["loss"] - full["loss_per_traj"].mean()) <= 1e-5 * abs(full["loss"])

    # (c) the 32 disjoint sub-batches {k, k + 32, k + 64, ...}; k = 3 is the oracle-checked one
    loss_sum, grad_sum = 0.0, np.zeros_like(full["grad_theta"])
    for k in range(stride):
        idx_k = np.arange(N_SAMPLED) * stride + k
        cfg_k, inp_k = synth.subset_trajectories(cfg, inp, idx_k)
        v_k = v_all[torch.from_numpy(idx_k).cuda()].cpu().numpy()
        part = harness.gpu_rollout(cfg_k, inp_k, v_k)
        if k == 3:
            np.testing.assert_array_equal(part["states"], alone["states"])
            np.testing.assert_array_equal(part["grad_theta"], alone["grad_theta"])
        loss_sum += part["loss"]
        grad_sum += part["grad_theta"]
        np.testing.assert_allclose(part["loss_per_traj"], full["loss_per_traj"][idx_k], rtol=0,
                                   atol=1e-5 * np.abs(full["loss_per_traj"]).max())
        if k % 8 == 7:
            harness.progress(f"stress: {k + 1} of {stride} sub-batches done")
    del v_all
    d_loss = abs(loss_sum / stride - full["loss"]) / abs(full["loss"])
    d_grad = np.abs(grad_sum / stride - full["grad_theta"]).max() / np.abs(full["grad_theta"]).max()
    d_grad_l2 = np.linalg.norm(grad_sum / stride - full["grad_theta"]) / np.linalg.norm(full["grad_theta"])
    print(f"[stress full batch vs its 32 sub-batches] loss={d_loss:.3e} grad_max={d_grad:.3e} grad_l2={d_grad_l2:.3e}",
          flush=True)
    assert d_loss <= 1e-5 and d_grad <= 1e-5 and d_grad_l2 <= 1e-5


# ------------------------------------------------------------------ one evaluation of the samples
@pytest.mark.parametrize("shape", [
    dict(d_s=2, d_a=1, N=64, L=256, B=16, S=16),
    dict(d_s=3, d_a=2, N=50, L=70, B=37, S=37),          # ragged N, L, B
    dict(d_s=6, d_a=2, N=300, L=200, B=130, S=13),       # shared samples, D = 8
    dict(d_s=8, d_a=8, N=33, L=45, B=5, S=5),            # largest input dimension
])
def test_sample_eval_value_and_jacobian(shape):
    x = np.random.default_rng(3).uniform(-1.2, 1.2, (shape["B"], shape["d_s"] + shape["d_a"])).astype(np.float32)
    _check_sample_eval(shape, x)


# the library picks the form of its float64 exp2 by launch size (polynomial on small launches, table
# look-up on large ones); BAGEL_EXP_TABLE = 1 / 2 forces one, so that both are checked at test sizes
EXP2_FORMS = {"polynomial": "1", "table": "2"}


@pytest.mark.parametrize("form", list(EXP2_FORMS))
def test_sample_eval_with_either_exp2(form, monkeypatch):
    monkeypatch.setenv("BAGEL_EXP_TABLE", EXP2_FORMS[form])
    shape = dict(d_s=6, d_a=2, N=300, L=200, B=130, S=13)
    x = np.random.default_rng(5).uniform(-1.2, 1.2, (shape["B"], 8)).astype(np.float32)
    _check_sample_eval(shape, x)


@pytest.mark.parametrize("D", range(2, 17))
def test_sample_eval_every_input_dimension(D, monkeypatch):
    """The step kernel is compiled once per GP input dimension: every one of them, in both exp2 forms,
    with ragged N, L and B and with samples shared by several trajectories on the even dimensions."""
    d_s = (D + 1) // 2
    for form, flag in EXP2_FORMS.items():
        monkeypatch.setenv("BAGEL_EXP_TABLE", flag)
        B = 64 + 3 * D
        shape = dict(d_s=d_s, d_a=D - d_s, N=40 + 7 * D, L=30 + 9 * D, B=B, S=B // 2 if B % 2 == 0 else B)
        x = np.random.default_rng(40 + D).uniform(-1.2, 1.2, (B, D)).astype(np.float32)
        harness.progress(f"sample evaluation D={D} {form} {shape}")
        _check_sample_eval(shape, x)


@pytest.mark.parametrize("form", list(EXP2_FORMS))
def test_sample_eval_inputs_far_from_the_data(form, monkeypatch):
    """GP inputs hundreds of length scales away from every training point: the kernel row is zero
    there (the step kernel flushes it beyond about 400 length scales), the feature part is not."""
    monkeypatch.setenv("BAGEL_EXP_TABLE", EXP2_FORMS[form])
    shape = dict(d_s=3, d_a=2, N=50, L=70, B=37, S=37)
    x = np.random.default_rng(4).uniform(-1.2, 1.2, (shape["B"], 5)).astype(np.float32)
    x[3] = 150.0                       # 80 to 170 length scales out (the recipe draws them from 0.5 ... 2)
    x[4] *= 400.0
    x[5] = -2500.0                     # beyond the kernel's range
    x[6, 2] = 1.0e4
    _check_sample_eval(shape, x)


def _check_sample_eval(shape, x):
    import torch
    from paper_2202_13638_amd import binding
    cfg = synth.Config("e", 11, shape["d_s"], shape["d_a"], 1, shape["N"], shape["L"], shape["B"], 2, (4,), 0.0,
                       "sinusoid", "const", 0, 0.7, 1e-3)
    inp = synth.make_inputs(cfg, S=shape["S"])
    dm = oracle.dims_from_config(cfg, S=shape["S"])
    v32 = oracle.prepare_samples(dm, inp).astype(np.float32)
    ctx = binding.Bagel(binding.dims_from_config(cfg, S=shape["S"]))
    g = harness.to_gpu(inp)
    ctx.bagel_set_samples(g["X"], g["lengthscale"], g["signal_var"], g["omega"], g["phase"], g["w"],
                          torch.from_numpy(v32).cuda())
    f = torch.empty((cfg.B, cfg.M), device="cuda")
    J = torch.empty((cfg.B, cfg.M, cfg.D), device="cuda")
    f_only = torch.empty((cfg.B, cfg.M), device="cuda")
    ctx.bagel_sample_eval(torch.from_numpy(x).cuda(), f, J)
    ctx.bagel_sample_eval(torch.from_numpy(x).cuda(), f_only, None)
    torch.cuda.synchronize()
    f, J, f_only = f.cpu().numpy(), J.cpu().numpy(), f_only.cpu().numpy()
    per = cfg.B // shape["S"]
    fr = np.zeros((cfg.B, cfg.M)); Jr = np.zeros((cfg.B, cfg.M, cfg.D))
    for b in range(cfg.B):
        fr[b], Jr[b] = oracle.sample_eval(dm, inp, inp["w"][b // per], v32[b // per], x[b])
    assert np.abs(f - fr).max() <= 2e-6 * max(1.0, np.abs(fr).max())
    assert np.abs(J - Jr).max() <= 1e-5 * max(1.0, np.abs(Jr).max())
    np.testing.assert_array_equal(f, f_only)      # the value does not depend on asking for the Jacobian


# ------------------------------------------------------------------ variants of the rollout
VARIANTS = {
    "bounded-two-tracked": dict(cfg=dict(d_s=3, d_a=2, d_g=2, hidden=(12, 7), act_bound=1.5, B=70, H=9), dims=dict()),
    "shared-samples": dict(cfg=dict(B=96, H=12), S=8, dims=dict()),
    "saturating-reward": dict(cfg=dict(B=33, H=10, act_bound=1.0), dims=dict(cost_kind=1, sigma_r=0.6)),
    "one-step-one-trajectory": dict(cfg=dict(B=1, H=1), dims=dict()),
    # the smallest model and the smallest policy: everything beyond them is padding inside the kernels
    "one-training-point-one-feature": dict(cfg=dict(N=1, L=1, B=16, H=8), dims=dict()),
    "hidden-layers-of-one-unit": dict(cfg=dict(hidden=(1, 1), B=40, H=6), dims=dict()),
    "one-sample-for-all-trajectories": dict(cfg=dict(B=70, H=9), S=1, dims=dict()),
    "checkpoint-ragged": dict(cfg=dict(B=20, H=23), dims=dict(ckpt_interval=5)),
    "wide-policy": dict(cfg=dict(B=65, H=6, hidden=(256, 256)), dims=dict()),
    # B a multiple of 32 and a layer with more than 128 rows and columns: the LDS-tiled weight gradient,
    # with full (256 x 256) and ragged (136 x 200) operand rows, several tiles per workgroup
    "wide-policy-tiled": dict(cfg=dict(B=96, H=7, hidden=(256, 256)), dims=dict()),
    "wide-policy-tiled-ragged": dict(cfg=dict(B=64, H=5, hidden=(200, 136)), dims=dict()),
    "wide-policy-tiled-one-split": dict(cfg=dict(B=160, H=6, hidden=(256, 256)), dims=dict(), env=dict(BAGEL_KSPLIT="4")),
}


@pytest.mark.parametrize("name", list(VARIANTS))
def test_rollout_variants(name, monkeypatch):
    spec = VARIANTS[name]
    for k, v in spec.get("env", {}).items():
        monkeypatch.setenv(k, v)
    base = dict(d_s=2, d_a=1, d_g=1, N=90, L=130, B=16, H=8, hidden=(16,), act_bound=0.0)
    base.update(spec["cfg"])
    cfg = synth.Config("v", 12, base["d_s"], base["d_a"], base["d_g"], base["N"], base["L"], base["B"], base["H"],
                       tuple(base["hidden"]), base["act_bound"], "sinusoid", "steps", 0, 0.5, 1e-3)
    S = spec.get("S")
    inp = synth.make_inputs(cfg, S=S)
    inp["theta"] = (inp["theta"] * 3).astype(np.float32)
    okw = {k: v for k, v in spec["dims"].items() if k != "ckpt_interval"}
    ref = harness.oracle_reference(cfg, inp, S=S, **okw)
    got = harness.gpu_rollout(cfg, inp, ref["v32"], S=S, **spec["dims"])
    harness.assert_parity(ref, got, label=name)
    fwd = harness.gpu_rollout(cfg, inp, ref["v32"], S=S, grad=False, **spec["dims"])
    np.testing.assert_array_equal(fwd["states"], got["states"])
    assert fwd["loss"] == got["loss"]


SWEEP_HIDDEN = [(8,), (33,), (64, 64), (96, 40), (128, 128), (130, 200), (200, 136), (256, 32), (32, 256), (256, 256),
                (255, 129), (160,), (256,)]
SWEEP_STATE = [dict(d_s=2, d_a=1, d_g=1), dict(d_s=6, d_a=2, d_g=2), dict(d_s=8, d_a=8, d_g=8), dict(d_s=3, d_a=1, d_g=2)]


@pytest.mark.parametrize("hi", range(len(SWEEP_HIDDEN)))
def test_policy_and_state_shape_sweep(hi, monkeypatch):
    """Every hidden-layer shape (one or two layers; widths below, at and between the tile sizes of the
    policy kernels) against every state/action/goal shape, with batch size, horizon, checkpointing,
    action bound, cost kind and the contraction split of narrow layers rotating through the cases.
    Some of these small random systems are chaotic over their few steps, so each case is held to the
    tolerance plus twenty times its own conditioning figure: the deviation of the oracle from itself when
    s0 moves by one unit in the last place of float32."""
    hidden = SWEEP_HIDDEN[hi]
    for si, sh in enumerate(SWEEP_STATE):
        B = [32, 64, 96, 70, 160][(hi + si) % 5]
        H = [5, 7, 6, 9][(hi + 2 * si) % 4]
        ck = [0, 3][(hi + si) % 2]
        bound = [0.0, 1.2][(hi // 2 + si) % 2]
        split = ["256", "3"][(hi + si // 2) % 2]
        monkeypatch.setenv("BAGEL_KSPLIT", split)
        cfg = synth.Config("sweep", 20 + hi, sh["d_s"], sh["d_a"], sh["d_g"], 90, 130, B, H, tuple(hidden), bound,
                           "sinusoid", "steps", 0, 0.5, 1e-3)
        inp = synth.make_inputs(cfg, trial=si)
        # an 8-dimensional action fed back through 8 states diverges within the horizon at the larger scale
        inp["theta"] = (inp["theta"] * (0.3 if sh["d_s"] == 8 else 2)).astype(np.float32)
        dims = dict(cost_kind=1, sigma_r=0.7) if (hi + si) % 3 == 0 else {}
        label = f"hidden{hidden}/ds{sh['d_s']}da{sh['d_a']}dg{sh['d_g']}/B{B}/H{H}/ckpt{ck}/bound{bound}/split{split}"
        harness.progress(f"sweep case {label}")
        ref = harness.oracle_reference(cfg, inp, **dims)
        got = harness.gpu_rollout(cfg, inp, ref["v32"], ckpt_interval=ck, **dims)
        moved = dict(inp)
        moved["s0"] = np.nextafter(inp["s0"], np.float32(np.inf), dtype=np.float32)
        cond = harness.deviations(ref, oracle.rollout(oracle.dims_from_config(cfg, **dims), moved, ref["v32"]))
        d = harness.deviations(ref, got)
        print(f"[parity {label}] " + " ".join(f"{k}={d[k]:.1e} (cond {cond[k]:.1e})" for k in d), flush=True)
        assert np.isfinite(got["states"]).all() and np.isfinite(got["grad_theta"]).all()
        for k in d:
            tol = harness.TOL_GRAD if k.startswith("grad") else (harness.TOL_STATE if k == "state" else harness.TOL_LOSS)
            assert d[k] <= tol + 20 * cond[k], (label, k, d[k], cond[k])


def test_rollout_with_table_exp2(monkeypatch):
    """The exp2 form of large launches, forced at a size the oracle finishes in seconds."""
    monkeypatch.setenv("BAGEL_EXP_TABLE", EXP2_FORMS["table"])
    cfg = _cfg("small", B=96, H=30)
    inp = synth.make_inputs(cfg)
    ref = harness.oracle_reference(cfg, inp)
    got = harness.gpu_rollout(cfg, inp, ref["v32"])
    harness.assert_parity(ref, got, label="small/B96/H30/table")


@pytest.mark.parametrize("trial", [1, 2, 3])
def test_other_draws_sizes_exp2_forms_and_checkpointing(trial, monkeypatch):
    """Further draws of the Small workload's inputs at three sizes (tile multiples and ragged N, L, B),
    each in both exp2 forms, with the full tape and with a checkpoint interval that does not divide H."""
    import dataclasses
    for form, flag in EXP2_FORMS.items():
        monkeypatch.setenv("BAGEL_EXP_TABLE", flag)
        for B, H, N, L in [(96, 25, 512, 1024), (70, 18, 333, 517), (130, 12, 200, 90)]:
            cfg = dataclasses.replace(synth.CONFIGS["small"], B=B, H=H, N=N, L=L)
            inp = synth.make_inputs(cfg, trial=trial)
            ref = harness.oracle_reference(cfg, inp)
            for ck in (0, 7):
                got = harness.gpu_rollout(cfg, inp, ref["v32"], ckpt_interval=ck)
                harness.assert_parity(ref, got, label=f"trial{trial}/{form}/ckpt{ck}/B{B}/H{H}/N{N}/L{L}")


def test_checkpointing_does_not_change_the_result():
    cfg = _cfg("small", B=64, H=40)
    inp = synth.make_inputs(cfg)
    ref = harness.oracle_reference(cfg, inp)
    plain = harness.gpu_rollout(cfg, inp, ref["v32"], ckpt_interval=0)
    for K in (1, 7, 8, 39, 40, 100):
        ck = harness.gpu_rollout(cfg, inp, ref["v32"], ckpt_interval=K)
        np.testing.assert_array_equal(ck["states"], plain["states"])
        assert ck["loss"] == plain["loss"]
        np.testing.assert_array_equal(ck["grad_s0"], plain["grad_s0"])
        np.testing.assert_allclose(ck["grad_theta"], plain["grad_theta"], rtol=2e-5,
                                   atol=2e-6 * np.abs(plain["grad_theta"]).max())
    harness.assert_parity(ref, plain, label="small/B64/H40")


@pytest.mark.parametrize("name,ckpt", [("tiny", 0), ("small", 0), ("small", 7)])
def test_gradient_call_captured_into_a_hip_graph(name, ckpt):
    """The rollout calls enqueue kernels only (no allocation, no memset, no host synchronisation), so a
    caller may capture one into a HIP graph.  Every replay, with eager calls and synchronisations between
    them, must reproduce the eager result bit for bit.  With checkpointing the backward pass forks onto the
    context's second stream and joins again, inside the capture."""
    import torch
    from paper_2202_13638_amd import binding
    cfg = _cfg(name)
    inp = synth.make_inputs(cfg)
    g = harness.to_gpu(inp)
    stream = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(stream):
        ctx = binding.Bagel(binding.dims_from_config(cfg, ckpt_interval=ckpt))          # the context works on `stream`
        ctx.bagel_prepare_samples(g["X"], g["y"], g["lengthscale"], g["signal_var"], g["noise_var"], g["omega"],
                                  g["phase"], g["w"], g["eps"], None)
        outs = [torch.full(sh, float("nan"), device="cuda")
                for sh in [(1,), (cfg.B,), (cfg.H + 1, cfg.B, cfg.d_s), (ctx.P,), (cfg.B, cfg.d_s)]]
        loss, lpt, states, gth, gs0 = outs

        def call():
            ctx.bagel_rollout_loss_grad(g["theta"], g["s0"], g["goals"], loss, gth, lpt, states, gs0)

        call()
        stream.synchronize()
        eager = [t.clone() for t in outs]
        assert all(torch.isfinite(t).all() for t in eager)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        call()
    for replay in range(3):
        for t in outs:
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(eager, outs):
            assert torch.equal(a, b), f"replay {replay}"
        with torch.cuda.stream(stream):
            call()                                                  # eager work between the replays
        stream.synchronize()
        for a, b in zip(eager, outs):
            assert torch.equal(a, b), f"eager call after replay {replay}"
    del graph
    ctx.close()


def test_repeated_calls_are_bitwise_reproducible():
    cfg = _cfg("small", B=200, H=15)
    inp = synth.make_inputs(cfg)
    ref = harness.oracle_reference(cfg, inp)
    a = harness.gpu_rollout(cfg, inp, ref["v32"])
    b = harness.gpu_rollout(cfg, inp, ref["v32"])
    for k in ("states", "grad_theta", "grad_s0", "loss_per_traj"):
        np.testing.assert_array_equal(a[k], b[k])


# ------------------------------------------------------------------ prepare
@pytest.mark.timeout(900)
@pytest.mark.parametrize("name,kw", [("tiny", {}), ("small", dict(B=48)), ("ragged", {}), ("one-point", {}),
                                     ("medium", dict(sub=64)), ("large_policy", dict(sub=64))])
def test_prepare_matches_oracle_solution(name, kw):
    """bagel_prepare_samples against the oracle's float64 solve, and the product path end to end
    (bagel_prepare_samples -> bagel_rollout_loss_grad) against the oracle driven from the UNROUNDED
    float64 v.  v is ill-conditioned (noise variance far below the signal variance): rounding it once to
    float32, which the float32 interface implies, already moves a rollout by `cond` below, measured here
    with the oracle alone (float64 v against the same v rounded).  The end-to-end deviation is held to a
    small multiple of that; tests/conditioning.py prints the same numbers for all five workloads."""
    if name == "ragged":
        cfg = synth.Config("p", 13, 3, 1, 1, 150, 77, 9, 3, (4,), 0.0, "sinusoid", "const", 0, 0.8, 1e-3)
        inp = synth.make_inputs(cfg)
    elif name == "one-point":                  # N = 1 (K_hat is a scalar), L = 1, B = S = 5
        cfg = synth.Config("p", 14, 2, 1, 1, 1, 1, 5, 4, (4,), 0.0, "sinusoid", "const", 0, 0.8, 1e-3)
        inp = synth.make_inputs(cfg)
    elif "sub" in kw:
        full = _cfg(name)
        idx = np.arange(kw["sub"]) * (full.B // kw["sub"]) + 3
        cfg, inp = synth.subset_trajectories(full, synth.make_inputs(full), idx)
    else:
        cfg = _cfg(name, **kw)
        inp = synth.make_inputs(cfg)
    dm = oracle.dims_from_config(cfg)
    v64 = oracle.prepare_samples(dm, inp)
    got = harness.gpu_rollout(cfg, inp, None, with_prepare=True, want_v=True)
    # forward error of a float64 Cholesky solve with cond(K_hat) ~ N alpha^2 / sigma_n^2, then one float32 rounding
    err = np.abs(got["v"] - v64).max() / np.abs(v64).max()
    print(f"[prepare {name}] max|dv|/max|v| = {err:.3e}", flush=True)
    assert err <= 5e-7
    exact = oracle.rollout(dm, inp, v64)                       # unrounded v
    cond = harness.deviations(exact, oracle.rollout(dm, inp, v64.astype(np.float32)))
    d = harness.deviations(exact, got)
    print(f"[prepare {name} end-to-end vs unrounded v] " + " ".join(f"{k}={x:.3e}" for k, x in d.items()), flush=True)
    print(f"[prepare {name} effect of rounding v once ] " + " ".join(f"{k}={x:.3e}" for k, x in cond.items()), flush=True)
    for k in ("state", "loss", "grad_l2", "grad_s0"):
        tol = {"state": harness.TOL_STATE, "loss": harness.TOL_LOSS}.get(k, harness.TOL_GRAD)
        assert d[k] <= 3.0 * cond[k] + tol, (k, d[k], cond[k])


def test_setup_work_space_is_made_once_and_kept():
    """The set-up calls share one work space: a second pass over them allocates nothing and gives the same bits."""
    import torch
    from paper_2202_13638_amd import binding
    cfg = _cfg("small", B=64, H=4)
    inp = synth.make_inputs(cfg)
    ctx = binding.Bagel(binding.dims_from_config(cfg))
    g = harness.to_gpu(inp)
    base = ctx.workspace_bytes()
    v = [torch.zeros((cfg.B, cfg.M, cfg.N), device="cuda") for _ in range(2)]
    lh = torch.cat([g["lengthscale"].log(), g["signal_var"].log()[:, None], g["noise_var"].log()[:, None]], dim=1).contiguous()
    yy = torch.from_numpy(inp["y"]).cuda()
    lml = [torch.zeros(cfg.M, device="cuda") for _ in range(2)]
    grad = [torch.zeros((cfg.M, cfg.D + 2), device="cuda") for _ in range(2)]
    sizes = []
    for rep in range(2):
        ctx.bagel_prepare_samples(g["X"], g["y"], g["lengthscale"], g["signal_var"], g["noise_var"], g["omega"],
                                  g["phase"], g["w"], g["eps"], v[rep])
        sizes.append(ctx.workspace_bytes())
        ctx.bagel_hyper_lml_grad(g["X"], yy, lh, lml[rep], grad[rep])
        sizes.append(ctx.workspace_bytes())
    torch.cuda.synchronize()
    assert sizes[0] > base                       # the first call made the work space
    assert sizes[1] >= sizes[0]                  # the next kind of call may enlarge it
    assert sizes[2] == sizes[1] and sizes[3] == sizes[1]      # the second pass allocates nothing
    assert torch.equal(v[0], v[1]) and torch.equal(lml[0], lml[1]) and torch.equal(grad[0], grad[1])
    ctx.close()


def test_prepare_reports_non_positive_definite():
    import torch
    from paper_2202_13638_amd import binding
    cfg = _cfg("tiny")
    inp = synth.make_inputs(cfg)
    inp["noise_var"] = np.full(cfg.M, -2.0, dtype=np.float32)
    ctx = binding.Bagel(binding.dims_from_config(cfg))
    g = harness.to_gpu(inp)
    with pytest.raises(binding.BagelError) as e:
        ctx.bagel_prepare_samples(g["X"], g["y"], g["lengthscale"], g["signal_var"], g["noise_var"], g["omega"],
                                  g["phase"], g["w"], g["eps"], None)
    assert e.value.code == binding.ENOTPD
    loss = torch.zeros(1, device="cuda")
    with pytest.raises(binding.BagelError) as e:
        ctx.bagel_rollout_loss(g["theta"], g["s0"], g["goals"], loss)
    assert e.value.code == binding.ENOTPREPARED
    ctx.close()


# ------------------------------------------------------------------ parameter update and inner loop
def test_adam_step_against_oracle_and_argument_checks():
    """bagel_adam_step on float32 arrays against the float64 oracle on the same values, over several
    updates with changing gradients (state stored in float32, so the bound is float32 rounding)."""
    import torch
    from paper_2202_13638_amd import binding
    cfg = _cfg("tiny")
    ctx = binding.Bagel(binding.dims_from_config(cfg))
    P = ctx.P
    rng = np.random.default_rng(11)
    theta = rng.standard_normal(P).astype(np.float32)
    th_o, m_o, v_o = theta.astype(np.float64), np.zeros(P), np.zeros(P)
    th_g = torch.from_numpy(theta).cuda()
    m_g, v_g = torch.zeros(P, device="cuda"), torch.zeros(P, device="cuda")
    # the interface takes the hyper-parameters as float32: the oracle gets exactly those values
    kw = {k: float(np.float32(x)) for k, x in dict(lr=1e-2, beta1=0.9, beta2=0.999, eps=1e-8).items()}
    m_scale, v_scale = np.zeros(P), np.zeros(P)      # largest value each stored moment went through
    for t in range(1, 9):
        g = (rng.standard_normal(P) * 10.0 ** rng.integers(-5, 2, P)).astype(np.float32)
        oracle.adam_step(th_o, g, m_o, v_o, t, **kw)
        ctx.bagel_adam_step(th_g, torch.from_numpy(g).cuda(), m_g, v_g, t, **kw)
        m_scale, v_scale = np.maximum(m_scale, np.abs(m_o)), np.maximum(v_scale, v_o)
    torch.cuda.synchronize()
    np.testing.assert_allclose(th_g.cpu().numpy(), th_o, rtol=0, atol=8 * 6e-8 * np.abs(th_o).max() + 8 * 1e-2 * 1e-5)
    assert (np.abs(m_g.cpu().numpy() - m_o) <= 8 * 6e-8 * m_scale + 1e-30).all()
    assert (np.abs(v_g.cpu().numpy() - v_o) <= 8 * 6e-8 * v_scale + 1e-30).all()
    for bad in (dict(step=0), dict(lr=0.0), dict(beta1=1.0), dict(beta2=-0.1), dict(eps=0.0)):
        args = dict(step=1, **kw)
        args.update(bad)
        with pytest.raises(binding.BagelError) as e:
            ctx.bagel_adam_step(th_g, m_g, m_g, v_g, args.pop("step"), **args)
        assert e.value.code == binding.EINVAL
    ctx.close()


def test_inner_loop_against_oracle():
    """bagel_optimize (rollout, gradient, Adam; two alternating sets of initial states and goals) against
    the oracle's loop, one iteration at a time from the same float32 state (parameters and moments): Adam
    divides the gradient by its own scale, so a gradient entry that is small against the gradient error
    moves by up to lr in either direction, and a free-running comparison drifts apart on exactly those
    entries.  Per iteration: loss to the loss tolerance; parameters with a clear gradient
    (|g| >= 1e-2 max|g|) to 2e-3 lr (the gradient tolerance, 1e-3 of max|g|, would allow a relative error
    of 0.1 on such an entry and hence 0.1 lr; the measured gradient error is about 1e-5 max|g|), all others
    within the largest step Adam can take.  The n-iteration
    call must then equal n one-iteration calls bit for bit."""
    import torch
    from paper_2202_13638_amd import binding
    cfg = _cfg("small", B=64, H=30)
    inp = synth.make_inputs(cfg)
    other = synth.make_inputs(cfg, trial=1)
    dm = oracle.dims_from_config(cfg)
    v32 = oracle.prepare_samples(dm, inp).astype(np.float32)
    s0_sets = np.stack([inp["s0"], other["s0"]])
    goal_sets = np.stack([inp["goals"], other["goals"]])
    n = 6
    hp = {k: float(np.float32(x)) for k, x in dict(lr=1e-2, beta1=0.9, beta2=0.999, eps=1e-8).items()}  # as the interface sees them
    lr = hp["lr"]

    ctx = binding.Bagel(binding.dims_from_config(cfg))
    g_in = harness.to_gpu(inp)
    ctx.bagel_set_samples(g_in["X"], g_in["lengthscale"], g_in["signal_var"], g_in["omega"], g_in["phase"], g_in["w"],
                          torch.from_numpy(v32).cuda())
    ss, gs = torch.from_numpy(s0_sets).cuda(), torch.from_numpy(goal_sets).cuda()
    th = np.asarray(inp["theta"], dtype=np.float32)
    am, av = np.zeros_like(th), np.zeros_like(th)
    worst = dict(loss=0.0, clear=0.0, rest=0.0)
    for i in range(n):
        # both sides start the iteration from the same float32 parameters and moments
        th_g, am_g, av_g = (torch.from_numpy(a.copy()).cuda() for a in (th, am, av))
        hist = torch.zeros(1, device="cuda")
        # iteration i uses set i % 2: present the sets rotated so that a one-iteration call picks it
        order = [i % 2, (i + 1) % 2]
        ctx.bagel_optimize(th_g, am_g, av_g, ss[order].contiguous(), gs[order].contiguous(), 1, hist, first_step=i + 1, **hp)
        torch.cuda.synchronize()
        th_o, am_o, av_o = th.astype(np.float64), am.astype(np.float64), av.astype(np.float64)
        r = oracle.rollout(dm, inp, v32, theta=th_o, s0=s0_sets[i % 2], goals=goal_sets[i % 2], want_states=False)
        oracle.adam_step(th_o, r["grad_theta"], am_o, av_o, i + 1, **hp)
        clear = np.abs(r["grad_theta"]) >= 1e-2 * np.abs(r["grad_theta"]).max()
        assert clear.sum() > 50
        d = np.abs(th_g.cpu().numpy().astype(np.float64) - th_o)
        worst["loss"] = max(worst["loss"], abs(float(hist.item()) - r["loss"]) / abs(r["loss"]))
        worst["clear"] = max(worst["clear"], d[clear].max())
        worst["rest"] = max(worst["rest"], d.max())
        # carry the oracle's state on, rounded to what the interface can hold
        th, am, av = th_o.astype(np.float32), am_o.astype(np.float32), av_o.astype(np.float32)
    print(f"[parity inner loop] per iteration: loss rel {worst['loss']:.3e}; theta: clear entries "
          f"{worst['clear']:.3e}, all {worst['rest']:.3e} (lr {lr:.3g})", flush=True)
    assert worst["loss"] <= harness.TOL_LOSS
    assert worst["clear"] <= 2e-3 * lr
    assert worst["rest"] <= 2.1 * lr

    # free-running: n iterations in one call == split calls with the state carried by the caller
    def run(chunks):
        theta = g_in["theta"].clone()
        m, v = torch.zeros_like(theta), torch.zeros_like(theta)
        hist = torch.zeros(n, device="cuda")
        done = 0
        for k in chunks:
            # a later call starts at iteration `done`: rotate the sets so that its first iteration uses set done % 2
            order = [done % 2, (done + 1) % 2]
            ctx.bagel_optimize(theta, m, v, ss[order].contiguous(), gs[order].contiguous(), k, hist[done:done + k],
                               first_step=done + 1, **hp)
            done += k
        torch.cuda.synchronize()
        return theta, hist
    t1, h1 = run([n])
    t2, h2 = run([2, 1, 3])
    assert torch.equal(t1, t2) and torch.equal(h1, h2)
    assert bool(torch.isfinite(t1).all()) and float(h1[0]) > 0.0
    ctx.close()


def test_inner_loop_with_checkpointing_equals_its_steps_taken_one_by_one():
    """With checkpointing the backward pass works on two streams.  Several iterations enqueued back to back by
    bagel_optimize must equal, bit for bit, gradient call + Adam step issued one at a time with a full
    synchronisation after each, and must be reproducible."""
    import torch
    from paper_2202_13638_amd import binding
    cfg = _cfg("small", B=96, H=23)
    inp = synth.make_inputs(cfg)
    g = harness.to_gpu(inp)
    ctx = binding.Bagel(binding.dims_from_config(cfg, ckpt_interval=5))
    ctx.bagel_prepare_samples(g["X"], g["y"], g["lengthscale"], g["signal_var"], g["noise_var"], g["omega"],
                              g["phase"], g["w"], g["eps"], None)
    hp = dict(lr=1e-2, beta1=0.9, beta2=0.999, eps=1e-8)
    n = 4
    s0_sets, goal_sets = g["s0"][None].contiguous(), g["goals"][None].contiguous()

    def free_running():
        theta = g["theta"].clone()
        m, v = torch.zeros_like(theta), torch.zeros_like(theta)
        hist = torch.zeros(n, device="cuda")
        ctx.bagel_optimize(theta, m, v, s0_sets, goal_sets, n, hist, **hp)
        torch.cuda.synchronize()
        return theta, m, v, hist

    a, b = free_running(), free_running()
    for x, y in zip(a, b):
        assert torch.equal(x, y)
    theta = g["theta"].clone()
    m, v = torch.zeros_like(theta), torch.zeros_like(theta)
    loss, grad = torch.zeros(1, device="cuda"), torch.zeros(ctx.P, device="cuda")
    hist = []
    for it in range(n):
        ctx.bagel_rollout_loss_grad(theta, g["s0"], g["goals"], loss, grad)
        torch.cuda.synchronize()
        hist.append(float(loss.item()))
        ctx.bagel_adam_step(theta, grad, m, v, it + 1, **hp)
        torch.cuda.synchronize()
    assert torch.equal(theta, a[0]) and torch.equal(m, a[1]) and torch.equal(v, a[2])
    assert hist == [float(x) for x in a[3].cpu()]
    assert hist[-1] < hist[0]
    ctx.close()


# ------------------------------------------------------------------ per-step posterior sampler
def _posterior_case(cfg, label, S=None, **dims_kw):
    """Oracle (exact eq. (2), (3) moments, reparameterised draws) against bagel_prepare_posterior +
    bagel_posterior_rollout_loss(_grad) on the same float32 inputs and draws."""
    import torch
    from paper_2202_13638_amd import binding
    inp = synth.make_inputs(cfg, S=S)
    xi = synth.make_normal_draws(cfg)
    dm = oracle.dims_from_config(cfg, S=S, **{k: v for k, v in dims_kw.items() if k != "ckpt_interval"})
    alpha, Kinv = oracle.posterior_prepare(dm, inp)
    ref = oracle.posterior_rollout(dm, inp, alpha, Kinv, xi)
    ctx = binding.Bagel(binding.dims_from_config(cfg, S=S, **dims_kw))
    g = harness.to_gpu(inp)
    B, H, ds = cfg.B, cfg.H, cfg.d_s
    loss = torch.full((1,), float("nan"), device="cuda")
    lpt = torch.full((B,), float("nan"), device="cuda")
    states = torch.full((H + 1, B, ds), float("nan"), device="cuda")
    gth = torch.full((ctx.P,), float("nan"), device="cuda")
    gs0 = torch.full((B, ds), float("nan"), device="cuda")
    xi_g = torch.from_numpy(xi).cuda()
    with pytest.raises(binding.BagelError) as e:
        ctx.bagel_posterior_rollout_loss(g["theta"], g["s0"], g["goals"], xi_g, loss)
    assert e.value.code == binding.ENOTPREPARED
    ctx.bagel_prepare_posterior(g["X"], g["y"], g["lengthscale"], g["signal_var"], g["noise_var"])
    ctx.bagel_posterior_rollout_loss(g["theta"], g["s0"], g["goals"], xi_g, loss, lpt, states)
    torch.cuda.synchronize()
    fwd = dict(loss=float(loss.item()), loss_per_traj=lpt.cpu().numpy().astype(np.float64),
               states=states.cpu().numpy().astype(np.float64))
    harness.assert_parity(ref, fwd, grad=False, label=f"{label}/fwd")
    ctx.bagel_posterior_rollout_loss_grad(g["theta"], g["s0"], g["goals"], xi_g, loss, gth, lpt, states, gs0)
    torch.cuda.synchronize()
    got = dict(loss=float(loss.item()), loss_per_traj=lpt.cpu().numpy().astype(np.float64),
               states=states.cpu().numpy().astype(np.float64), grad_theta=gth.cpu().numpy().astype(np.float64),
               grad_s0=gs0.cpu().numpy().astype(np.float64))
    harness.assert_parity(ref, got, label=f"{label}/grad")
    # the samplers share the model tables: installing one leaves the other unprepared
    with pytest.raises(binding.BagelError) as e:
        ctx.bagel_rollout_loss(g["theta"], g["s0"], g["goals"], loss)
    assert e.value.code == binding.ENOTPREPARED
    ctx.close()
    return got


def test_posterior_sampler_small_ragged():
    # N, B not multiples of the tile sizes; one hidden layer
    cfg = synth.Config("pp", 21, 3, 2, 2, 200, 16, 37, 12, (16,), 0.0, "sinusoid", "steps", 0, 0.6, 1e-3)
    _posterior_case(cfg, "posterior-ragged")


def test_posterior_sampler_bounded_saturating_checkpointed():
    cfg = synth.Config("pq", 22, 2, 1, 1, 130, 16, 64, 23, (32, 16), 0.8, "sinusoid", "const", 0, 0.5, 1e-3)
    plain = _posterior_case(cfg, "posterior-bounded", cost_kind=1, sigma_r=0.6)
    ck = _posterior_case(cfg, "posterior-bounded-ckpt", cost_kind=1, sigma_r=0.6, ckpt_interval=5)
    np.testing.assert_array_equal(plain["states"], ck["states"])
    np.testing.assert_allclose(plain["grad_theta"], ck["grad_theta"], rtol=1e-5, atol=1e-6 * np.abs(plain["grad_theta"]).max())


def test_posterior_sampler_one_training_point():
    # K_hat is a scalar: mu = k y / K_hat, sigma^2 = alpha^2 - k^2 / K_hat
    cfg = synth.Config("p1", 23, 2, 1, 1, 1, 16, 20, 6, (8,), 0.0, "sinusoid", "steps", 0, 0.5, 1e-3)
    _posterior_case(cfg, "posterior-one-point")


@pytest.mark.parametrize("d_s,d_a,d_g,N,B,H,hidden,bound", [
    (6, 2, 2, 300, 70, 6, (16, 8), 1.0),      # D = 8
    (7, 3, 1, 129, 33, 5, (8,), 0.0),         # D = 10
    (2, 1, 1, 700, 130, 4, (16,), 0.0),       # N over several tile rows, B over several tile columns
    (8, 8, 3, 64, 5, 3, (4,), 0.5),           # D = 16
])
def test_posterior_sampler_shapes(d_s, d_a, d_g, N, B, H, hidden, bound):
    cfg = synth.Config("ps", 40 + d_s, d_s, d_a, d_g, N, 16, B, H, hidden, bound, "sinusoid", "steps", 0, 0.6, 1e-3)
    _posterior_case(cfg, f"posterior-D{d_s + d_a}")
    _posterior_case(cfg, f"posterior-D{d_s + d_a}-ckpt", ckpt_interval=2)


@pytest.mark.timeout(600)
def test_posterior_sampler_small_config_size():
    """The Small configuration's model (N=512, 4 outputs, policy 5-64-64-1) with a shorter batch and horizon."""
    _posterior_case(_cfg("small", B=64, H=20), "posterior-small")


# ------------------------------------------------------------------ hyper-parameter learning
@pytest.mark.parametrize("N", [1, 2, 65])
def test_marginal_likelihood_few_training_points(N):
    """One point (K_hat a scalar), two, and one more than a block of the factorisation."""
    import torch
    from paper_2202_13638_amd import binding
    cfg = synth.Config("h1", 32, 2, 1, 1, N, 16, 4, 2, (4,), 0.0, "sinusoid", "const", 0, 0.5, 1e-3)
    inp = synth.make_inputs(cfg)
    lh0 = np.concatenate([np.log(inp["lengthscale"]), np.log(inp["signal_var"])[:, None],
                          np.log(inp["noise_var"])[:, None]], axis=1).astype(np.float32)
    ctx = binding.Bagel(binding.dims_from_config(cfg))
    g = harness.to_gpu(inp)
    lml = torch.zeros(cfg.M, device="cuda")
    grad = torch.zeros((cfg.M, cfg.D + 2), device="cuda")
    ctx.bagel_hyper_lml_grad(g["X"], g["y"], torch.from_numpy(lh0).cuda(), lml, grad)
    torch.cuda.synchronize()
    for m in range(cfg.M):
        ref, ref_g = oracle.hyper_lml_grad(inp["X"], inp["y"][m], lh0[m])
        assert abs(float(lml[m]) - ref) <= 2e-7 * abs(ref) + 1e-7
        np.testing.assert_allclose(grad[m].cpu().numpy(), ref_g, rtol=2e-6, atol=2e-6 * np.abs(ref_g).max() + 1e-7)
    ctx.close()


def test_marginal_likelihood_and_fit_against_oracle():
    """bagel_hyper_lml_grad against the numpy oracle (float64 on both sides, float32 interface), on a ragged
    N; then bagel_hyper_fit against the oracle's fit loop, which keeps its state in float32 like the
    interface does.  The gradient of the marginal likelihood has no entries that vanish against the
    others, so the free-running comparison is meaningful here."""
    import torch
    from paper_2202_13638_amd import binding
    cfg = synth.Config("hy", 31, 3, 1, 1, 150, 16, 8, 2, (4,), 0.0, "sinusoid", "const", 0, 0.5, 1e-3)
    inp = synth.make_inputs(cfg)
    M, D = cfg.M, cfg.D
    lh0 = np.concatenate([np.log(inp["lengthscale"]), np.log(inp["signal_var"])[:, None],
                          np.log(inp["noise_var"])[:, None]], axis=1).astype(np.float32)
    ctx = binding.Bagel(binding.dims_from_config(cfg))
    g = harness.to_gpu(inp)
    lml = torch.zeros(M, device="cuda")
    grad = torch.zeros((M, D + 2), device="cuda")
    ctx.bagel_hyper_lml_grad(g["X"], g["y"], torch.from_numpy(lh0).cuda(), lml, grad)
    torch.cuda.synchronize()
    for m in range(M):
        ref, ref_g = oracle.hyper_lml_grad(inp["X"], inp["y"][m], lh0[m])
        assert abs(float(lml[m]) - ref) <= 2e-7 * abs(ref)
        np.testing.assert_allclose(grad[m].cpu().numpy(), ref_g, rtol=2e-6, atol=2e-6 * np.abs(ref_g).max())
    # fit
    n, lr = 12, 5e-2
    start = np.tile(np.log(np.array([1.0] * D + [1.0, 0.1], dtype=np.float32)), (M, 1)).astype(np.float32)
    lh_o, m_o, v_o, hist_o = oracle.hyper_fit(inp["X"], inp["y"], start, n, lr=lr)
    lh_g = torch.from_numpy(start.copy()).cuda()
    am, av = torch.zeros_like(lh_g), torch.zeros_like(lh_g)
    hist = torch.zeros((n, M), device="cuda")
    ctx.bagel_hyper_fit(g["X"], g["y"], lh_g, am, av, n, hist, lr=lr)
    torch.cuda.synchronize()
    d_hist = np.abs(hist.cpu().numpy() - hist_o) / np.abs(hist_o)
    d_lh = np.abs(lh_g.cpu().numpy().astype(np.float64) - lh_o)
    print(f"[parity hyper fit] lml rel {d_hist.max():.3e}; log hyper-parameters abs {d_lh.max():.3e} after {n} updates",
          flush=True)
    assert d_hist.max() <= 1e-5 and d_lh.max() <= 1e-4
    assert np.all(hist_o[-1] > hist_o[0]) and bool((hist[-1] > hist[0]).all())
    ctx.close()


def test_marginal_likelihood_deep_blocking():
    """Marginal likelihood and gradient at a size where the factorisation and the substitutions recurse
    (N = 700: ranges of 704 -> 384 + 320 -> 192 + 192 + 192 + 128 columns) and with more outputs than the
    library works on side by side."""
    import torch
    from paper_2202_13638_amd import binding
    cfg = synth.Config("hy2", 32, 4, 1, 1, 700, 16, 8, 2, (4,), 0.0, "sinusoid", "const", 0, 0.5, 1e-3)
    inp = synth.make_inputs(cfg)
    M, D = cfg.M, cfg.D
    lh0 = np.concatenate([np.log(inp["lengthscale"]), np.log(inp["signal_var"])[:, None],
                          np.log(inp["noise_var"])[:, None]], axis=1).astype(np.float32)
    ctx = binding.Bagel(binding.dims_from_config(cfg))
    g = harness.to_gpu(inp)
    lml = torch.zeros(M, device="cuda")
    grad = torch.zeros((M, D + 2), device="cuda")
    ctx.bagel_hyper_lml_grad(g["X"], g["y"], torch.from_numpy(lh0).cuda(), lml, grad)
    torch.cuda.synchronize()
    for m in range(M):
        ref, ref_g = oracle.hyper_lml_grad(inp["X"], inp["y"][m], lh0[m])
        assert abs(float(lml[m]) - ref) <= 2e-7 * abs(ref)
        np.testing.assert_allclose(grad[m].cpu().numpy(), ref_g, rtol=5e-6, atol=5e-6 * np.abs(ref_g).max())
    ctx.close()


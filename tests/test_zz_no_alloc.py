"""GPU check of bagel_sample_eval_static, the sample evaluation for callers that cannot allocate:
through the C ABI, against the existing entry points (bagel_set_samples + bagel_sample_eval on a
context) and against the float64 oracle, on two calls in a row, the second with a smaller input
(the calls share one static device buffer, which keeps the first call's contents)."""
import numpy as np
import pytest

import oracle
from paper_2202_13638_amd import synth

pytestmark = pytest.mark.gpu

SHAPES = [
    dict(d_s=6, d_a=2, N=300, L=200, B=130, S=13),     # ragged N, L, B; shared samples; D = 8
    dict(d_s=3, d_a=2, N=50, L=70, B=37, S=37),        # smaller in every extent
]


def _case(shape, seed):
    import torch
    from paper_2202_13638_amd import binding
    import harness
    cfg = synth.Config("e", 11, shape["d_s"], shape["d_a"], 1, shape["N"], shape["L"], shape["B"], 2, (4,), 0.0,
                       "sinusoid", "const", 0, 0.7, 1e-3)
    inp = synth.make_inputs(cfg, trial=seed, S=shape["S"])
    dm = oracle.dims_from_config(cfg, S=shape["S"])
    v32 = oracle.prepare_samples(dm, inp).astype(np.float32)
    x = np.random.default_rng(seed).uniform(-1.2, 1.2, (cfg.B, cfg.D)).astype(np.float32)
    g = harness.to_gpu(inp)
    g["v"] = torch.from_numpy(v32).cuda()
    g["x"] = torch.from_numpy(x).cuda()
    dims = binding.dims_from_config(cfg, S=shape["S"])
    return cfg, inp, dm, v32, x, g, dims


def _static(dims, g, cfg, with_jac=True):
    import torch
    from paper_2202_13638_amd import binding
    f = torch.full((cfg.B, cfg.M), float("nan"), device="cuda")
    J = torch.full((cfg.B, cfg.M, cfg.D), float("nan"), device="cuda") if with_jac else None
    binding.bagel_sample_eval_static(dims, g["X"], g["lengthscale"], g["signal_var"], g["omega"], g["phase"],
                                     g["w"], g["v"], g["x"], f, J)
    return f, J


def _with_context(dims, g, cfg):
    import torch
    from paper_2202_13638_amd import binding
    ctx = binding.Bagel(dims)
    ctx.bagel_set_samples(g["X"], g["lengthscale"], g["signal_var"], g["omega"], g["phase"], g["w"], g["v"])
    f = torch.empty((cfg.B, cfg.M), device="cuda")
    J = torch.empty((cfg.B, cfg.M, cfg.D), device="cuda")
    ctx.bagel_sample_eval(g["x"], f, J)
    torch.cuda.synchronize()
    ctx.close()
    return f.cpu().numpy(), J.cpu().numpy()


def test_static_sample_eval_two_calls_in_a_row_second_smaller():
    import torch
    cases = [_case(shape, seed) for seed, shape in enumerate(SHAPES)]
    # the two calls under test, back to back on one stream, nothing else in between
    outs = [_static(dims, g, cfg) for cfg, inp, dm, v32, x, g, dims in cases]
    torch.cuda.synchronize()
    for (cfg, inp, dm, v32, x, g, dims), (f, J) in zip(cases, outs):
        f, J = f.cpu().numpy(), J.cpu().numpy()
        assert np.isfinite(f).all() and np.isfinite(J).all()
        # against the existing entry points: same kernels, same work split -> same float32 numbers
        f_ctx, J_ctx = _with_context(dims, g, cfg)
        np.testing.assert_allclose(f, f_ctx, rtol=0, atol=1e-6 * max(1.0, np.abs(f_ctx).max()))
        np.testing.assert_allclose(J, J_ctx, rtol=0, atol=1e-6 * max(1.0, np.abs(J_ctx).max()))
        # against the oracle, at the bar of the sample-evaluation parity tests
        per = cfg.B // dims.S
        fr = np.zeros((cfg.B, cfg.M)); Jr = np.zeros((cfg.B, cfg.M, cfg.D))
        for b in range(cfg.B):
            fr[b], Jr[b] = oracle.sample_eval(dm, inp, inp["w"][b // per], v32[b // per], x[b])
        assert np.abs(f - fr).max() <= 2e-6 * max(1.0, np.abs(fr).max())
        assert np.abs(J - Jr).max() <= 1e-5 * max(1.0, np.abs(Jr).max())
    # value only (jac = NULL) gives the same values
    cfg, inp, dm, v32, x, g, dims = cases[0]
    f_only, _ = _static(dims, g, cfg, with_jac=False)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(f_only.cpu().numpy(), outs[0][0].cpu().numpy())


def test_static_sample_eval_rejects_what_does_not_fit():
    from paper_2202_13638_amd import binding
    cfg, inp, dm, v32, x, g, dims = _case(SHAPES[1], 1)
    big = binding.make_dims(d_s=3, d_a=2, d_g=1, N=4096, L=4096, S=4096, B=4096, H=2, hidden=(4,))
    with pytest.raises((binding.BagelError, ValueError)) as ei:
        import torch
        z = torch.zeros(1, device="cuda")
        rc = binding.load().bagel_sample_eval_static(*([__import__("ctypes").byref(big), None] + [z.data_ptr()] * 10))
        if rc != binding.OK:
            raise binding.BagelError(rc, binding.load().bagel_last_error(None).decode())
    assert "static buffer" in str(ei.value)

"""Host-only checks of the C-ABI library: it loads, exports every symbol the header declares,
and rejects bad dimensions before touching a device.  No compute calls (no GPU here)."""
import ctypes as C
import os
import re

import pytest

from paper_2202_13638_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2202_13638_amd import build
        build.build()
    return binding.load()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "bagel.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = sorted(set(re.findall(r"\b(bagel_[a-z_0-9]+)\s*\(", header)))
    assert declared, "no declarations found"
    for name in declared:
        assert hasattr(lib, name), f"{name} is declared in bagel.h but not exported"
    assert sorted(binding.EXPORTS) == declared


def test_num_params_matches_configs(lib):
    expected = {"tiny": 81, "small": 4609, "medium": 4609, "large_policy": 67585, "stress": 68610, "paper_exp1": 121}
    for name, cfg in synth.CONFIGS.items():
        assert binding.bagel_num_params(binding.dims_from_config(cfg)) == expected[name] == cfg.P


@pytest.mark.parametrize("field,value", [
    ("d_s", 0), ("d_s", 9), ("d_a", 0), ("d_g", 3), ("N", 0), ("L", -1), ("S", 3), ("S", 32), ("H", 0),
    ("n_hidden", 0), ("n_hidden", 3), ("ckpt_interval", -1), ("cost_kind", 2),
])
def test_bad_dims_are_rejected_without_a_device(lib, field, value):
    dims = binding.make_dims(d_s=2, d_a=1, d_g=1, N=8, L=8, S=4, B=16, H=5, hidden=(8,))
    setattr(dims, field, value)
    assert binding.bagel_num_params(dims) == binding.EINVAL
    h = C.c_void_p()
    rc = lib.bagel_create(C.byref(h), C.byref(dims), None)
    assert rc == binding.EINVAL and not h.value
    assert lib.bagel_last_error(None).decode().startswith("bagel_create:")


def test_bad_hidden_tracked_and_null_arguments(lib):
    dims = binding.make_dims(d_s=2, d_a=1, d_g=1, N=8, L=8, S=4, B=16, H=5, hidden=(257,))
    assert binding.bagel_num_params(dims) == binding.EINVAL
    dims = binding.make_dims(d_s=2, d_a=1, d_g=1, N=8, L=8, S=4, B=16, H=5, hidden=(8,), tracked=[2])
    assert binding.bagel_num_params(dims) == binding.EINVAL
    dims = binding.make_dims(d_s=2, d_a=1, d_g=1, N=8, L=8, S=4, B=16, H=5, hidden=(8,), cost_kind=1, sigma_r=0.0)
    assert binding.bagel_num_params(dims) == binding.EINVAL
    assert lib.bagel_create(None, None, None) == binding.EINVAL
    assert lib.bagel_destroy(None) == binding.OK
    assert lib.bagel_rollout_loss(None, None, None, None, None, None, None) == binding.EINVAL
    assert lib.bagel_workspace_bytes(None) == 0
    assert lib.bagel_adam_step(None, None, None, None, None, 1, 1e-2, 0.9, 0.999, 1e-8) == binding.EINVAL
    assert lib.bagel_hyper_lml_grad(None, None, None, None, None, None) == binding.EINVAL
    assert lib.bagel_hyper_fit(None, None, None, None, None, None, 1, 1, 1e-2, 0.9, 0.999, 1e-8, None) == binding.EINVAL
    assert lib.bagel_prepare_posterior(None, None, None, None, None, None) == binding.EINVAL
    assert lib.bagel_posterior_rollout_loss(None, None, None, None, None, None, None, None) == binding.EINVAL
    assert lib.bagel_optimize(None, None, None, None, None, None, 1, 1, 1, 1e-2, 0.9, 0.999, 1e-8, None) == binding.EINVAL


def test_sizes_beyond_the_work_decomposition_are_rejected_without_a_device(lib):
    """The largest problems: the sample evaluation addresses its work units with a 16-bit grid index, and
    B * H is bounded; both limits are checked before anything is allocated."""
    h = C.c_void_p()
    dims = binding.make_dims(d_s=8, d_a=8, d_g=8, N=40_000_000, L=8, S=64, B=64, H=5, hidden=(8,))
    assert lib.bagel_create(C.byref(h), C.byref(dims), None) == binding.EINVAL and not h.value
    assert "work units" in lib.bagel_last_error(None).decode()
    dims = binding.make_dims(d_s=2, d_a=1, d_g=1, N=8, L=8, S=1, B=2_000_000_000, H=1000, hidden=(8,))
    assert lib.bagel_create(C.byref(h), C.byref(dims), None) == binding.EINVAL and not h.value
    assert "too large" in lib.bagel_last_error(None).decode()


def test_binding_rejects_host_tensors():
    import torch
    with pytest.raises(ValueError):
        binding._ptr(torch.zeros(3), (3,), "x")
    with pytest.raises(ValueError):
        binding._ptr(None, (3,), "x")
    assert binding._ptr(None, (3,), "x", optional=True) is None

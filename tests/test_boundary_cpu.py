"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every function include/srm.h declares, and rejects bad arguments before any
HIP call."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import srm_synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def srm():
    import paper_2605_08696_amd as pkg
    from paper_2605_08696_amd import build as b
    if b.is_stale():
        b.build_lib()
    pkg.lib()
    return pkg


def declared_functions():
    text = open(os.path.join(ROOT, "include", "srm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(srm_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_boundary():
    names = declared_functions()
    for must in ("srm_init_weights", "srm_prefill", "srm_decode_step", "srm_parallel_forward",
                 "srm_free", "srm_state_bytes", "srm_workspace_bytes", "srm_last_error"):
        assert must in names


def test_library_exports_every_declared_symbol(srm):
    L = srm.lib()
    for name in declared_functions():
        assert hasattr(L, name), name


def _cfg_struct(srm, **over):
    from paper_2605_08696_amd.binding import srm_config
    base = dict(vocab=32, d_model=16, n_layers=1, n_heads=2, mlp_expansion=4, n_ctx=16,
                weight_dtype=0, ln_eps=1e-5)
    base.update(over)
    return srm_config(**base)


def test_init_rejects_bad_configs_before_touching_the_gpu(srm):
    from paper_2605_08696_amd.binding import srm_host_weights
    L = srm.lib()
    hw = srm_host_weights()
    h = C.c_void_p()
    cases = [dict(vocab=0), dict(n_heads=3), dict(d_model=20), dict(d_model=8192, n_heads=4),
             dict(weight_dtype=7), dict(weight_dtype=1, d_model=32), dict(ln_eps=0.0), dict(n_ctx=0)]
    for over in cases:
        rc = L.srm_init_weights(C.byref(_cfg_struct(srm, **over)), C.byref(hw), C.byref(h))
        assert rc == -1, over
        assert L.srm_last_error() != b""
    # valid config, null weight pointers
    rc = L.srm_init_weights(C.byref(_cfg_struct(srm)), C.byref(hw), C.byref(h))
    assert rc == -1 and b"null" in L.srm_last_error()
    assert L.srm_init_weights(None, None, None) == -1


def test_init_rejects_lambda_out_of_range(srm):
    cfg = srm_synth.tiny_config(vocab=32, d_model=16, n_layers=1, n_heads=2, n_ctx=16)
    w = srm_synth.make_weights(cfg)
    w["layers"][0]["lam"][1] = 1.5
    with pytest.raises(srm.SrmError) as e:
        srm.Model(cfg, w)
    assert e.value.code == -1 and "lambda" in str(e.value)


def test_sizes_of_null_model_are_zero(srm):
    L = srm.lib()
    assert L.srm_state_bytes(None, 4) == 0
    assert L.srm_workspace_bytes(None, 4) == 0
    assert L.srm_linear_scratch_bytes(0, 5) == 0
    assert L.srm_linear_scratch_bytes(3, 130) >= 3 * 3 * 8


def test_null_arguments_are_rejected(srm):
    L = srm.lib()
    assert L.srm_decode_step(None, 1, 0, None, None, None, None, None, None, 0, None) == -1
    assert L.srm_prefill(None, None, 1, 1, 1, None, None, None, None, 0, None) == -1
    assert L.srm_parallel_forward(None, None, 1, 1, None, None, None, 0, None) == -1
    assert L.srm_mixer_update(None, 0, 0, 1, None, None, None, None) == -1
    assert L.srm_mixer_project_update(None, 0, 0, 1, None, None, None, None) == -1
    assert L.srm_linear(0, 0, None, None, None, 1, 1, 1, None, None, None, None) == -1


def test_binding_shape_checks(srm):
    cfg = srm_synth.tiny_config(vocab=32, d_model=16, n_layers=1, n_heads=2, n_ctx=16)
    w = srm_synth.make_weights(cfg)
    w["embed"] = w["embed"][:-1]
    with pytest.raises(ValueError):
        srm.Model(cfg, w)


def test_bf16_rounding_of_inputs_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.005859375, 1.01171875, -2.5, 3.0e38], dtype=np.float32)
    import torch
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(srm_synth.round_to_bf16(x), ref)
    r = np.random.default_rng(0).standard_normal(10000).astype(np.float32)
    np.testing.assert_array_equal(srm_synth.round_to_bf16(r),
                                  torch.from_numpy(r).to(torch.bfloat16).to(torch.float32).numpy())

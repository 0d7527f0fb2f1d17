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
    assert L.srm_mixer_block(None, 0, 0, None, 1, None, None, None, None, None) == -1
    assert L.srm_linear(0, 0, None, None, None, 1, 1, 1, None, None, None, None) == -1


def _plan_case(srm, cfg, lens, ws_rows):
    """The library's plan for a ragged prefill, checked against the passes and buffer extents recomputed
    here: partial states of the chunked scan are [prompts of the pass][chunks][state width] fp32 and live in
    the pass's MLP buffer of rows x ff activation elements."""
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    ws = srm.workspace_bytes_config(cfg, ws_rows)
    plan = srm.prefill_ragged_plan(cfg, off, ws)
    max_rows = ws_rows
    while srm.workspace_bytes_config(cfg, max_rows + 1) <= ws:
        max_rows += 1
    passes, n0 = [], 0
    while n0 < len(lens):
        n1 = n0
        while n1 < len(lens) and off[n1 + 1] - off[n0] <= max_rows:
            n1 += 1
        passes.append((n0, n1))
        n0 = n1
    assert plan["passes"] == len(passes)
    wsize = 2 if cfg.weight_dtype == "bf16" else 4
    ff = cfg.d_model * cfg.mlp_expansion
    for c in (plan["chunk_len"],):
        if c:
            nch = -(-max(lens) // c)
            for n0, n1 in passes:
                need = (n1 - n0) * nch * cfg.state_width * 4
                room = int(off[n1] - off[n0]) * ff * wsize
                assert need <= room, (lens[:4], ws_rows, n0, n1, need, room)
    if plan["chunk_len_by_shape"] and not plan["chunk_len"]:
        assert plan["scratch_need"] > plan["scratch_room"]
    return plan


def test_chunked_scan_scratch_stays_inside_the_workspace(srm):
    """Many short prompts next to one long one: the chunk count follows the longest prompt, the buffer the rows
    of the pass; the partial states of the chunked scan would overrun it, so the call must fall back."""
    cfg = srm_synth.tiny_config(vocab=64, d_model=256, n_layers=1, n_heads=4, n_ctx=512, weight_dtype="bf16")
    skew = [1] * 199 + [256]
    plan = _plan_case(srm, cfg, skew, ws_rows=sum(skew))
    assert plan["chunk_len_by_shape"] == 16 and plan["chunk_len"] == 0
    assert plan["scratch_need"] == 200 * 16 * 256 * 4 and plan["scratch_room"] == 455 * 1024 * 2
    plan = _plan_case(srm, cfg, skew, ws_rows=256)                   # the documented minimum: several passes
    assert plan["chunk_len"] == 0 and plan["passes"] >= 2
    # a few long prompts: the chunked scan is taken and fits
    plan = _plan_case(srm, cfg, [512] * 8, ws_rows=8 * 512)
    assert plan["chunk_len"] > 0 and plan["scratch_need"] <= plan["scratch_room"]
    plan = _plan_case(srm, cfg, [200, 77, 1, 130, 16], ws_rows=424)
    assert plan["chunk_len"] > 0
    rng = np.random.default_rng(5)
    for trial in range(60):
        n = int(rng.integers(1, 300))
        lens = rng.integers(1, 3, size=n) if trial % 2 else rng.integers(1, 400, size=n)
        lens[int(rng.integers(0, n))] = int(rng.integers(64, 512))
        lens = [int(v) for v in lens]
        rows = int(rng.integers(max(lens), sum(lens) + 1))
        for c in (cfg, srm_synth.tiny_config(vocab=64, d_model=64, n_layers=1, n_heads=2, n_ctx=512,
                                             head_layout="column", mixer_kernel=8)):
            _plan_case(srm, c, lens, rows)


def test_plan_rejects_what_the_prefill_rejects(srm):
    cfg = srm_synth.tiny_config(vocab=64, d_model=64, n_layers=1, n_heads=2, n_ctx=32)
    ws = srm.workspace_bytes_config(cfg, 64)
    assert ws > 0 and srm.workspace_bytes_config(cfg, 0) == 0
    with pytest.raises(srm.SrmError):
        srm.prefill_ragged_plan(cfg, [0, 40], ws)            # longer than n_ctx
    with pytest.raises(srm.SrmError):
        srm.prefill_ragged_plan(cfg, [0, 0], ws)             # empty prompt
    with pytest.raises(srm.SrmError):
        srm.prefill_ragged_plan(cfg, [0, 20], srm.workspace_bytes_config(cfg, 8))   # workspace below one prompt


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

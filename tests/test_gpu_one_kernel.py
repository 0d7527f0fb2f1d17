"""Generation of a handful of samples in one persistent kernel (the path srm_generate takes for
small fp32 batches) against the oracle and against the ordinary step kernels."""
import dataclasses
import os

import numpy as np
import pytest
import torch

import srm_synth
from gpu_util import to_dev, check_tokens

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def srm():
    import paper_2605_08696_amd as pkg
    pkg.lib()
    return pkg


@pytest.fixture(scope="module")
def orc_mod(oracle_mod):
    return oracle_mod


def _generate(model, prompts, G, one_kernel, temperature=None, seed=0):
    """Prefill, then G - 1 further tokens with srm_generate; returns (tokens [B][G], state)."""
    B, P = prompts.shape
    ws = model.new_workspace(B * P)
    st, tk = model.new_state(B), torch.empty(B, dtype=torch.int32, device="cuda")
    kw = {} if temperature is None else {"temperature": temperature, "seed": seed}
    if temperature is None:
        model.prefill(to_dev(prompts), 1, st, tk, workspace=ws)
        first = tk.cpu().numpy().copy()
        pos0, steps = P, G - 1
    else:                                   # sampling: the first token is drawn by the generate call too
        dp = to_dev(prompts)
        model.prefill(dp[:, :P - 1].contiguous(), 1, st, tk, workspace=ws)
        tk.copy_(dp[:, P - 1])
        first, pos0, steps = None, P - 1, G
    out = torch.full((steps, B), -7, dtype=torch.int32, device="cuda")
    old = os.environ.get("SRM_MEGAKERNEL")
    os.environ["SRM_MEGAKERNEL"] = "2" if one_kernel else "0"      # 2: the path whatever the model's size
    try:
        assert (model.one_kernel_blocks(B) > 0) == one_kernel
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            model.generate(B, pos0, steps, tk, st, out, workspace=ws, **kw)
        side.synchronize()
    finally:
        if old is None:
            del os.environ["SRM_MEGAKERNEL"]
        else:
            os.environ["SRM_MEGAKERNEL"] = old
    toks = out.cpu().numpy().T
    assert (tk.cpu().numpy() == toks[:, -1]).all()
    if first is not None:
        toks = np.concatenate([first[:, None], toks], axis=1)
    return toks, st


@pytest.mark.parametrize("B", [1, 3, 8])
def test_one_kernel_generation_matches_oracle_and_step_kernels(srm, orc_mod, B):
    cfg = srm_synth.CONFIGS["C1"]
    w = srm_synth.make_weights(cfg)
    prompts = srm_synth.make_prompts(cfg)[:B]
    G = 32
    ref = orc_mod.Oracle(cfg, w, "f64").greedy(prompts, G, want_logits=True)
    model = srm.Model(cfg, w)
    print(f"one-kernel generation C1 B={B}", flush=True)
    got, st = _generate(model, prompts, G, True)
    assert check_tokens(got, ref["tokens"], ref["margin"], np.abs(ref["logits"]).max(axis=2)) == 0
    s_ref = ref["state"]
    s_got = st.permute(1, 0, 2).cpu().numpy()
    assert np.abs(s_got - s_ref).max() <= 1e-4 * np.abs(s_ref).max()
    got2, st2 = _generate(model, prompts, G, False)
    np.testing.assert_array_equal(got, got2)
    assert (st - st2).abs().max() <= 1e-5 * st2.abs().max()


def test_one_kernel_sampling_matches_oracle(srm, orc_mod):
    cfg = srm_synth.CONFIGS["C1"]
    w = srm_synth.make_weights(cfg)
    w["head"] = w["head"] * 25.0
    prompts = srm_synth.make_prompts(cfg)[:5]
    G, T, seed = 20, 0.7, 99
    ref = orc_mod.Oracle(cfg, w, "f64").greedy(prompts, G, want_logits=True, temperature=T, seed=seed)
    model = srm.Model(cfg, w)
    print("one-kernel sampling", flush=True)
    got, _ = _generate(model, prompts, G, True, temperature=T, seed=seed)
    assert check_tokens(got, ref["tokens"], ref["margin"], np.abs(ref["logits"]).max(axis=2)) == 0
    greedy = orc_mod.Oracle(cfg, w, "f64").greedy(prompts, G)
    assert (got != greedy["tokens"]).any()


@pytest.mark.parametrize("variant", [dict(head_layout="combined"), dict(head_layout="column", mixer_kernel=3),
                                     dict(head_layout="row", n_heads=1), dict(d_model=320, n_heads=4),
                                     dict(d_model=1024, n_heads=4, mlp_expansion=2, B=1)])
def test_one_kernel_generation_variants_and_odd_sizes(srm, orc_mod, variant):
    kw = dict(vocab=333, d_model=64, n_layers=3, n_heads=2, n_ctx=48, seed=91)
    kw.update(variant)
    B = kw.pop("B", 4)
    cfg = srm_synth.tiny_config(**kw)
    w = srm_synth.make_weights(cfg, stress=True)
    P, G = 6, 24
    prompts = srm_synth.make_prompts(cfg, batch=B, length=P)
    ref = orc_mod.Oracle(cfg, w, "f64").greedy(prompts, G, want_logits=True)
    model = srm.Model(cfg, w)
    print(f"one-kernel generation {variant}", flush=True)
    got, st = _generate(model, prompts, G, True)
    assert check_tokens(got, ref["tokens"], ref["margin"], np.abs(ref["logits"]).max(axis=2)) == 0
    s_got = st.permute(1, 0, 2).cpu().numpy()
    assert np.abs(s_got - ref["state"]).max() <= 1e-4 * np.abs(ref["state"]).max()


def test_one_kernel_path_is_taken_only_where_it_applies(srm):
    cfg = srm_synth.CONFIGS["C1"]
    w = srm_synth.make_weights(cfg)
    model = srm.Model(cfg, w)
    # by default only while rows x matrix elements stay small; never above 8 rows
    assert model.one_kernel_blocks(4) > 0 and model.one_kernel_blocks(8) == 0
    os.environ["SRM_MEGAKERNEL"] = "2"
    try:
        assert model.one_kernel_blocks(8) > 0 and model.one_kernel_blocks(9) == 0
    finally:
        del os.environ["SRM_MEGAKERNEL"]
    for other in (dataclasses.replace(cfg, state_dtype="fp16"), dataclasses.replace(cfg, use_projections=False)):
        assert srm.Model(other, w).one_kernel_blocks(4) == 0
    cb = srm_synth.tiny_config(vocab=256, d_model=64, n_layers=1, n_heads=2, n_ctx=8, weight_dtype="bf16")
    assert srm.Model(cb, srm_synth.make_weights(cb)).one_kernel_blocks(4) == 0
    # one step, and a grid larger than the default
    prompts = srm_synth.make_prompts(cfg)[:2]
    a, _ = _generate(model, prompts, 2, True)
    os.environ["SRM_MEGA_BLOCKS"] = "40"
    try:
        assert model.one_kernel_blocks(2) == 40
        b, _ = _generate(model, prompts, 12, True)
    finally:
        del os.environ["SRM_MEGA_BLOCKS"]
    c, _ = _generate(model, prompts, 12, False)
    np.testing.assert_array_equal(b, c)
    np.testing.assert_array_equal(a, c[:, :2])

"""Nucleus (top-p) sampling on the GPU against the oracle's rule: the sampler
alone on given logits, then inside the decode step (single calls, graph replay,
ragged positions)."""
import numpy as np
import pytest
import torch

import srm_synth
from gpu_util import to_dev

pytestmark = pytest.mark.gpu

MASS_TOL = 1e-5        # a cut decided by less probability than this may fall either way in fp32


@pytest.fixture(scope="module")
def srm():
    import paper_2605_08696_amd as pkg
    pkg.lib()
    return pkg


@pytest.fixture(scope="module")
def orc_mod(oracle_mod):
    return oracle_mod


def _check_rows(orc_mod, got, logits, T, top_p, seed, pos_of, b_of=None):
    """Every GPU choice equals the oracle's choice from the same logits, unless the oracle's own
    decision was a near tie (nucleus boundary within MASS_TOL, or top-2 scores within 1e-5 of
    the logit scale).  Returns (tolerated, rows where truncation changed the plain draw)."""
    tolerated = changed = 0
    for r in range(logits.shape[0]):
        b = r if b_of is None else b_of[r]
        tok, mg, mm = orc_mod.pick_topp(logits[r], T, top_p, seed, pos_of(r), b, want_margins=True)
        if orc_mod.pick(logits[r], T, seed, pos_of(r), b) != tok:
            changed += 1
        if got[r] != tok:
            assert mm < MASS_TOL or mg < 1e-5 * np.abs(logits[r]).max(), f"row {r}: {got[r]} != {tok}"
            tolerated += 1
    return tolerated, changed


@pytest.mark.parametrize("V,scale,T,top_p", [(40, 2.0, 1.0, 0.5), (1000, 3.0, 0.7, 0.9), (4099, 0.05, 0.7, 0.9),
                                            (4099, 4.0, 1.5, 0.99), (32000, 2.0, 0.7, 0.9), (32000, 0.02, 0.7, 0.9),
                                            (777, 6.0, 0.7, 0.05)])
def test_sample_logits_matches_oracle(srm, orc_mod, V, scale, T, top_p):
    rows = 256 if V >= 32000 else 600
    rng = np.random.default_rng(V + int(100 * top_p))
    logits = (rng.standard_normal((rows, V)) * scale).astype(np.float32)
    logits[3, :] = logits[3, 0]                               # a row of equal logits: everything is kept
    if V > 100:
        logits[4, 10:20] = logits[4].max() + 1.0              # ties at the top
    print(f"sample_logits V={V} scale={scale} T={T} top_p={top_p} rows={rows}", flush=True)
    dl = to_dev(logits)
    out = torch.full((rows,), -5, dtype=torch.int32, device="cuda")
    seed, pos = 77, 9
    srm.sample_logits(dl, T, top_p, seed, pos, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    tolerated, changed = _check_rows(orc_mod, got, logits, T, top_p, seed, lambda r: pos)
    assert tolerated <= max(2, rows // 50)
    if top_p <= 0.9:
        assert changed > 0                                      # the truncation mattered for some rows
    # same call again: bit-reproducible
    out2 = torch.empty_like(out)
    srm.sample_logits(dl, T, top_p, seed, pos, out2)
    assert torch.equal(out, out2)
    # top_p = 1: the plain Gumbel-max draw
    srm.sample_logits(dl, T, 1.0, seed, pos, out2)
    torch.cuda.synchronize()
    plain = out2.cpu().numpy()
    for r in range(0, rows, 7):
        assert plain[r] == orc_mod.pick(logits[r], T, seed, pos, r)


def test_sample_logits_frequencies_follow_truncated_softmax(srm, orc_mod):
    import scipy.stats
    lg = np.array([1.2, -0.3, 0.4, 2.0, 0.0, -1.5, 0.9, 0.1], np.float32)
    T, top_p, R = 0.7, 0.9, 80000
    keep, _ = orc_mod.nucleus(lg, T, top_p)
    p = np.exp(lg.astype(np.float64) / T) * keep; p /= p.sum()
    out = torch.empty(R, dtype=torch.int32, device="cuda")
    srm.sample_logits(to_dev(np.tile(lg, (R, 1))), T, top_p, 5, 0, out)
    torch.cuda.synchronize()
    counts = np.bincount(out.cpu().numpy(), minlength=lg.size)
    assert counts[~keep].sum() == 0
    assert scipy.stats.chisquare(counts[keep], p[keep] * R).pvalue > 1e-4


def _topp_run(model, prompts_np, G, T, top_p, seed, mode):
    """Prefill all but the last prompt token, then G nucleus-sampled steps."""
    B, P = prompts_np.shape
    dp = to_dev(prompts_np)
    ws = model.new_workspace(B * P)
    st, tk = model.new_state(B), torch.empty(B, dtype=torch.int32, device="cuda")
    model.prefill(dp[:, :P - 1].contiguous(), 1, st, tk, workspace=ws)
    tk.copy_(dp[:, P - 1])
    lg = torch.empty((B, model.vocab), dtype=torch.float32, device="cuda")
    out = torch.empty((G, B), dtype=torch.int32, device="cuda")
    if mode == "generate":
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            model.generate(B, P - 1, G, tk, st, out, workspace=ws, temperature=T, seed=seed, top_p=top_p, logits=lg)
        side.synchronize()
    elif mode == "ragged":
        pos = torch.full((B,), P - 1, dtype=torch.int32, device="cuda")
        for g in range(G):
            model.decode_step_ragged(B, pos, tk, st, tk, advance=True, temperature=T, seed=seed, top_p=top_p,
                                     logits=lg, workspace=ws)
            out[g] = tk
        assert (pos == P - 1 + G).all()
    else:
        for g in range(G):
            model.decode_step(B, P - 1 + g, tk, st, tk, logits=lg, workspace=ws, temperature=T, seed=seed,
                              top_p=top_p)
            out[g] = tk
    torch.cuda.synchronize()
    return out.cpu().numpy().T


@pytest.mark.parametrize("mode", ["steps", "generate", "ragged"])
def test_topp_generation_matches_oracle_fp32(srm, orc_mod, mode):
    cfg = srm_synth.CONFIGS["C1"]
    w = srm_synth.make_weights(cfg)
    w["head"] = w["head"] * 25.0                                # peaked enough for the nucleus to be a strict subset
    prompts = srm_synth.make_prompts(cfg)
    G, T, top_p, seed = 24, 0.7, 0.9, 2024
    print(f"top-p generation mode={mode}", flush=True)
    ref = orc_mod.Oracle(cfg, w, "f64").greedy(prompts, G, want_logits=True, temperature=T, seed=seed, top_p=top_p)
    plain = orc_mod.Oracle(cfg, w, "f64").greedy(prompts, G, temperature=T, seed=seed)
    assert (ref["tokens"] != plain["tokens"]).any()             # the truncation changes this run
    model = srm.Model(cfg, w)
    got = _topp_run(model, prompts, G, T, top_p, seed, mode)
    absmax = np.abs(ref["logits"]).max(axis=2)
    bad = got != ref["tokens"]
    near = (ref["margin"] < 1e-4 * absmax) | (ref["mass_margin"] < MASS_TOL)
    # a tolerated near tie may change everything after it in that row: compare up to the first one
    for b in range(got.shape[0]):
        stop = np.argmax(near[b]) if near[b].any() else G
        assert not bad[b, :stop].any(), f"row {b} differs from the oracle before any near tie"
    assert near.sum() <= 2
    # top_p = 1 through the same entry point is plain sampling; temperature 0 is greedy
    np.testing.assert_array_equal(_topp_run(model, prompts, 6, T, 1.0, seed, mode), plain["tokens"][:, :6])
    greedy = orc_mod.Oracle(cfg, w, "f64").greedy(prompts, 6)
    np.testing.assert_array_equal(_topp_run(model, prompts, 6, 0.0, 0.9, seed, mode), greedy["tokens"])


def test_topp_step_bf16_rows_against_oracle_rule(srm, orc_mod):
    """bf16 MFMA head (several tiles): every row's token equals the oracle's nucleus choice from the
    GPU's own logits, and the uniform and ragged entry points agree bit for bit."""
    cfg = srm_synth.tiny_config(vocab=1500, d_model=128, n_layers=2, n_heads=4, n_ctx=16, weight_dtype="bf16", seed=31)
    w = srm_synth.make_weights(cfg, stress=True)
    w["head"] = srm_synth.round_to_bf16(w["head"] * 30.0)
    model = srm.Model(cfg, w)
    B, T, top_p, seed, pos = 700, 0.8, 0.7, 11, 3
    rng = np.random.default_rng(2)
    tok = to_dev(rng.integers(0, cfg.vocab, B).astype(np.int32))
    st0 = torch.randn(cfg.n_layers * B * cfg.d_model, device="cuda") * 0.1
    ws = model.new_workspace(B)
    lg = torch.empty((B, cfg.vocab), dtype=torch.float32, device="cuda")
    out = torch.empty(B, dtype=torch.int32, device="cuda")
    st = st0.clone()
    print(f"top-p bf16 step B={B}", flush=True)
    model.decode_step(B, pos, tok, st, out, logits=lg, workspace=ws, temperature=T, seed=seed, top_p=top_p)
    torch.cuda.synchronize()
    logits = lg.cpu().numpy()
    tolerated, changed = _check_rows(orc_mod, out.cpu().numpy(), logits, T, top_p, seed, lambda r: pos)
    assert tolerated <= 3 and changed > 0
    st2, out2 = st0.clone(), torch.empty_like(out)
    posr = torch.full((B,), pos, dtype=torch.int32, device="cuda")
    posr[5] = -1                                                # one idle slot
    model.decode_step_ragged(B, posr, tok, st2, out2, advance=True, temperature=T, seed=seed, top_p=top_p, logits=lg,
                             workspace=ws)
    torch.cuda.synchronize()
    live = torch.ones(B, dtype=torch.bool, device="cuda"); live[5] = False
    assert torch.equal(out2[live], out[live]) and int(out2[5]) == -1
    assert int(posr[5]) == -1 and (posr[live] == pos + 1).all()
    with pytest.raises(srm.SrmError):                           # the truncation needs the logits buffer
        model.decode_step(B, pos, tok, st, out, workspace=ws, temperature=T, seed=seed, top_p=top_p)

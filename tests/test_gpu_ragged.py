"""Ragged batches through the C ABI: prompts of different lengths packed back to
back, decode with one position per sample, slots that join and leave a running
batch.  Samples are independent, so the oracle's answer for a ragged batch is
simply each sample run alone on its own prompt."""
import numpy as np
import pytest
import torch

import srm_synth
from gpu_util import to_dev, rel_err_rows, check_tokens

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def srm():
    import paper_2605_08696_amd as pkg
    pkg.lib()
    return pkg


@pytest.fixture(scope="module")
def orc_mod(oracle_mod):
    return oracle_mod


@pytest.fixture(scope="module")
def c1(srm, orc_mod):
    cfg = srm_synth.CONFIGS["C1"]
    w = srm_synth.make_weights(cfg)
    return cfg, w, srm.Model(cfg, w), orc_mod.Oracle(cfg, w, "f64")


def _pack(prompts, lengths):
    toks = np.concatenate([prompts[i, :n] for i, n in enumerate(lengths)]).astype(np.int32)
    off = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    return toks, off


def _oracle_streams(orc, prompts, lengths, G, temperature=0.0, seed=0, slots=None):
    """Per sample: G tokens, logits, margins from the oracle run on that prompt alone."""
    out = []
    for i, n in enumerate(lengths):
        b = i if slots is None else slots[i]
        out.append(orc.greedy(prompts[i:i + 1, :n], G, want_logits=True, temperature=temperature, seed=seed, b0=b))
    return out


LENGTHS = [1, 5, 16, 9, 2, 12, 16, 3]


@pytest.mark.parametrize("small_ws", [False, True])
def test_ragged_prefill_then_ragged_decode_matches_oracle(c1, small_ws):
    cfg, w, model, orc = c1
    prompts = srm_synth.make_prompts(cfg)                      # [8][16]
    B, G = len(LENGTHS), 20
    ref = _oracle_streams(orc, prompts, LENGTHS, G)
    toks, off = _pack(prompts, LENGTHS)
    print(f"ragged prefill+decode B={B} lengths={LENGTHS} small_ws={small_ws}", flush=True)
    rows = 20 if small_ws else int(off[-1])                    # 20 rows: several passes of whole prompts
    ws = model.new_workspace(max(rows, B))
    st = model.new_state(B)
    st.fill_(float("nan"))                                     # every destination must be written
    tk = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    pos = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    lg = torch.empty((B, cfg.vocab), dtype=torch.float32, device="cuda")
    keep = model.prefill_ragged(to_dev(toks), off, st, tk, pos=pos, logits=lg, workspace=ws)
    torch.cuda.synchronize()
    del keep
    np.testing.assert_array_equal(pos.cpu().numpy(), LENGTHS)
    got = np.empty((B, G), np.int32)
    got[:, 0] = tk.cpu().numpy()
    first_logits = np.stack([r["logits"][0, 0] for r in ref])
    assert rel_err_rows(lg.cpu().numpy(), first_logits) <= 1e-4
    for g in range(1, G):
        model.decode_step_ragged(B, pos, tk, st, tk, advance=True, workspace=ws)
        got[:, g] = tk.cpu().numpy()
    np.testing.assert_array_equal(pos.cpu().numpy(), np.array(LENGTHS) + G - 1)
    for b in range(B):
        absmax = np.abs(ref[b]["logits"][0]).max(axis=1)
        assert check_tokens(got[b], ref[b]["tokens"][0], ref[b]["margin"][0], absmax) == 0
    # state after the last step against the oracle (the oracle consumed one token more: compare one step earlier
    # is not available, so run the oracle's own recurrence for G - 1 generated tokens)
    for b in (0, 2, 5):
        seq = np.concatenate([prompts[b, :LENGTHS[b]], ref[b]["tokens"][0, :G - 1]])[None, :]
        s_ref = orc.greedy(seq, 1)["state"][0]
        s_got = st.view(cfg.n_layers, B, cfg.d_model)[:, b, :].cpu().numpy()
        assert np.abs(s_got - s_ref).max() <= 1e-4 * np.abs(s_ref).max()


def test_ragged_equals_uniform_when_positions_agree(srm):
    """All samples at one position: the ragged step is bit-identical to srm_decode_step (bf16, several tiles)."""
    cfg = srm_synth.tiny_config(vocab=1000, d_model=128, n_layers=3, n_heads=4, n_ctx=32, weight_dtype="bf16", seed=5)
    w = srm_synth.make_weights(cfg, stress=True)
    model = srm.Model(cfg, w)
    B, P = 700, 6
    rng = np.random.default_rng(9)
    prompts = rng.integers(0, cfg.vocab, (B, P)).astype(np.int32)
    ws = model.new_workspace(B * P)
    sa, sb = model.new_state(B), model.new_state(B)
    ta = torch.empty(B, dtype=torch.int32, device="cuda")
    tb = torch.empty(B, dtype=torch.int32, device="cuda")
    print(f"ragged==uniform B={B} P={P}", flush=True)
    model.prefill(to_dev(prompts), 1, sa, ta, workspace=ws)
    pos = torch.empty(B, dtype=torch.int32, device="cuda")
    off = np.arange(B + 1, dtype=np.int32) * P
    keep = model.prefill_ragged(to_dev(prompts.reshape(-1)), off, sb, tb, pos=pos, workspace=ws)
    torch.cuda.synchronize()
    del keep
    assert torch.equal(ta, tb) and torch.equal(sa, sb)
    for g in range(4):
        model.decode_step(B, P + g, ta, sa, ta, workspace=ws)
        model.decode_step_ragged(B, pos, tb, sb, tb, advance=True, workspace=ws)
        assert torch.equal(ta, tb) and torch.equal(sa, sb)
    # sampled: same draws, since the counter is keyed on (seed, position, sample)
    for g in range(3):
        model.decode_step(B, P + 4 + g, ta, sa, ta, workspace=ws, temperature=0.9, seed=3)
        model.decode_step_ragged(B, pos, tb, sb, tb, advance=True, temperature=0.9, seed=3, workspace=ws)
        assert torch.equal(ta, tb) and torch.equal(sa, sb)


def test_slots_join_and_leave_a_running_batch(c1):
    """Six slots; four start, two are admitted later through a slot list, one leaves.  Every
    slot's stream equals the oracle's stream for its prompt; idle slots are untouched."""
    cfg, w, model, orc = c1
    prompts = srm_synth.make_prompts(cfg)
    S = 6
    first = {0: (0, 7), 2: (1, 16), 3: (2, 3), 5: (3, 11)}      # slot -> (prompt row, length)
    later = {1: (4, 5), 4: (5, 1)}
    G1, G2 = 5, 6
    ws = model.new_workspace(64)
    st = model.new_state(S)
    st.fill_(123.0)
    tk = torch.full((S,), 0, dtype=torch.int32, device="cuda")
    pos = torch.full((S,), -1, dtype=torch.int32, device="cuda")
    print("slots join/leave", flush=True)

    def admit(group):
        slots = sorted(group)
        rows = [group[s][0] for s in slots]; lens = [group[s][1] for s in slots]
        toks, off = _pack(prompts[rows], lens)
        keep = model.prefill_ragged(to_dev(toks), off, st, tk, slot=to_dev(np.array(slots, np.int32)), pos=pos,
                                    workspace=ws)
        torch.cuda.synchronize()
        del keep

    admit(first)
    sv = st.view(cfg.n_layers, S, cfg.d_model)
    assert (sv[:, 1] == 123.0).all() and (sv[:, 4] == 123.0).all()          # idle slots not written
    np.testing.assert_array_equal(pos.cpu().numpy(), [7, -1, 16, 3, -1, 11])
    streams = {s: [int(tk[s])] for s in first}
    for g in range(G1):
        model.decode_step_ragged(S, pos, tk, st, tk, advance=True, workspace=ws)
        t = tk.cpu().numpy()
        assert t[1] == -1 and t[4] == -1
        for s in first:
            streams[s].append(int(t[s]))
        tk[1] = 0; tk[4] = 0
    assert (sv[:, 1] == 123.0).all() and (sv[:, 4] == 123.0).all()
    # slot 3 leaves, slots 1 and 4 join
    pos[3] = -1
    frozen = sv[:, 3].clone()
    admit(later)
    for s in later:
        streams[s] = [int(tk[s])]
    for g in range(G2):
        model.decode_step_ragged(S, pos, tk, st, tk, advance=True, workspace=ws)
        t = tk.cpu().numpy()
        assert t[3] == -1
        for s in streams:
            if s != 3:
                streams[s].append(int(t[s]))
        tk[3] = 0
    assert torch.equal(sv[:, 3], frozen)
    everyone = dict(first); everyone.update(later)
    for s, (row, n) in everyone.items():
        ref = orc.greedy(prompts[row:row + 1, :n], len(streams[s]), want_logits=True)
        absmax = np.abs(ref["logits"][0]).max(axis=1)
        assert check_tokens(np.array(streams[s]), ref["tokens"][0], ref["margin"][0], absmax) == 0


def test_ragged_sampled_matches_oracle(c1):
    """Temperature sampling with per-sample positions: prefill all but the last prompt token,
    feed the last one to the first sampled step (a one-token prompt starts from the zero state)."""
    cfg, w, model, orc = c1
    prompts = srm_synth.make_prompts(cfg)
    B, G, T, seed = len(LENGTHS), 12, 0.7, 4242
    ref = _oracle_streams(orc, prompts, LENGTHS, G, temperature=T, seed=seed)
    ws = model.new_workspace(int(sum(LENGTHS)))
    st = model.new_state(B)
    st.zero_()
    tk = torch.zeros(B, dtype=torch.int32, device="cuda")
    pos = torch.zeros(B, dtype=torch.int32, device="cuda")
    has = [b for b in range(B) if LENGTHS[b] > 1]
    toks, off = _pack(prompts[has], [LENGTHS[b] - 1 for b in has])
    print(f"ragged sampled B={B}", flush=True)
    keep = model.prefill_ragged(to_dev(toks), off, st, tk, slot=to_dev(np.array(has, np.int32)), pos=pos, workspace=ws)
    torch.cuda.synchronize()
    del keep
    np.testing.assert_array_equal(pos.cpu().numpy(), np.array(LENGTHS) - 1)
    tk.copy_(to_dev(np.array([prompts[b, LENGTHS[b] - 1] for b in range(B)], np.int32)))
    got = np.empty((B, G), np.int32)
    for g in range(G):
        model.decode_step_ragged(B, pos, tk, st, tk, advance=True, temperature=T, seed=seed, workspace=ws)
        got[:, g] = tk.cpu().numpy()
    for b in range(B):
        absmax = np.abs(ref[b]["logits"][0]).max(axis=1)
        assert check_tokens(got[b], ref[b]["tokens"][0], ref[b]["margin"][0], absmax) == 0


def test_ragged_bf16_logits_against_oracle(srm, orc_mod):
    """bf16 model, 300 packed prompts of random lengths (several GEMM tiles, ragged tail):
    first-token logits and two decode steps of sampled rows against the oracle."""
    cfg = srm_synth.tiny_config(vocab=500, d_model=128, n_layers=3, n_heads=4, n_ctx=24, weight_dtype="bf16", seed=8)
    w = srm_synth.make_weights(cfg)
    model = srm.Model(cfg, w)
    orc = orc_mod.Oracle(cfg, w, "f64")
    rng = np.random.default_rng(11)
    N = 300
    lens = rng.integers(1, 17, N)
    prompts = rng.integers(0, cfg.vocab, (N, 16)).astype(np.int32)
    toks, off = _pack(prompts, lens)
    ws = model.new_workspace(int(off[-1]))
    st = model.new_state(N)
    tk = torch.empty(N, dtype=torch.int32, device="cuda")
    pos = torch.empty(N, dtype=torch.int32, device="cuda")
    lg = torch.empty((N, cfg.vocab), dtype=torch.float32, device="cuda")
    print(f"ragged bf16 N={N} rows={int(off[-1])}", flush=True)
    keep = model.prefill_ragged(to_dev(toks), off, st, tk, pos=pos, logits=lg, workspace=ws)
    torch.cuda.synchronize()
    del keep
    rows = [0, 1, 17, 150, 298, 299]
    steps = [lg.cpu().numpy()]
    forced = {b: orc.greedy(prompts[b:b + 1, :lens[b]], 3, want_logits=True) for b in rows}
    for g in range(2):
        for b in rows:                                       # teacher-force the checked rows on the oracle's tokens
            tk[b] = int(forced[b]["tokens"][0, g])
        model.decode_step_ragged(N, pos, tk, st, tk, advance=True, logits=lg, workspace=ws)
        steps.append(lg.cpu().numpy())
    for b in rows:
        for g in range(3):
            assert rel_err_rows(steps[g][b][None], forced[b]["logits"][0, g][None]) <= 2e-2
    t = tk.cpu().numpy()
    assert ((t >= 0) & (t < cfg.vocab)).all() and bool(torch.isfinite(st).all())


@pytest.mark.parametrize("B", [13000, 66000])
def test_ragged_decode_large_batch_fused_equals_separate(srm, B, monkeypatch):
    """13 000 samples of width 1024 (the in-projection takes the 256x256 tile, the state update rides in its
    epilogue) and 66 000 (more tiles than compute units: the persistent form of that tile) at per-sample
    positions, idle slots (-1) included: the same states, tokens and positions as with the separate ragged
    state-update kernel, and idle samples untouched."""
    cfg = srm_synth.tiny_config(vocab=300, d_model=1024, n_layers=1, n_heads=4, n_ctx=8, weight_dtype="bf16", seed=9)
    w = srm_synth.make_weights(cfg, stress=True)
    model = srm.Model(cfg, w)
    rng = np.random.default_rng(12)
    pos0 = rng.integers(-1, cfg.n_ctx - 2, B).astype(np.int32)
    tok0 = rng.integers(0, cfg.vocab, B).astype(np.int32)
    S0 = rng.standard_normal((cfg.n_layers, B, cfg.d_model)).astype(np.float32)
    ws = model.new_workspace(B)
    res = []
    for fuse in (True, False):
        if not fuse:
            monkeypatch.setenv("SRM_FUSE_MIXER", "0")
        st, tk, pos = to_dev(S0), to_dev(tok0), to_dev(pos0)
        print(f"ragged large batch B={B} fuse={fuse}", flush=True)
        for _ in range(2):
            model.decode_step_ragged(B, pos, tk, st, tk, advance=True, workspace=ws)
        torch.cuda.synchronize()
        res.append((st.cpu().numpy(), tk.cpu().numpy(), pos.cpu().numpy()))
    for a, b in zip(res[0], res[1]):
        np.testing.assert_array_equal(a, b)
    st, tk, pos = res[0]
    idle = pos0 < 0
    assert idle.any() and (~idle).any()
    np.testing.assert_array_equal(st[:, idle], S0[:, idle])
    np.testing.assert_array_equal(pos[idle], pos0[idle])
    np.testing.assert_array_equal(pos[~idle], pos0[~idle] + 2)
    assert not np.array_equal(st[:, ~idle], S0[:, ~idle])


@pytest.mark.parametrize("d,B", [(256, 40), (512, 300)])
def test_ragged_decode_with_token_mixing_in_one_kernel(srm, d, B, monkeypatch):
    """bf16 model, a few dozen to a few hundred slots at their own positions (idle ones included): the ragged step
    whose token mixing is one kernel per layer against the ragged step of separate kernels (the library's switch):
    the same positions, states and logits to bf16 rounding, idle slots untouched bit for bit."""
    cfg = srm_synth.tiny_config(vocab=200, d_model=d, n_layers=3, n_heads=4, n_ctx=12, weight_dtype="bf16", seed=14)
    w = srm_synth.make_weights(cfg, stress=True)
    model = srm.Model(cfg, w)
    rng = np.random.default_rng(15 + B)
    pos0 = rng.integers(-1, cfg.n_ctx - 3, B).astype(np.int32)
    tok0 = rng.integers(0, cfg.vocab, B).astype(np.int32)
    S0 = rng.standard_normal((cfg.n_layers, B, cfg.d_model)).astype(np.float32)
    ws = model.new_workspace(B)
    res = []
    for mode in ("1", "0"):
        monkeypatch.setenv("SRM_TOKEN_MIX", mode)
        st, tk, pos = to_dev(S0), to_dev(tok0), to_dev(pos0)
        lg = torch.empty((B, cfg.vocab), dtype=torch.float32, device="cuda")
        print(f"ragged token mixing d={d} B={B} SRM_TOKEN_MIX={mode}", flush=True)
        steps = []
        for _ in range(3):
            # (teacher-forced on tok0: a token that flips between the two forms would make the later steps incomparable)
            model.decode_step_ragged(B, pos, to_dev(tok0), st, tk, advance=True, logits=lg, workspace=ws)
            steps.append(lg.clone())
        torch.cuda.synchronize()
        res.append((st.cpu().numpy(), pos.cpu().numpy(), [x.cpu().numpy() for x in steps]))
    idle = pos0 < 0
    assert idle.any() and (~idle).any()
    np.testing.assert_array_equal(res[0][1], res[1][1])
    np.testing.assert_array_equal(res[0][0][:, idle], S0[:, idle])
    assert np.abs(res[0][0] - res[1][0]).max() <= 2e-2 * np.abs(res[1][0]).max()
    for a, b in zip(res[0][2], res[1][2]):
        assert rel_err_rows(a[~idle], b[~idle]) <= 2e-2
    model.close()


def test_ragged_decode_of_a_handful_of_samples_without_layernorm_launches(srm, monkeypatch):
    """bf16 model, 6 slots at their own positions (one idle): the ragged step whose LayerNorms are made by the
    consuming GEMMs equals the ragged step with LayerNorm launches (the library's switch) bit for bit."""
    cfg = srm_synth.tiny_config(vocab=200, d_model=256, n_layers=3, n_heads=4, n_ctx=12, weight_dtype="bf16", seed=10)
    w = srm_synth.make_weights(cfg, stress=True)
    model = srm.Model(cfg, w)
    B = 6
    rng = np.random.default_rng(13)
    pos0 = np.array([0, 3, -1, 7, 2, 5], np.int32)
    tok0 = rng.integers(0, cfg.vocab, B).astype(np.int32)
    S0 = rng.standard_normal((cfg.n_layers, B, cfg.d_model)).astype(np.float32)
    ws = model.new_workspace(B)
    res = []
    for on_load in (True, False):
        if not on_load:
            monkeypatch.setenv("SRM_LN_ON_LOAD", "0")
        st, tk, pos = to_dev(S0), to_dev(tok0), to_dev(pos0)
        lg = torch.empty((B, cfg.vocab), dtype=torch.float32, device="cuda")
        print(f"ragged handful B={B} on_load={on_load}", flush=True)
        for _ in range(3):
            model.decode_step_ragged(B, pos, tk, st, tk, advance=True, logits=lg, workspace=ws)
        torch.cuda.synchronize()
        res.append((st.cpu().numpy(), tk.cpu().numpy(), pos.cpu().numpy(), lg.cpu().numpy()[pos0 >= 0]))
    for a, b in zip(res[0], res[1]):
        np.testing.assert_array_equal(a, b)
    np.testing.assert_array_equal(res[0][0][:, 2], S0[:, 2])          # the idle slot's state is untouched
    assert np.isfinite(res[0][3]).all()


def test_ragged_errors(c1, srm):
    cfg, w, model, orc = c1
    ws = model.new_workspace(32)
    st = model.new_state(4)
    tk = torch.zeros(4, dtype=torch.int32, device="cuda")
    toks = torch.zeros(64, dtype=torch.int32, device="cuda")
    with pytest.raises(srm.SrmError):                         # empty prompt
        model.prefill_ragged(toks, [0, 3, 3, 5], st, tk, workspace=ws)
    with pytest.raises(srm.SrmError):                         # longer than n_ctx
        model.prefill_ragged(torch.zeros(600, dtype=torch.int32, device="cuda"), [0, cfg.n_ctx + 1], st, tk,
                             workspace=model.new_workspace(600))
    with pytest.raises(srm.SrmError):                         # more prompts than samples in the state
        model.prefill_ragged(toks, [0, 1, 2, 3, 4, 5], st, tk, workspace=ws)
    with pytest.raises(srm.SrmError):                         # one prompt larger than the workspace
        model.prefill_ragged(toks, [0, 40], st, tk, workspace=ws)
    with pytest.raises(srm.SrmError):                         # slot list with fan-out
        model.prefill_ragged(toks, [0, 2], st, tk, fanout_k=2, slot=torch.zeros(1, dtype=torch.int32, device="cuda"),
                             workspace=ws)
    with pytest.raises(srm.SrmError):                         # workspace too small for the batch
        model.decode_step_ragged(4, tk, tk, st, tk, workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    torch.cuda.synchronize()


# ---- chunked scan: prefill of few, long prompts ------------------------------------------------
@pytest.mark.parametrize("N,P", [(1, 256), (2, 200), (3, 65)])
def test_chunked_scan_prefill_matches_oracle_and_decode_steps(c1, N, P):
    """Few long prompts take the chunked mixer scan; it must agree with the oracle's recurrence
    and, to fp32 rounding, with P single decode steps."""
    cfg, w, model, orc = c1
    rng = np.random.default_rng(100 + P)
    prompts = rng.integers(0, cfg.vocab, (N, P)).astype(np.int32)
    ref = orc.greedy(prompts, 1, want_logits=True)
    print(f"chunked scan prefill N={N} P={P}", flush=True)
    ws = model.new_workspace(N * P)
    st, tk = model.new_state(N), torch.empty(N, dtype=torch.int32, device="cuda")
    lg = torch.empty((N, cfg.vocab), dtype=torch.float32, device="cuda")
    st.fill_(float("nan"))
    model.prefill(to_dev(prompts), 1, st, tk, logits=lg, workspace=ws)
    torch.cuda.synchronize()
    assert rel_err_rows(lg.cpu().numpy(), ref["logits"][:, 0]) <= 1e-4
    s_got = st.view(cfg.n_layers, N, cfg.d_model).permute(1, 0, 2).cpu().numpy()
    assert np.abs(s_got - ref["state"]).max() <= 1e-4 * np.abs(ref["state"]).max()
    absmax = np.abs(ref["logits"][:, 0]).max(axis=1)
    assert check_tokens(tk.cpu().numpy(), ref["tokens"][:, 0], ref["margin"][:, 0], absmax) == 0
    # against the step-by-step path
    st_b, tk_b = model.new_state(N), torch.empty(N, dtype=torch.int32, device="cuda")
    st_b.zero_()
    pc = to_dev(prompts).t().contiguous()
    for t in range(P):
        model.decode_step(N, t, pc[t], st_b, tk_b, workspace=ws)
    torch.cuda.synchronize()
    assert (st - st_b).abs().max() <= 1e-5 * st_b.abs().max()
    # a workspace that holds one prompt per pass gives the same bits (the chunking depends on the call only)
    st_c, tk_c = model.new_state(N), torch.empty(N, dtype=torch.int32, device="cuda")
    model.prefill(to_dev(prompts), 1, st_c, tk_c, workspace=torch.empty(model.workspace_bytes(P), dtype=torch.uint8,
                                                                         device="cuda"))
    torch.cuda.synchronize()
    assert torch.equal(st, st_c) and torch.equal(tk, tk_c)


def test_chunked_scan_ragged_prompts(c1):
    cfg, w, model, orc = c1
    lens = [200, 77, 1, 130, 16]
    rng = np.random.default_rng(7)
    prompts = rng.integers(0, cfg.vocab, (len(lens), 200)).astype(np.int32)
    toks, off = _pack(prompts, lens)
    N = len(lens)
    ws = model.new_workspace(int(off[-1]))
    st, tk = model.new_state(N), torch.empty(N, dtype=torch.int32, device="cuda")
    st.fill_(float("nan"))
    lg = torch.empty((N, cfg.vocab), dtype=torch.float32, device="cuda")
    print(f"chunked scan ragged lens={lens}", flush=True)
    keep = model.prefill_ragged(to_dev(toks), off, st, tk, logits=lg, workspace=ws)
    torch.cuda.synchronize()
    del keep
    sv = st.view(cfg.n_layers, N, cfg.d_model)
    for b, n in enumerate(lens):
        ref = orc.greedy(prompts[b:b + 1, :n], 1, want_logits=True)
        assert rel_err_rows(lg[b:b + 1].cpu().numpy(), ref["logits"][:, 0]) <= 1e-4
        assert np.abs(sv[:, b].cpu().numpy() - ref["state"][0]).max() <= 1e-4 * np.abs(ref["state"][0]).max()
        assert int(tk[b]) == int(ref["tokens"][0, 0])


def test_skewed_lengths_fall_back_to_the_sequential_scan(c1, srm):
    """Many one-token prompts next to a long one: the chunk count of the chunked scan follows the long prompt,
    its scratch the few rows of the pass, so the call must take the sequential scan (and stay inside the
    workspace).  Checked against the oracle on the long prompt and some short ones."""
    cfg, w, model, orc = c1
    lens = [1] * 120 + [200]
    rng = np.random.default_rng(11)
    prompts = rng.integers(0, cfg.vocab, (len(lens), 200)).astype(np.int32)
    toks, off = _pack(prompts, lens)
    N = len(lens)
    ws = model.new_workspace(int(off[-1]))
    plan = srm.prefill_ragged_plan(cfg, off, ws.numel())
    assert plan["chunk_len_by_shape"] > 0 and plan["chunk_len"] == 0 and plan["scratch_need"] > plan["scratch_room"]
    st, tk = model.new_state(N), torch.empty(N, dtype=torch.int32, device="cuda")
    st.fill_(float("nan"))
    lg = torch.empty((N, cfg.vocab), dtype=torch.float32, device="cuda")
    guard = torch.full((1 << 20,), 7, dtype=torch.uint8, device="cuda")     # allocated right after the workspace
    print(f"skewed ragged prefill, {N} prompts, plan {plan}", flush=True)
    keep = model.prefill_ragged(to_dev(toks), off, st, tk, logits=lg, workspace=ws)
    torch.cuda.synchronize()
    del keep
    assert bool((guard == 7).all())
    sv = st.view(cfg.n_layers, N, cfg.d_model)
    for b in (0, 1, 59, 119, 120):
        ref = orc.greedy(prompts[b:b + 1, :lens[b]], 1, want_logits=True)
        assert rel_err_rows(lg[b:b + 1].cpu().numpy(), ref["logits"][:, 0]) <= 1e-4
        assert np.abs(sv[:, b].cpu().numpy() - ref["state"][0]).max() <= 1e-4 * np.abs(ref["state"][0]).max()
        assert int(tk[b]) == int(ref["tokens"][0, 0])


def test_chunked_scan_bf16(srm, orc_mod):
    cfg = srm_synth.tiny_config(vocab=300, d_model=128, n_layers=3, n_heads=4, n_ctx=160, weight_dtype="bf16", seed=13)
    w = srm_synth.make_weights(cfg, stress=True)
    model = srm.Model(cfg, w)
    orc = orc_mod.Oracle(cfg, w, "f64")
    N, P = 4, 150
    prompts = np.random.default_rng(3).integers(0, cfg.vocab, (N, P)).astype(np.int32)
    ref = orc.greedy(prompts, 1, want_logits=True)
    ws = model.new_workspace(N * P)
    st, tk = model.new_state(N), torch.empty(N, dtype=torch.int32, device="cuda")
    lg = torch.empty((N, cfg.vocab), dtype=torch.float32, device="cuda")
    print(f"chunked scan bf16 N={N} P={P}", flush=True)
    model.prefill(to_dev(prompts), 1, st, tk, logits=lg, workspace=ws)
    torch.cuda.synchronize()
    assert rel_err_rows(lg.cpu().numpy(), ref["logits"][:, 0]) <= 2e-2
    s_got = st.view(cfg.n_layers, N, cfg.d_model).permute(1, 0, 2).cpu().numpy()
    assert np.abs(s_got - ref["state"]).max() <= 2e-2 * np.abs(ref["state"]).max()


def test_generate_ragged_stops_samples_at_eos(c1):
    """The device-side serving loop: ragged prompts, G steps per call with graph replay, a sample
    that emits the end token goes idle.  Two calls in a row continue each other."""
    cfg, w, model, orc = c1
    prompts = srm_synth.make_prompts(cfg)
    B, G = len(LENGTHS), 20
    ref = _oracle_streams(orc, prompts, LENGTHS, G)
    streams = np.stack([r["tokens"][0] for r in ref])            # [B][G], index 0 = token after the prompt
    # an end token that some stream emits after its first token, and none emits first
    cand = [int(t) for t in streams[:, 3:9].ravel() if t not in streams[:, 0]]
    eos = cand[0]
    want = np.full((B, G - 1), -1, np.int64)
    end_pos = np.zeros(B, np.int64)
    for b in range(B):
        hit = [j for j in range(1, G) if streams[b, j] == eos]
        stop = hit[0] if hit else G - 1
        want[b, :stop] = streams[b, 1:stop + 1]
        end_pos[b] = -1 if hit else LENGTHS[b] + G - 1
    assert (want == -1).any() and (want[:, -1] != -1).any()
    toks, off = _pack(prompts, LENGTHS)
    ws = model.new_workspace(int(off[-1]))
    print(f"generate_ragged B={B} eos={eos}", flush=True)
    for split in (None, 8):                                      # one call of 19 steps; 8 + 11 steps
        st = model.new_state(B)
        tk = torch.empty(B, dtype=torch.int32, device="cuda")
        pos = torch.empty(B, dtype=torch.int32, device="cuda")
        keep = model.prefill_ragged(to_dev(toks), off, st, tk, pos=pos, workspace=ws)
        torch.cuda.synchronize()
        del keep
        out = torch.full((G - 1, B), -7, dtype=torch.int32, device="cuda")
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            if split is None:
                model.generate_ragged(B, G - 1, pos, tk, st, out, eos_id=eos, workspace=ws)
            else:
                model.generate_ragged(B, split, pos, tk, st, out[:split], eos_id=eos, workspace=ws)
                # idle samples keep emitting -1 as their token: feed something valid
                tk.clamp_(min=0)
                model.generate_ragged(B, G - 1 - split, pos, tk, st, out[split:], eos_id=eos, workspace=ws)
        side.synchronize()
        np.testing.assert_array_equal(out.cpu().numpy().T, want)
        np.testing.assert_array_equal(pos.cpu().numpy(), end_pos)

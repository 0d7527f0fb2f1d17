"""Kernel-level GPU checks through the C ABI: the GEMM with each fused epilogue
and each tile shape, the argmax tie rule, and the recurrent state update
against the oracle's mixer step."""
import numpy as np
import pytest
import torch

import srm_synth
from gpu_util import to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def srm():
    import paper_2605_08696_amd as pkg
    pkg.lib()
    return pkg


def _gelu(x):
    import scipy.special
    return x * scipy.special.ndtr(x)


def _linear_case(srm, dtype, M, N, K, epi, tile, seed):
    rng = np.random.default_rng(seed)
    A = rng.standard_normal((M, K)).astype(np.float32)
    W = (rng.standard_normal((N, K)) / np.sqrt(K)).astype(np.float32)
    bias = rng.standard_normal(N).astype(np.float32)
    if dtype == srm.SRM_BF16:
        A, W = srm_synth.round_to_bf16(A), srm_synth.round_to_bf16(W)
    tt = torch.bfloat16 if dtype == srm.SRM_BF16 else torch.float32
    dA, dW, dB = to_dev(A, tt), to_dev(W, tt), to_dev(bias)
    ref = A.astype(np.float64) @ W.astype(np.float64).T + bias
    print(f"linear dtype={dtype} M={M} N={N} K={K} epi={epi} tile={tile}", flush=True)
    if epi in (0, 1):
        out = torch.full((M, N), 7.0, dtype=tt, device="cuda")
        srm.linear(dtype, epi, dA, dW, dB, out=out, tile=tile)
        want = ref if epi == 0 else _gelu(ref)
        got = out.float().cpu().numpy()
        tol = 2.0 ** -8 if dtype == srm.SRM_BF16 else 2e-6
        assert np.abs(got - want).max() <= tol * max(1.0, np.abs(want).max())
    elif epi == 2:
        base = rng.standard_normal((M, N)).astype(np.float32)
        out = to_dev(base)
        srm.linear(dtype, 2, dA, dW, dB, out=out, tile=tile)
        got = out.cpu().numpy()
        assert np.abs(got - (ref + base)).max() <= 4e-6 * np.abs(ref).max() + 1e-6
    elif epi == 4:
        out = torch.zeros((M, N), dtype=torch.float32, device="cuda")
        srm.linear(dtype, 4, dA, dW, dB, out=out, tile=tile)
        assert np.abs(out.cpu().numpy() - ref).max() <= 4e-6 * np.abs(ref).max()
    else:
        out = torch.zeros((M, N), dtype=torch.float32, device="cuda")
        am = torch.full((M,), -1, dtype=torch.int32, device="cuda")
        scratch = torch.empty(srm.linear_scratch_bytes(M, N), dtype=torch.uint8, device="cuda")
        srm.linear(dtype, 3, dA, dW, dB, out=out, argmax=am, scratch=scratch, tile=tile)
        got = out.cpu().numpy()
        assert np.abs(got - ref).max() <= 4e-6 * np.abs(ref).max()
        # argmax is decided on the kernel's own fp32 logits
        np.testing.assert_array_equal(am.cpu().numpy(), got.argmax(axis=1))
        am2 = torch.full((M,), -1, dtype=torch.int32, device="cuda")
        srm.linear(dtype, 3, dA, dW, dB, out=None, argmax=am2, scratch=scratch, tile=tile)
        np.testing.assert_array_equal(am2.cpu().numpy(), got.argmax(axis=1))
    torch.cuda.synchronize()


@pytest.mark.parametrize("tile", [0, 1, 2, 3, 4])
@pytest.mark.parametrize("epi", [0, 1, 2, 3, 4])
def test_linear_bf16_tiles_and_epilogues(srm, tile, epi):
    # several tiles in both directions plus ragged edges in M and N
    _linear_case(srm, srm.SRM_BF16, 300, 328, 192, epi, tile, seed=10 * tile + epi)


@pytest.mark.parametrize("shape", [(1, 64, 64), (37, 130, 64), (513, 1000, 256), (1024, 512, 1024)])
def test_linear_bf16_auto_tile_shapes(srm, shape):
    M, N, K = shape
    for epi in (0, 3):
        _linear_case(srm, srm.SRM_BF16, M, N, K, epi, None, seed=M + N)


@pytest.mark.parametrize("shape", [(1, 5, 3), (8, 256, 256), (70, 130, 37), (128, 64, 100), (5, 130, 64), (17, 70, 128),
                                   (32, 4096, 256), (33, 64, 64)])
@pytest.mark.parametrize("epi", [0, 1, 2, 3, 4])
def test_linear_fp32(srm, shape, epi):
    M, N, K = shape
    _linear_case(srm, srm.SRM_FP32, M, N, K, epi, None, seed=M * 7 + epi)


@pytest.mark.parametrize("dtype_name", ["fp32", "bf16"])
def test_argmax_ties_go_to_the_lowest_index(srm, dtype_name):
    dtype = srm.SRM_BF16 if dtype_name == "bf16" else srm.SRM_FP32
    tt = torch.bfloat16 if dtype_name == "bf16" else torch.float32
    M, N, K = 9, 700, 64
    rng = np.random.default_rng(3)
    A = srm_synth.round_to_bf16(rng.standard_normal((M, K)).astype(np.float32))
    W = srm_synth.round_to_bf16(rng.standard_normal((N, K)).astype(np.float32) * 0.1)
    # plant identical rows far apart (different column tiles and lanes): exact ties
    W[650] = W[17]; W[300] = W[17]
    W[17] *= 0; W[300] *= 0; W[650] *= 0
    bias = np.zeros(N, np.float32); bias[[17, 300, 650]] = 100.0     # all three tie at the top
    am = torch.full((M,), -1, dtype=torch.int32, device="cuda")
    scratch = torch.empty(srm.linear_scratch_bytes(M, N), dtype=torch.uint8, device="cuda")
    srm.linear(dtype, 3, to_dev(A, tt), to_dev(W, tt), to_dev(bias), out=None, argmax=am, scratch=scratch)
    np.testing.assert_array_equal(am.cpu().numpy(), np.full(M, 17))


@pytest.mark.parametrize("dtype_name", ["fp32", "bf16"])
@pytest.mark.parametrize("B", [1, 5, 1000, 4099])
def test_state_update_matches_oracle_step(srm, dtype_name, B):
    from oracle import srm_oracle
    d = 128 if dtype_name == "bf16" else 48
    H = 4
    cfg = srm_synth.tiny_config(vocab=16, d_model=d, n_layers=2, n_heads=H, n_ctx=8,
                                weight_dtype=dtype_name, seed=31)
    w = srm_synth.make_weights(cfg, stress=True)
    orc = srm_oracle.Oracle(cfg, w, "f64")
    model = srm.Model(cfg, w)
    rng = np.random.default_rng(B)
    u = rng.standard_normal((B, d)).astype(np.float32)
    if dtype_name == "bf16":
        u = srm_synth.round_to_bf16(u)
    S0 = rng.standard_normal((B, d)).astype(np.float32)
    layer, pos = 1, 5
    lw = w["layers"][layer]
    S_ref = S0.astype(np.float64)
    m_ref = np.empty((B, d))
    for b in range(B):
        m_ref[b] = orc.mixer_step(S_ref[b], u[b], lw["alpha"][:, pos], lw["beta"][:, pos], lw["lam"])
    print(f"state_update {dtype_name} B={B}", flush=True)
    dS = to_dev(S0)
    du = to_dev(u, model.act_dtype)
    dm = torch.empty_like(du)
    model.mixer_update(layer, pos, B, du, dS, dm)
    torch.cuda.synchronize()
    assert np.abs(dS.cpu().numpy() - S_ref).max() <= 4e-7 * np.abs(S_ref).max()
    tol = 2.0 ** -8 if dtype_name == "bf16" else 4e-7
    assert np.abs(dm.float().cpu().numpy() - m_ref).max() <= tol * np.abs(m_ref).max()
    # second call continues from the updated state (in-place semantics)
    for b in range(B):
        orc.mixer_step(S_ref[b], u[b], lw["alpha"][:, pos + 1], lw["beta"][:, pos + 1], lw["lam"])
    model.mixer_update(layer, pos + 1, B, du, dS, dm)
    torch.cuda.synchronize()
    assert np.abs(dS.cpu().numpy() - S_ref).max() <= 8e-7 * np.abs(S_ref).max()


@pytest.mark.parametrize("dtype_name,d,B", [("fp32", 48, 5), ("fp32", 64, 700), ("bf16", 128, 5), ("bf16", 512, 1000),
                                            ("bf16", 1024, 4099), ("bf16", 1024, 13000)])
@pytest.mark.parametrize("half_state", [False, True])
def test_project_update_equals_projection_then_update(srm, dtype_name, d, B, half_state):
    """srm_mixer_project_update (in-projection with the state update in its epilogue, every tile shape up to the
    256x256 one at 13000 rows) against srm_linear with the same W_in followed by srm_mixer_update: the same bits
    in the state and in the mixer output, and both against the oracle's step on sampled rows."""
    from oracle import srm_oracle
    if half_state and dtype_name == "fp32" and B > 100:
        pytest.skip("one binary16 case per weight type is enough")
    cfg = srm_synth.tiny_config(vocab=16, d_model=d, n_layers=2, n_heads=4, n_ctx=8, weight_dtype=dtype_name, seed=77,
                                state_dtype="fp16" if half_state else "fp32")
    w = srm_synth.make_weights(cfg, stress=True)
    model = srm.Model(cfg, w)
    rng = np.random.default_rng(B + d)
    a = rng.standard_normal((B, d)).astype(np.float32)
    if dtype_name == "bf16":
        a = srm_synth.round_to_bf16(a)
    S0 = rng.standard_normal((B, d)).astype(np.float32)
    layer, pos = 1, 6
    lw = w["layers"][layer]
    st_t = torch.float16 if half_state else torch.float32
    da = to_dev(a, model.act_dtype)
    S_f = to_dev(S0).to(st_t)
    S_s = S_f.clone()
    m_f = torch.empty((B, d), dtype=model.act_dtype, device="cuda")
    m_s = torch.empty_like(m_f)
    u = torch.empty_like(m_f)
    print(f"project_update {dtype_name} d={d} B={B} half={half_state}", flush=True)
    model.mixer_project_update(layer, pos, B, da, S_f, m_f)
    dt = srm.SRM_BF16 if dtype_name == "bf16" else srm.SRM_FP32
    srm.linear(dt, 0, da, to_dev(lw["w_in"], model.act_dtype), to_dev(lw["b_in"]), out=u)
    model.mixer_update(layer, pos, B, u, S_s, m_s)
    torch.cuda.synchronize()
    if dtype_name == "bf16":
        assert torch.equal(S_f, S_s) and torch.equal(m_f, m_s)
    else:       # fp32: the few-row GEMV and the tile kernel may sum k in different orders
        assert (S_f.float() - S_s.float()).abs().max() <= 2e-6 * S_s.float().abs().max()
        assert (m_f - m_s).abs().max() <= 2e-6 * m_s.abs().max()
    orc = srm_oracle.Oracle(cfg, w, "f64")
    for b in sorted({0, B // 3, B - 1}):
        S_ref = S0[b].astype(np.float16 if half_state else np.float32).astype(np.float64)
        u_ref = lw["w_in"].astype(np.float64) @ a[b].astype(np.float64) + lw["b_in"]
        m_ref = orc.mixer_step(S_ref, u_ref, lw["alpha"][:, pos], lw["beta"][:, pos], lw["lam"])
        tol = 2e-2 if dtype_name == "bf16" or half_state else 1e-5
        assert np.abs(S_f[b].float().cpu().numpy() - S_ref).max() <= tol * np.abs(S_ref).max()
        assert np.abs(m_f[b].float().cpu().numpy() - m_ref).max() <= tol * np.abs(m_ref).max()


def test_error_codes_on_the_gpu(srm):
    cfg = srm_synth.tiny_config(vocab=32, d_model=16, n_layers=1, n_heads=2, n_ctx=16)
    model = srm.Model(cfg, srm_synth.make_weights(cfg))
    B = 3
    st = model.new_state(B)
    ws = model.new_workspace(B)
    tok = torch.zeros(B, dtype=torch.int32, device="cuda")
    with pytest.raises(srm.SrmError) as e:
        model.decode_step(B, 16, tok, st, tok, workspace=ws)          # pos == n_ctx
    assert e.value.code == -1
    with pytest.raises(srm.SrmError) as e:
        model.decode_step(B, 0, tok, st, tok, workspace=ws[:64])      # workspace too small
    assert e.value.code == -2
    with pytest.raises(srm.SrmError):
        model.prefill(torch.zeros((2, 17), dtype=torch.int32, device="cuda"), 1, model.new_state(2),
                      torch.zeros(2, dtype=torch.int32, device="cuda"), workspace=model.new_workspace(64))
    assert model.state_bytes(7) == cfg.n_layers * 7 * cfg.d_model * 4


@pytest.mark.parametrize("tile", [0, 1, 2, 3, 4])
@pytest.mark.parametrize("epi", [0, 1, 2, 3, 4])
def test_linear_bf16_interior_tiles(srm, tile, epi):
    """Shapes that are whole multiples of every tile: the epilogues take their no-edge paths."""
    _linear_case(srm, srm.SRM_BF16, 512, 768, 128, epi, tile, seed=300 + 10 * tile + epi)


def test_linear_bf16_interior_tiles_n_multiple_of_4_only(srm):
    _linear_case(srm, srm.SRM_BF16, 256, 260, 64, 0, 2, seed=41)
    _linear_case(srm, srm.SRM_BF16, 256, 260, 64, 1, 2, seed=42)


@pytest.mark.parametrize("streaming", [True, False])
@pytest.mark.parametrize("nbytes", [16, 4096 * 16 + 48, 64 << 20])
def test_probe_copy_copies(srm, streaming, nbytes):
    print(f"probe_copy bytes={nbytes} streaming={streaming}", flush=True)
    src = torch.randint(0, 255, (nbytes + 32,), dtype=torch.uint8, device="cuda")
    dst = torch.full((nbytes + 32,), 255, dtype=torch.uint8, device="cuda")
    moved = srm.probe_copy(dst[:nbytes], src[:nbytes], streaming=streaming)
    torch.cuda.synchronize()
    assert moved == 2 * nbytes
    assert torch.equal(dst[:nbytes], src[:nbytes]) and (dst[nbytes:] == 255).all()
    with pytest.raises(srm.SrmError):
        srm.probe_copy(dst[:24], src[:24])


def test_probe_mfma_counts_every_product(srm):
    blocks, iters = 3, 1000
    out = torch.zeros(blocks * 256, device="cuda")
    print(f"probe_mfma blocks={blocks} iters={iters}", flush=True)
    flop = srm.probe_mfma(out, blocks, iters)
    torch.cuda.synchronize()
    assert flop == blocks * 4 * iters * 4 * 2.0 * 32 * 32 * 16
    assert (out == 1024.0 * iters).all()          # 64 accumulator registers per lane, each 16 * iters
    assert srm.probe_mfma(out, blocks, iters, random_operands=True) == flop
    torch.cuda.synchronize()
    assert torch.isfinite(out).all() and not (out == 1024.0 * iters).all()
    with pytest.raises(srm.SrmError):
        srm.probe_mfma(out, 0, iters)


@pytest.mark.parametrize("dtype_name", ["fp32", "bf16"])
@pytest.mark.parametrize("epi", [0, 1, 2, 3, 4])
@pytest.mark.parametrize("shape", [(1, 16, 64), (3, 70, 128), (8, 1000, 1024), (16, 130, 4096), (11, 32000, 512)])
def test_linear_few_rows_streaming_gemv(srm, dtype_name, epi, shape):
    """A handful of rows: fp32 takes the streaming GEMV (every epilogue, ragged column counts, one and two
    passes of eight rows, the widest K its LDS stage holds, 16- and 64-column blocks), bf16 the 64x64 MFMA tile
    with mostly empty rows."""
    M, N, K = shape
    dtype = srm.SRM_BF16 if dtype_name == "bf16" else srm.SRM_FP32
    _linear_case(srm, dtype, M, N, K, epi, None, seed=1000 + M + epi)


def test_linear_fp32_more_rows_than_one_pass(srm):
    for M in (9, 24, 32):
        _linear_case(srm, srm.SRM_FP32, M, 200, 256, 2, None, seed=M)


@pytest.mark.parametrize("shape", [(4400, 4000, 256), (700, 520, 384), (8200, 6000, 256)])
@pytest.mark.parametrize("epi", [0, 1, 2, 3, 4])
def test_linear_bf16_persistent_kernel(srm, shape, epi):
    """The persistent 256x256 kernel (tile code 9): fewer tiles than CUs, a few more (some work-groups take two),
    and three to four per work-group, ragged in M and N, four and six k tiles."""
    M, N, K = shape
    if M > 8000 and epi not in (1, 3):
        pytest.skip("the largest shape runs the two epilogues that large batches take this kernel for")
    _linear_case(srm, srm.SRM_BF16, M, N, K, epi, 9, seed=900 + epi)


def test_linear_bf16_persistent_kernel_rejects_odd_k_tile_counts(srm):
    A = torch.zeros((512, 192), dtype=torch.bfloat16, device="cuda")
    W = torch.zeros((512, 192), dtype=torch.bfloat16, device="cuda")
    out = torch.zeros((512, 512), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(srm.SrmError) as e:
        srm.linear(srm.SRM_BF16, 0, A, W, None, out=out, tile=9)
    assert e.value.code == -1


@pytest.mark.parametrize("d,B", [(256, 5), (256, 100), (512, 16), (512, 333), (512, 1024)])
@pytest.mark.parametrize("half_state", [False, True])
def test_mixer_block_one_kernel(srm, d, B, half_state):
    """srm_mixer_block (LayerNorm1, in-projection, state update, out-projection, residual add and LayerNorm2 of a
    layer in one kernel) against the oracle's LayerNorm / linear / mixer step in fp64 on sampled rows, with one
    shared position and with one position per row (some of them outside the context: state kept, zeros mixed)."""
    from oracle import srm_oracle
    if half_state and B > 400:
        pytest.skip("one large binary16 case is enough")
    n_ctx = 8
    cfg = srm_synth.tiny_config(vocab=16, d_model=d, n_layers=2, n_heads=4, n_ctx=n_ctx, weight_dtype="bf16", seed=78,
                                state_dtype="fp16" if half_state else "fp32")
    w = srm_synth.make_weights(cfg, stress=True)
    model = srm.Model(cfg, w)
    orc = srm_oracle.Oracle(cfg, w, "f64")
    rng = np.random.default_rng(B + d)
    x0 = (rng.standard_normal((B, d)) * 1.5 + 0.3).astype(np.float32)
    S0 = rng.standard_normal((B, d)).astype(np.float32)
    layer = 1
    lw = w["layers"][layer]
    st_t = torch.float16 if half_state else torch.float32
    pos_rows = rng.integers(-1, n_ctx + 1, size=B).astype(np.int32)      # -1 and n_ctx: inactive rows
    rows = sorted({0, 1, B // 3, B - 2 if B > 1 else 0, B - 1})
    for shared in (True, False):
        print(f"mixer_block d={d} B={B} half={half_state} shared_pos={shared}", flush=True)
        x = to_dev(x0)
        S = to_dev(S0).to(st_t)
        out = torch.full((B, d), 7.0, dtype=torch.bfloat16, device="cuda")
        if shared:
            model.mixer_block(layer, 6, B, x, S, out)
        else:
            model.mixer_block(layer, 0, B, x, S, out, pos_rows=to_dev(pos_rows, torch.int32))
        torch.cuda.synchronize()
        xg, Sg, og = x.cpu().numpy(), S.float().cpu().numpy(), out.float().cpu().numpy()
        for b in rows:
            pos = 6 if shared else int(pos_rows[b])
            a = orc.layernorm(x0[b].astype(np.float64), lw["ln1_g"], lw["ln1_b"], cfg.ln_eps)
            S_ref = S0[b].astype(np.float16 if half_state else np.float32).astype(np.float64)
            if 0 <= pos < n_ctx:
                u = orc.linear(lw["w_in"], lw["b_in"], a)
                m = orc.mixer_step(S_ref, u, lw["alpha"][:, pos], lw["beta"][:, pos], lw["lam"])
            else:
                m = np.zeros(d)
            x_ref = x0[b].astype(np.float64) + orc.linear(lw["w_out"], lw["b_out"], m)
            o_ref = orc.layernorm(x_ref, lw["ln2_g"], lw["ln2_b"], cfg.ln_eps)
            tol = 2e-2
            assert np.abs(Sg[b] - S_ref).max() <= tol * max(1.0, np.abs(S_ref).max()), (b, pos)
            assert np.abs(xg[b] - x_ref).max() <= tol * np.abs(x_ref).max(), (b, pos)
            assert np.abs(og[b] - o_ref).max() <= 2 * tol * np.abs(o_ref).max(), (b, pos)
        if not shared:
            inactive = (pos_rows < 0) | (pos_rows >= n_ctx)
            if inactive.any():
                np.testing.assert_array_equal(Sg[inactive], S0[inactive].astype(np.float16 if half_state else np.float32)
                                              .astype(np.float32))
    model.close()


def test_mixer_block_rejects_what_it_cannot_run(srm):
    cfg = srm_synth.tiny_config(vocab=16, d_model=128, n_layers=1, n_heads=4, n_ctx=8, weight_dtype="bf16", seed=3)
    model = srm.Model(cfg, srm_synth.make_weights(cfg))
    x = torch.zeros((4, 128), device="cuda")
    S = torch.zeros((4, 128), device="cuda")
    out = torch.zeros((4, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(srm.SrmError) as e:
        model.mixer_block(0, 0, 4, x, S, out)
    assert e.value.code == -1
    model.close()

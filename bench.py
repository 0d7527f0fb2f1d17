#!/usr/bin/env python3
"""Benchmark of the SRM recurrent decode path on one MI355X.

A step is one pass of the whole hot path (embedding gather, L blocks of
LayerNorm / in-projection / recurrent state update / out-projection /
LayerNorm / MLP, final LayerNorm, LM head with fused argmax) over one batch:
one new token for every sample.  Inputs (weights, prompts, prefilled state)
are resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C4|C3|C1]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
PEAK_BF16_TFLOPS = 2500.0      # dense bf16 MFMA
PEAK_FP32_TFLOPS = 157.3


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="C4", choices=["C1", "C3", "C4"])
    ap.add_argument("--concurrency", action="store_true",
                    help="instead of the timed step: the C5 sweep (256 prompts x k replicas) and the largest "
                         "resident batch that still completes a decode step")
    ap.add_argument("--temperature", type=float, default=0.0,
                    help="sample with this temperature (fused Gumbel-max) instead of greedy argmax")
    ap.add_argument("--no-projections", action="store_true",
                    help="the non-projected model variant (mixer layers without in/out head projections)")
    ap.add_argument("--state-dtype", choices=["fp32", "fp16"], default="fp32",
                    help="fp16: the recurrent cache and decay constants in half precision (a model variant)")
    ap.add_argument("--head-layout", choices=["mixed", "row", "column", "combined"], default="mixed",
                    help="row / column: one kind of head only; combined: two matrices per head, twice the cache "
                         "(model variants)")
    ap.add_argument("--mixer-kernel", type=int, default=1,
                    help="k > 1: k column-repeat filters along the hidden dimension per mixer layer (a model variant; "
                         "implies --head-layout column)")
    ap.add_argument("--batch", type=int, default=0,
                    help="decode batch instead of the workload's own (e.g. C4's model at a small batch: the "
                         "weight-streaming regime)")
    ap.add_argument("--top-p", type=float, default=1.0,
                    help="with --temperature: nucleus truncation (the paper's rollouts use 0.9 at temperature 0.7)")
    ap.add_argument("--per-step-calls", action="store_true",
                    help="time K srm_decode_step calls instead of one srm_generate call of K steps")
    ap.add_argument("--no-prefill", action="store_true", help="start from a zero state and random tokens "
                    "(for kernel traces that should hold decode kernels only)")
    ap.add_argument("--pmc-probe", action="store_true",
                    help="only launch, a few times each: a plain 1 GiB copy, the state update over all layer slabs, "
                         "the MLP-up GEMM and the LM-head GEMM (for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--kernel-iters", type=int, default=20, help="launches per kernel leg")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-legs", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the short runs of C1, C3 and C5 (k = 1024) that the default C4 run appends")
    return ap.parse_args()


def time_launches(torch, fn, iters, warm=3):
    """Average duration (s) of fn() over `iters` back-to-back launches, timed with
    events on the stream the kernels are launched on (torch's current stream)."""
    for _ in range(warm):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    e1.synchronize()
    return e0.elapsed_time(e1) * 1e-3 / iters


def kernel_legs(torch, srm, model, cfg, B, iters):
    """Time each kernel of the step alone at the workload's shapes."""
    d, ff, V, L = cfg.d_model, cfg.d_ff, cfg.vocab, cfg.n_layers
    bf = cfg.weight_dtype == "bf16"
    dt = srm.SRM_BF16 if bf else srm.SRM_FP32
    tt = torch.bfloat16 if bf else torch.float32
    esz = 2 if bf else 4
    g = torch.Generator(device="cuda").manual_seed(0)

    def rnd(*shape, scale=1.0):
        return (torch.randn(*shape, device="cuda", generator=g) * scale).to(tt)

    legs = {}
    a = rnd(B, d)
    gact = rnd(B, ff)
    shapes = {  # name: (A, N, K, epilogue, fp32 residual out?)
        "gemm_in": (a, d, d, 0), "gemm_out": (a, d, d, 2),
        "gemm_up": (a, ff, d, 1), "gemm_down": (gact, d, ff, 2),
    }
    for name, (A, N, K, epi) in shapes.items():
        W = rnd(N, K, scale=0.02)
        bias = torch.zeros(N, device="cuda")
        out = torch.zeros((B, N), device="cuda", dtype=torch.float32 if epi == 2 else tt)
        t = time_launches(torch, lambda: srm.linear(dt, epi, A, W, bias, out=out), iters)
        fl = 2.0 * B * N * K
        legs[name] = {"ms": t * 1e3, "tflops": fl / t * 1e-12, "M": B, "N": N, "K": K}
        if bf:
            legs[name].update(gemm_timeline(torch, srm, lambda: srm.linear(dt, epi, A, W, bias, out=out), B, N, K))
        del W, out
    W = rnd(V, d, scale=0.02)
    am = torch.empty(B, dtype=torch.int32, device="cuda")
    scratch = torch.empty(srm.linear_scratch_bytes(B, V), dtype=torch.uint8, device="cuda")
    t = time_launches(torch, lambda: srm.linear(dt, 3, a, W, None, out=None, argmax=am, scratch=scratch), iters)
    legs["gemm_head_argmax"] = {"ms": t * 1e3, "tflops": 2.0 * B * V * d / t * 1e-12, "M": B, "N": V, "K": d}
    if bf:
        legs["gemm_head_argmax"].update(gemm_timeline(
            torch, srm, lambda: srm.linear(dt, 3, a, W, None, out=None, argmax=am, scratch=scratch), B, V, d))
    del W, scratch
    # state update: cycle over the L layer slabs exactly as a step does
    half = getattr(cfg, "state_dtype", "fp32") == "fp16"
    sd = getattr(cfg, "state_width", d)             # 2d with combined heads
    state = torch.zeros((L, B, sd), dtype=torch.float16 if half else torch.float32, device="cuda")
    u = rnd(B, sd)
    m = torch.empty_like(u)
    it = [0]

    def su():
        model.mixer_update(it[0] % L, 5, B, u, state[it[0] % L], m)
        it[0] += 1

    t = time_launches(torch, su, max(iters, 2 * L), warm=L)
    nbytes = B * sd * ((4 if half else 8) + 2 * esz)
    legs["state_update"] = {"ms": t * 1e3, "gbs": nbytes / t * 1e-9, "bytes": nbytes}
    if getattr(cfg, "use_projections", True):
        # the form the step runs with bf16 weights: in-projection with the update in its epilogue (u never in memory)
        def pu():
            model.mixer_project_update(it[0] % L, 5, B, a, state[it[0] % L], m)
            it[0] += 1

        t = time_launches(torch, pu, max(iters, 2 * L), warm=L)
        fused_bytes = B * sd * ((4 if half else 8) + esz) + B * d * esz + sd * d * esz
        legs["gemm_in_with_state_update"] = {"ms": t * 1e3, "tflops": 2.0 * B * sd * d / t * 1e-12,
                                             "gbs": fused_bytes / t * 1e-9, "bytes": fused_bytes,
                                             "two_launch_ms": legs["gemm_in"]["ms"] + legs["state_update"]["ms"]
                                             if sd == d else None}
    return legs


def gemm_timeline(torch, srm, launch, M, N, K):
    """Where the time of a bf16 GEMM launch goes, from the kernel's own clocks (srm_linear_timeline_probe): every
    work-group stores the 100 MHz wall clock at its start, k-loop start, k-loop end and after its last store,
    and the shader cycle counter around the k loop.  Launches run back to back, the last one is read."""
    import numpy as np
    cap = 1 << 16
    buf = torch.zeros(8 * cap, dtype=torch.int64, device="cuda")
    srm.linear_timeline_probe(buf, cap)
    for _ in range(4):
        launch()
    srm.linear_timeline_probe(None)
    torch.cuda.synchronize()
    tr = buf.cpu().numpy().reshape(cap, 8)
    tr = tr[tr[:, 3] > 0]
    if len(tr) == 0:
        return {}
    t0, t1, t2, t3, c1, c2, hw = (tr[:, i].astype(np.int64) for i in range(7))
    us = 0.01                                       # one tick of the 100 MHz clock
    ghz = float(((c2 - c1) / np.maximum(t2 - t1, 1)).mean() * 0.1)
    cu = ((hw >> 32) << 16) | (hw & 0xFF00)         # XCC, shader engine / array, CU
    gaps, per_cu = [], {}
    for i in np.argsort(t0):
        k = int(cu[i])
        if k in per_cu:
            gaps.append((t0[i] - per_cu[k]) * us)
        per_cu[k] = t3[i]
    loop_us = float((t2 - t1).mean() * us)
    flop_per_wg = 2.0 * M * N * K / len(tr)
    return {"shader_clock_ghz": ghz,
            "timeline": {"work_groups": int(len(tr)), "cus": len(per_cu),
                         "prologue_us": float((t1 - t0).mean() * us), "k_loop_us": loop_us,
                         "epilogue_us": float((t3 - t2).mean() * us),
                         "turnaround_us": float(np.mean(gaps)) if gaps else 0.0,
                         "launch_span_us": float((t3.max() - t0.min()) * us),
                         "k_loop_tflops_all_cus": flop_per_wg / (loop_us * 1e-6) * len(per_cu) * 1e-12,
                         # cycles the four matrix pipes of a CU need for the work-group's flops (a 32x32x16 bf16
                         # product, 32768 flop, occupies a SIMD's pipe for 32 cycles) over the cycles the loop took
                         "k_loop_mfma_busy_frac": float(flop_per_wg / 4096.0 / (c2 - c1).mean())}}


def achievable_rates(torch, srm):
    """What the chip delivers to the simplest possible kernels: a plain 1 GiB copy (read + write,
    streaming and ordinary loads/stores; the better one counts) and a register-resident chain of
    bf16 matrix-core products on 8 wavefronts per SIMD."""
    src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    rates = {}
    for name, streaming in (("copy_streaming_gbs", True), ("copy_plain_gbs", False)):
        t = time_launches(torch, lambda: srm.probe_copy(dst, src, streaming=streaming), 10)
        rates[name] = 2.0 * src.numel() * 4 / t * 1e-9
    del src, dst
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    blocks, iters = cus * 8, 20000
    out = torch.empty(blocks * 256, device="cuda")
    flop = [0.0]

    def run():
        flop[0] = srm.probe_mfma(out, blocks, iters)

    t = time_launches(torch, run, 5, warm=2)
    assert bool((out == 1024.0 * iters).all())

    def run_random():      # operands with random bits: more power per product, a lower clock
        srm.probe_mfma(out, blocks, iters, random_operands=True)

    t_rand = time_launches(torch, run_random, 5, warm=2)
    assert bool(torch.isfinite(out).all())
    return {"copy_gbs": max(rates.values()), **rates, "copy_bytes": 2 << 30,
            "mfma_bf16_tflops": flop[0] / t * 1e-12, "mfma_bf16_tflops_random_operands": flop[0] / t_rand * 1e-12,
            "mfma_probe": f"{blocks} work-groups x 4 wavefronts x {iters} x 4 "
            "independent 32x32x16 bf16 products, operands in registers (all ones; and pseudo-random in (-1, 1))"}


def cpu_baseline(cfg, w, rows, T):
    """The fp32 oracle, as it stands, on `rows` samples x T teacher-forced positions."""
    import numpy as np
    from oracle import srm_oracle
    import srm_synth
    orc = srm_oracle.Oracle(cfg, w, "f32")
    toks = srm_synth.make_prompts(cfg, batch=rows, length=T, seed=99)
    t0 = time.perf_counter()
    orc.recurrent_forward(toks, pos0=cfg.prompt_len, want_hidden=False, want_logits=False, want_greedy=True)
    dt = time.perf_counter() - t0
    threads = min(rows, int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)))
    return {"value": rows * T / dt, "unit": "tokens/s", "cores": threads, "per_core": rows * T / dt / threads, "kind": "oracle",
            "sample": f"{rows} samples x {T} decode positions of {cfg.name} (fp32 build, OpenMP over samples), {dt:.1f} s"}


def concurrency_sweep(torch, srm, srm_synth, steps, state_dtype="fp32"):
    """C5: 256 distinct prompts prefilled once, state fanned out to k replicas each, greedy decode;
    then the largest batch (state + workspace resident) that completes one decode step."""
    cfg = srm_synth.CONFIGS["C5"]
    if state_dtype != "fp32":
        import dataclasses
        cfg = dataclasses.replace(cfg, state_dtype=state_dtype)
    w = srm_synth.make_weights(cfg)
    model = srm.Model(cfg, w)
    prompts = torch.from_numpy(srm_synth.make_prompts(cfg)).cuda()
    N, P = prompts.shape
    out = {"metric": "generated tokens/sec on 1 MI355X at max batch", "unit": "tokens/s", "n_gpus": 1,
           "data": "synthetic", "dtype": "bf16", "sweep": [], "config": {"workload": f"C5: C4's model, 256 prompts x k, {state_dtype} state"}}
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for k in cfg.fanout:
        B = N * k
        state = model.new_state(B)
        ws = model.new_workspace(max(B, N * P))
        tok = torch.empty(B, dtype=torch.int32, device="cuda")
        e0.record()
        model.prefill(prompts, k, state, tok, workspace=ws)
        e1.record(); e1.synchronize()
        t_pre = e0.elapsed_time(e1) * 1e-3
        for i in range(2):
            model.decode_step(B, P + i, tok, state, tok, workspace=ws)
        e0.record()
        for i in range(steps):
            model.decode_step(B, P + 2 + i, tok, state, tok, workspace=ws)
        e1.record(); e1.synchronize()
        t = e0.elapsed_time(e1) * 1e-3 / steps
        out["sweep"].append({"k": k, "batch": B, "tokens_per_s": B / t, "ms_per_step": t * 1e3,
                             "prefill_s": t_pre, "state_gib": model.state_bytes(B) / 2**30})
        del state, ws, tok
        torch.cuda.empty_cache()
    # largest resident batch: the state of every sequence + a workspace for slices of 131072 samples
    # (a decode call takes the step in slices when the workspace is smaller than the batch); one successful step
    free, total = torch.cuda.mem_get_info()
    slice_rows = 131072
    ws = model.new_workspace(slice_rows)
    per_seq = model.state_bytes(1) + 8
    hi = int((free - ws.numel() - (2 << 30)) / per_seq) // 4096 * 4096
    best = None
    B = hi
    while B > 0 and best is None:
        try:
            state = model.new_state(B)
            tok = torch.zeros(B, dtype=torch.int32, device="cuda")
            e0.record()
            model.decode_step(B, 0, tok, state, tok, workspace=ws)
            e1.record(); e1.synchronize()
            ok = bool(((tok >= 0) & (tok < cfg.vocab)).all())
            if ok:
                best = {"batch": B, "ms_per_step": e0.elapsed_time(e1), "tokens_per_s": B / (e0.elapsed_time(e1) * 1e-3),
                        "state_gib": model.state_bytes(B) / 2**30, "workspace_gib": ws.numel() / 2**30,
                        "rows_per_slice": slice_rows, "hbm_total_gib": total / 2**30}
            del state, tok
        except (RuntimeError, torch.cuda.OutOfMemoryError):
            pass
        torch.cuda.empty_cache()
        B = int(B * 0.95) // 4096 * 4096
    out["max_resident"] = best
    out["value"] = max(r["tokens_per_s"] for r in out["sweep"])
    torch.cuda.synchronize()
    model.close()
    print(json.dumps(out))


def quick_workload(torch, srm, srm_synth, name, steps, fanout=1, model=None, weights=None):
    """A few graph-replayed decode steps of another configuration (prefilled state), for the one-line summary."""
    cfg = srm_synth.CONFIGS[name]
    w = weights if weights is not None else srm_synth.make_weights(cfg)
    own = model is None
    if own:
        model = srm.Model(cfg, w)
    prompts = torch.from_numpy(srm_synth.make_prompts(cfg)).cuda()
    N, P = prompts.shape
    B = N * fanout
    state = model.new_state(B)
    ws = model.new_workspace(max(B, min(N * P, 1 << 17)))
    tok = torch.empty(B, dtype=torch.int32, device="cuda")
    model.prefill(prompts, fanout, state, tok, workspace=ws)
    store = torch.empty((steps, B), dtype=torch.int32, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    with torch.cuda.stream(side):
        model.generate(B, P, 3, tok, state, store, workspace=ws, temperature=0.0, seed=1)      # warm-up + capture
        side.synchronize()
        t0 = time.perf_counter()
        e0.record()
        model.generate(B, P + 3, steps, tok, state, store, workspace=ws, temperature=0.0, seed=1)
        e1.record()
        side.synchronize()
        wall = time.perf_counter() - t0
    torch.cuda.synchronize()
    t = max(wall, e0.elapsed_time(e1) * 1e-3) / steps
    tk = tok.cpu().numpy()
    assert ((tk >= 0) & (tk < cfg.vocab)).all()
    res = {"batch": B, "steps": steps, "ms_per_step": t * 1e3, "tokens_per_s": B / t,
           "state_gib": model.state_bytes(B) / 2**30}
    if own:
        model.close()
    del state, ws, tok, store, prompts
    torch.cuda.empty_cache()
    return res


def measured_traffic(kernel_key):
    """HBM-side bytes per launch (read + written) of a kernel at the C4 shapes, from the committed
    rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary (scaled by the copy-kernel factors stated there)."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_C4_kernels.json.txt")
    try:
        t = json.load(open(path))[kernel_key]
        return t["read_bytes"] + t["write_bytes"]
    except (OSError, KeyError, ValueError):
        return None


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (samples are independent; a multi-GPU run is "
              "N copies of this one with the batch split); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    import paper_2605_08696_amd as srm
    import srm_synth

    srm.lib()                                     # fails loudly if the HIP library is missing
    torch.cuda.set_device(0)
    if args.concurrency:
        concurrency_sweep(torch, srm, srm_synth, min(args.steps, 8), args.state_dtype)
        return
    cfg = srm_synth.CONFIGS[args.workload]
    if args.mixer_kernel > 1:
        args.head_layout = "column"
    if args.no_projections or args.state_dtype != "fp32" or args.head_layout != "mixed":
        import dataclasses
        cfg = dataclasses.replace(cfg, use_projections=not args.no_projections, state_dtype=args.state_dtype,
                                  head_layout=args.head_layout, mixer_kernel=args.mixer_kernel)
    if args.batch > 0:
        import dataclasses
        cfg = dataclasses.replace(cfg, batch=args.batch)
    B, P = cfg.batch, cfg.prompt_len
    t0 = time.perf_counter()
    w = srm_synth.make_weights(cfg)
    prompts = srm_synth.make_prompts(cfg)
    model = srm.Model(cfg, w)
    t_setup = time.perf_counter() - t0

    state = model.new_state(B)
    ws = model.new_workspace(max(B, min(B * P, 1 << 17)))
    tok = torch.empty(B, dtype=torch.int32, device="cuda")
    dprompts = torch.from_numpy(prompts).cuda()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    if args.pmc_probe:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")      # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        kernel_legs(torch, srm, model, cfg, B, 4)
        torch.cuda.synchronize()
        model.close()
        print(json.dumps({"pmc_probe": "done", "copy_bytes_read": src.numel() * 4, "copy_bytes_written": src.numel() * 4}))
        return
    e0.record()
    if args.no_prefill:
        tok.copy_(dprompts[:, 0])
    else:
        model.prefill(dprompts, 1, state, tok, workspace=ws)
    e1.record()
    e1.synchronize()
    prefill_s = e0.elapsed_time(e1) * 1e-3

    n_steps = args.warmup + args.steps
    assert P + n_steps <= cfg.n_ctx, "steps + warmup exceed the model's positions"
    # All steps run on a side stream: srm_generate replays one captured step from a HIP graph there
    # (the legacy default stream cannot be captured).
    samp = {"temperature": args.temperature, "seed": 1} if args.temperature > 0 else {}
    gsamp = {"temperature": args.temperature, "seed": 1}
    if args.temperature > 0 and args.top_p < 1.0:
        scratch_logits = torch.empty((B, cfg.vocab), dtype=torch.float32, device="cuda")
        samp.update(top_p=args.top_p, logits=scratch_logits)
        gsamp.update(top_p=args.top_p, logits=scratch_logits)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    store = torch.empty((max(args.steps, args.warmup), B), dtype=torch.int32, device="cuda")
    with torch.cuda.stream(side):
        pos = P
        if args.per_step_calls:
            for _ in range(args.warmup):
                model.decode_step(B, pos, tok, state, tok, workspace=ws, **samp)
                pos += 1
        elif args.warmup:
            model.generate(B, pos, args.warmup, tok, state, store, workspace=ws, **gsamp)
            pos += args.warmup
        side.synchronize()
        t_wall0 = time.perf_counter()
        e0.record()
        if args.per_step_calls:
            for _ in range(args.steps):
                model.decode_step(B, pos, tok, state, tok, workspace=ws, **samp)
                pos += 1
        else:
            model.generate(B, pos, args.steps, tok, state, store, workspace=ws, **gsamp)
        e1.record()
        side.synchronize()
        wall = time.perf_counter() - t_wall0
    torch.cuda.synchronize()
    dev_s = e0.elapsed_time(e1) * 1e-3
    step_s = max(wall, dev_s) / args.steps
    tk = tok.cpu().numpy()
    assert ((tk >= 0) & (tk < cfg.vocab)).all() and bool(torch.isfinite(state).all())

    d, ff, V, L = cfg.d_model, cfg.d_ff, cfg.vocab, cfg.n_layers
    gemm_dd = 20.0 if cfg.use_projections else 16.0         # flop / d^2 per token per layer
    flops_step = B * (gemm_dd * L * d * d + 2.0 * V * d)
    esz = 2 if cfg.weight_dtype == "bf16" else 4
    ssz = 2 if cfg.state_dtype == "fp16" else 4
    bytes_step = (gemm_dd / 2 * L * d * d + V * d) * esz + 2.0 * ssz * B * L * cfg.state_width + B * d * esz
    out = {
        "metric": "generated tokens/sec on 1 MI355X at max batch",
        "value": B / step_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": step_s * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if esz == 2 else "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: SRM d_model {d}, {L} layers, 4 mixed heads, MLP x4, vocab {V}, "
                               f"{cfg.weight_dtype} weights / {cfg.state_dtype} state, batch {B}, prompt {P}, greedy decode" +
                               ("" if cfg.use_projections else ", non-projected mixer layers") +
                               ("" if cfg.head_layout == "mixed" else f", {cfg.head_layout} heads") +
                               ("" if cfg.mixer_kernel <= 1 else f", {cfg.mixer_kernel} filters along the hidden dimension"),
                   "batch": B, "prompt_len": P, "state_bytes": model.state_bytes(B)},
        "step": {"algorithmic_tflop": flops_step * 1e-12, "algorithmic_gb": bytes_step * 1e-9,
                 "achieved_gbs": bytes_step / step_s * 1e-9, "hbm_frac": bytes_step / step_s * 1e-9 / PEAK_HBM_GBS,
                 "achieved_tflops": flops_step / step_s * 1e-12, "mfma_frac": flops_step / step_s * 1e-12 / PEAK_BF16_TFLOPS
                 if esz == 2 else None,
                 "device_ms_per_step": dev_s / args.steps * 1e3, "wall_ms_per_step": wall / args.steps * 1e3},
        "prefill": {"seconds": prefill_s, "tokens_per_s": B * P / prefill_s},
        "next_token": "greedy argmax" if args.temperature == 0 else
                      f"sampled, temperature {args.temperature} (fused Gumbel-max)" +
                      (f", top-p {args.top_p} (nucleus pass over materialised logits)" if args.top_p < 1.0 else ""),
        "driver": "K srm_decode_step calls" if args.per_step_calls else
                  ("one srm_generate call (all steps in one persistent kernel)"
                   if model.one_kernel_blocks(B) > 0 and not (args.temperature > 0 and args.top_p < 1.0)
                   else "one srm_generate call (HIP-graph replay of the step)"),
        "setup_seconds": t_setup,
    }
    if not args.no_kernel_legs:
        legs = kernel_legs(torch, srm, model, cfg, B, args.kernel_iters)
        out["kernels"] = legs
        ach = achievable_rates(torch, srm)
        out["achievable"] = ach
        if esz == 2:
            up = legs["gemm_up"]
            # (the library runs the 256x256 tile as a persistent kernel once there are more tiles than CUs)
            persistent = B >= 4096 and -(-B // 256) * -(-ff // 256) > torch.cuda.get_device_properties(0).multi_processor_count
            up_kernel = "gemm_bf16_persist_kernel<EPI=GELU>" if persistent else "gemm_bf16_kernel<256,256,2,4,EPI=GELU>"
            out["roofline"] = {"kernel": up_kernel + " (MLP up, GELU epilogue)", "bound": "mfma",
                               "achieved": up["tflops"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                               "frac": up["tflops"] / PEAK_BF16_TFLOPS,
                               "traffic": measured_traffic(up_kernel) if cfg.name == "C4" else None,
                               "frac_of_achievable": up["tflops"] / ach["mfma_bf16_tflops"],
                               "frac_of_achievable_random_operands": up["tflops"] / ach["mfma_bf16_tflops_random_operands"],
                               "avg_launch_ms": up["ms"], "flop_per_launch": 2.0 * B * ff * d,
                               "algorithmic_bytes_per_launch": (B * d + ff * d + B * ff) * 2.0}
            if "shader_clock_ghz" in up:
                # the published peak is the rate at the maximum clock (2.4 GHz); under the power of this kernel
                # the chip holds a lower clock, which scales the matrix cores' rate with it
                ghz = up["shader_clock_ghz"]
                out["roofline"].update(shader_clock_ghz=ghz, peak_at_that_clock=PEAK_BF16_TFLOPS * ghz / 2.4,
                                       frac_of_peak_at_that_clock=up["tflops"] / (PEAK_BF16_TFLOPS * ghz / 2.4))
        else:
            up = legs["gemm_up"]
            out["roofline"] = {"kernel": "gemm_f32_kernel (MLP up)", "bound": "alu", "achieved": up["tflops"],
                               "peak": PEAK_FP32_TFLOPS, "unit": "TFLOP/s", "frac": up["tflops"] / PEAK_FP32_TFLOPS,
                               "traffic": None, "avg_launch_ms": up["ms"]}
        su = legs["state_update"]
        sd_w = getattr(cfg, "state_width", d)
        # the update as a kernel of its own: the HBM-bound form of the path's defining step.  The timed step
        # of a bf16 model runs it inside the in-projection's epilogue (leg gemm_in_with_state_update), which
        # saves writing and re-reading u; the stand-alone kernel is what srm_mixer_update launches.
        fu = legs.get("gemm_in_with_state_update")
        if fu and esz == 2:
            # the form the timed step runs: in-projection GEMM with the state update in its epilogue.  HBM side:
            # algorithmic bytes (state read + written, A read, W read, m written) over the launch time against
            # 8 TB/s; the launch also carries 2*B*d*d flop on the matrix cores, which run first (k loop), then
            # the epilogue streams the state - the two phases do not overlap inside one launch.
            tr = measured_traffic("gemm_bf16_kernel<256,256,2,4,EPI=MIX>") if cfg.name == "C4" and B == 16384 else None
            out["roofline_state_update_fused"] = {
                "kernel": "gemm_bf16_kernel<EPI=MIX> (in-projection + state update, the launch the step runs)",
                "bound": "hbm", "achieved": fu["gbs"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": fu["gbs"] / PEAK_HBM_GBS, "traffic": tr, "frac_of_achievable": fu["gbs"] / ach["copy_gbs"],
                "avg_launch_ms": fu["ms"], "bytes_per_launch": fu["bytes"],
                "measured_traffic_gbs": None if tr is None else tr / (fu["ms"] * 1e-3) * 1e-9,
                "mfma_tflops": fu["tflops"], "mfma_frac": fu["tflops"] / PEAK_BF16_TFLOPS,
                "time_at_hbm_roofline_ms": fu["bytes"] / (PEAK_HBM_GBS * 1e9) * 1e3,
                "time_at_mfma_roofline_ms": 2.0 * B * sd_w * d / (PEAK_BF16_TFLOPS * 1e12) * 1e3}
        out["roofline_state_update"] = {"kernel": "state_update_kernel (srm_mixer_update: the update as a launch of its own; "
                                                  "the timed bf16 step runs it inside the in-projection instead, see "
                                                  "roofline_state_update_fused)", "bound": "hbm", "achieved": su["gbs"],
                                        "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": su["gbs"] / PEAK_HBM_GBS,
                                        "traffic": measured_traffic("state_update_kernel<bf16,2>") if cfg.name == "C4" else None,
                                        "frac_of_achievable": su["gbs"] / ach["copy_gbs"],
                                        "avg_launch_ms": su["ms"], "bytes_per_launch": su["bytes"]}
    if not args.no_cpu_baseline:
        rows = min(16, os.cpu_count() or 1)
        T = {"C4": 200, "C3": 256, "C1": 240}[cfg.name]      # about 10-20 s of host work
        out["cpu_baseline"] = cpu_baseline(cfg, w, rows, min(T, cfg.n_ctx - P))
    if not args.no_other_workloads and cfg.name == "C4" and args.batch == 0 and args.temperature == 0 \
            and cfg.use_projections and cfg.state_dtype == "fp32" and cfg.head_layout == "mixed":
        # the other configurations, a few steps each (greedy, graph replay of the step; C5 on this model's weights)
        del state, ws, tok, dprompts, store
        torch.cuda.empty_cache()
        ow = {}
        ow["C1 (fp32, B 8)"] = quick_workload(torch, srm, srm_synth, "C1", 64)
        ow["C3 (bf16, B 1024)"] = quick_workload(torch, srm, srm_synth, "C3", 64)
        ow["C5 k=1024 (bf16, B 262144, C4's model)"] = quick_workload(torch, srm, srm_synth, "C5", 8, fanout=1024,
                                                                      model=model, weights=w)
        out["other_workloads"] = ow
        state = ws = tok = dprompts = store = None
    # explicit, ordered teardown: drain the device, free the model (its cached step graph and weights), then
    # the tensors - nothing is left to interpreter finalisation, when a profiler's tool may already be gone
    torch.cuda.synchronize()
    model.close()
    del state, ws, tok, dprompts, store
    print(json.dumps(out))


if __name__ == "__main__":
    main()

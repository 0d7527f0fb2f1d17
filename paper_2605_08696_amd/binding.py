"""ctypes binding of libsrm.so: same names and argument order as include/srm.h.

Argument marshalling only.  Device buffers are torch CUDA tensors; their
dtype, contiguity and size are checked here, on the host, before a pointer is
handed to the library.
"""
from __future__ import annotations

import atexit
import ctypes as C
import os
import sys
import weakref
from typing import Optional

import numpy as np

SRM_FP32, SRM_BF16, SRM_FP16 = 0, 1, 2
_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsrm.so")
_lib = None
# Models that still own device memory.  They are closed by an exit handler, i.e. before the interpreter
# starts tearing modules down: srm_free then runs while the HIP runtime, torch and any profiler tool
# loaded into the process are still intact.  A destructor that fires later, during finalisation, frees nothing.
_live_models: "weakref.WeakSet" = weakref.WeakSet()


@atexit.register
def _close_live_models():
    for m in list(_live_models):
        m.close()

_LAYER_FIELDS = ("ln1_g", "ln1_b", "w_in", "b_in", "alpha", "beta", "lambda", "w_out", "b_out",
                 "ln2_g", "ln2_b", "w_up", "b_up", "w_down", "b_down")
_FP = C.POINTER(C.c_float)


class SrmError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libsrm error {code}: {msg}")
        self.code = code


class srm_config(C.Structure):
    _fields_ = [("vocab", C.c_int32), ("d_model", C.c_int32), ("n_layers", C.c_int32),
                ("n_heads", C.c_int32), ("mlp_expansion", C.c_int32), ("n_ctx", C.c_int32),
                ("weight_dtype", C.c_int32), ("ln_eps", C.c_float), ("state_dtype", C.c_int32),
                ("no_projections", C.c_int32), ("head_layout", C.c_int32),
                ("mixer_kernel", C.c_int32)]


class srm_host_layer(C.Structure):
    _fields_ = [(n, _FP) for n in _LAYER_FIELDS]


class srm_host_weights(C.Structure):
    _fields_ = [("embed", _FP), ("head", _FP), ("lnf_g", _FP), ("lnf_b", _FP),
                ("layers", C.POINTER(srm_host_layer))]


def lib():
    """Load libsrm.so; fails loudly if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`"
                              " (there is no fallback path)")
        L = C.CDLL(_LIB_PATH)
        vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
        L.srm_init_weights.restype = C.c_int
        L.srm_init_weights.argtypes = [C.POINTER(srm_config), C.POINTER(srm_host_weights), C.POINTER(vp)]
        L.srm_free.restype = None
        L.srm_free.argtypes = [vp]
        L.srm_state_bytes.restype = sz
        L.srm_state_bytes.argtypes = [vp, i64]
        L.srm_workspace_bytes.restype = sz
        L.srm_workspace_bytes.argtypes = [vp, i64]
        L.srm_decode_step.restype = C.c_int
        L.srm_decode_step.argtypes = [vp, i64, i32, vp, vp, vp, vp, vp, vp, sz, vp]
        L.srm_generate.restype = C.c_int
        L.srm_generate.argtypes = [vp, i64, i32, i32, vp, vp, vp, C.c_float, C.c_uint32, vp, sz, vp]
        L.srm_decode_step_sampled.restype = C.c_int
        L.srm_decode_step_sampled.argtypes = [vp, i64, i32, vp, vp, vp, C.c_float, C.c_uint32, vp, vp, vp, sz, vp]
        L.srm_linear_argmax_noalloc.restype = C.c_int
        L.srm_linear_argmax_noalloc.argtypes = [i32, vp, vp, vp, i64, i32, i32, vp, vp]
        L.srm_linear_argmax_noalloc_max_bytes.restype = sz
        L.srm_linear_argmax_noalloc_max_bytes.argtypes = []
        L.srm_linear_timeline_probe.restype = None
        L.srm_linear_timeline_probe.argtypes = [vp, i64]
        L.srm_workspace_bytes_config.restype = sz
        L.srm_workspace_bytes_config.argtypes = [vp, i64]
        L.srm_prefill_ragged_plan.restype = C.c_int
        L.srm_prefill_ragged_plan.argtypes = [vp, vp, i32, sz, vp]
        L.srm_prefill.restype = C.c_int
        L.srm_prefill.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp, vp, sz, vp]
        L.srm_decode_step_ragged.restype = C.c_int
        L.srm_decode_step_ragged.argtypes = [vp, i64, vp, i32, vp, vp, vp, C.c_float, C.c_float, C.c_uint32, vp, vp,
                                             sz, vp]
        L.srm_generate_ragged.restype = C.c_int
        L.srm_generate_ragged.argtypes = [vp, i64, i32, vp, vp, vp, vp, i32, C.c_float, C.c_float, C.c_uint32, vp, vp,
                                          sz, vp]
        L.srm_decode_step_topp.restype = C.c_int
        L.srm_decode_step_topp.argtypes = [vp, i64, i32, vp, vp, vp, C.c_float, C.c_float, C.c_uint32, vp, vp, vp, sz,
                                           vp]
        L.srm_generate_topp.restype = C.c_int
        L.srm_generate_topp.argtypes = [vp, i64, i32, i32, vp, vp, vp, C.c_float, C.c_float, C.c_uint32, vp, vp, sz,
                                        vp]
        L.srm_sample_logits.restype = C.c_int
        L.srm_sample_logits.argtypes = [vp, i64, i32, C.c_float, C.c_float, C.c_uint32, i32, vp, vp]
        L.srm_prefill_ragged.restype = C.c_int
        L.srm_prefill_ragged.argtypes = [vp, vp, vp, vp, i32, i32, vp, i64, vp, vp, vp, vp, vp, sz, vp]
        L.srm_parallel_forward.restype = C.c_int
        L.srm_parallel_forward.argtypes = [vp, vp, i32, i32, vp, vp, vp, sz, vp]
        L.srm_mixer_update.restype = C.c_int
        L.srm_mixer_update.argtypes = [vp, i32, i32, i64, vp, vp, vp, vp]
        L.srm_mixer_project_update.restype = C.c_int
        L.srm_mixer_project_update.argtypes = [vp, i32, i32, i64, vp, vp, vp, vp]
        L.srm_mixer_block.restype = C.c_int
        L.srm_mixer_block.argtypes = [vp, i32, i32, vp, i64, vp, vp, vp, vp, vp]
        L.srm_linear.restype = C.c_int
        L.srm_linear.argtypes = [i32, i32, vp, vp, vp, i64, i32, i32, vp, vp, vp, vp]
        L.srm_linear_scratch_bytes.restype = sz
        L.srm_linear_scratch_bytes.argtypes = [i64, i32]
        L.srm_generate_one_kernel_blocks.restype = C.c_int32
        L.srm_generate_one_kernel_blocks.argtypes = [vp, i64]
        L.srm_probe_copy.restype = C.c_int
        L.srm_probe_copy.argtypes = [vp, vp, sz, i32, vp]
        L.srm_probe_mfma.restype = C.c_int
        L.srm_probe_mfma.argtypes = [vp, i32, i32, i32, C.POINTER(C.c_double), vp]
        L.srm_last_error.restype = C.c_char_p
        L.srm_last_error.argtypes = []
        _lib = L
    return _lib


def _check(rc: int):
    if rc != 0:
        raise SrmError(rc, lib().srm_last_error().decode())


def _torch():
    import torch
    return torch


def _dev(t, dtype, numel: int, name: str) -> int:
    """Device pointer of a tensor after host-side checks."""
    if not t.is_cuda:
        raise ValueError(f"{name}: must be a CUDA tensor")
    if t.dtype != dtype:
        raise ValueError(f"{name}: dtype {t.dtype}, expected {dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name}: must be contiguous")
    if t.numel() < numel:
        raise ValueError(f"{name}: {t.numel()} elements, need {numel}")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    torch = _torch()
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


HEAD_LAYOUTS = {"mixed": 0, "row": 1, "column": 2, "combined": 3}


def c_config(cfg) -> "srm_config":
    """The srm_config of a srm_synth-style configuration object."""
    return srm_config(cfg.vocab, cfg.d_model, cfg.n_layers, cfg.n_heads, cfg.mlp_expansion, cfg.n_ctx,
                      SRM_BF16 if cfg.weight_dtype == "bf16" else SRM_FP32, cfg.ln_eps,
                      SRM_FP16 if getattr(cfg, "state_dtype", "fp32") == "fp16" else SRM_FP32,
                      0 if getattr(cfg, "use_projections", True) else 1,
                      HEAD_LAYOUTS[getattr(cfg, "head_layout", "mixed")], int(getattr(cfg, "mixer_kernel", 1)))


class srm_prefill_plan(C.Structure):
    _fields_ = [("passes", C.c_int32), ("chunk_len", C.c_int32), ("chunk_len_by_shape", C.c_int32),
                ("n_chunks", C.c_int32), ("scratch_need", C.c_size_t), ("scratch_room", C.c_size_t)]


def workspace_bytes_config(cfg, rows: int) -> int:
    c = c_config(cfg)
    return lib().srm_workspace_bytes_config(C.byref(c), int(rows))


def prefill_ragged_plan(cfg, offsets, workspace_bytes: int) -> dict:
    """srm_prefill_ragged_plan (host only): how a ragged prefill of these prompts would be cut and scanned."""
    off = np.ascontiguousarray(offsets, dtype=np.int32)
    c = c_config(cfg)
    plan = srm_prefill_plan()
    _check(lib().srm_prefill_ragged_plan(C.byref(c), off.ctypes.data_as(C.POINTER(C.c_int32)), len(off) - 1,
                                         int(workspace_bytes), C.byref(plan)))
    return {n: getattr(plan, n) for n, _ in srm_prefill_plan._fields_}


class Model:
    """Owns one srm_model.  cfg needs vocab, d_model, n_layers, n_heads,
    mlp_expansion, n_ctx, weight_dtype ("fp32"|"bf16") and ln_eps; weights is
    {"embed","head","lnf_g","lnf_b": float32 ndarray, "layers": [{...}]} with
    the layer tensor names of include/srm.h ("lam" for lambda)."""

    def __init__(self, cfg, weights: dict):
        L = lib()
        self.vocab, self.d, self.L, self.H = cfg.vocab, cfg.d_model, cfg.n_layers, cfg.n_heads
        self.ff = cfg.d_model * cfg.mlp_expansion
        self.n_ctx = cfg.n_ctx
        self.dtype = SRM_BF16 if cfg.weight_dtype == "bf16" else SRM_FP32
        c = c_config(cfg)
        kmix = int(getattr(cfg, "mixer_kernel", 1))
        copies = kmix if kmix > 1 else 2 if getattr(cfg, "head_layout", "mixed") == "combined" else 1
        self.sd = self.d * copies                          # state (and mixer) width per sample and layer
        self.state_half = getattr(cfg, "state_dtype", "fp32") == "fp16"
        keep = []

        def fp(a, shape):
            a = np.ascontiguousarray(a, dtype=np.float32)
            if a.shape != tuple(shape):
                raise ValueError(f"weight shape {a.shape}, expected {tuple(shape)}")
            keep.append(a)
            return a.ctypes.data_as(_FP)

        d, ff, H, n, V = self.d, self.ff, self.H * copies, self.n_ctx, self.vocab
        shapes = {"ln1_g": (d,), "ln1_b": (d,), "w_in": (d, d), "b_in": (d,), "alpha": (H, n),
                  "beta": (self.H if kmix > 1 else H, n), "lambda": (H,), "w_out": (d, d), "b_out": (d,), "ln2_g": (d,),
                  "ln2_b": (d,), "w_up": (ff, d), "b_up": (ff,), "w_down": (d, ff), "b_down": (d,)}
        if len(weights["layers"]) != self.L:
            raise ValueError("wrong number of layers")
        layers = (srm_host_layer * self.L)()
        for l, lw in enumerate(weights["layers"]):
            for name in _LAYER_FIELDS:
                src = lw["lam"] if name == "lambda" and "lam" in lw else lw[name]
                setattr(layers[l], name, fp(src, shapes[name]))
        hw = srm_host_weights(fp(weights["embed"], (V, d)), fp(weights["head"], (V, d)),
                              fp(weights["lnf_g"], (d,)), fp(weights["lnf_b"], (d,)), layers)
        h = C.c_void_p()
        _check(L.srm_init_weights(C.byref(c), C.byref(hw), C.byref(h)))
        self._h = h
        _live_models.add(self)

    def close(self):
        """Free the device copies of the weights and the cached step graph (idempotent).  Work of this
        model that is still queued on a stream must have completed: synchronise first."""
        h, self._h = getattr(self, "_h", None), None
        if h:
            lib().srm_free(h)
        _live_models.discard(self)

    def __del__(self):
        # During interpreter finalisation the runtime below may already be going down, and the
        # process exit releases the device memory anyway.
        if not sys.is_finalizing():
            self.close()

    @property
    def act_dtype(self):
        torch = _torch()
        return torch.bfloat16 if self.dtype == SRM_BF16 else torch.float32

    @property
    def state_torch_dtype(self):
        torch = _torch()
        return torch.float16 if self.state_half else torch.float32

    def state_bytes(self, batch: int) -> int:
        return lib().srm_state_bytes(self._h, batch)

    def workspace_bytes(self, rows: int) -> int:
        return lib().srm_workspace_bytes(self._h, rows)

    def one_kernel_blocks(self, batch: int) -> int:
        """Grid size of the one-kernel path srm_generate takes for this batch (0: ordinary step kernels)."""
        return int(lib().srm_generate_one_kernel_blocks(self._h, batch))

    def new_state(self, batch: int):
        torch = _torch()
        return torch.zeros((self.L, batch, self.sd), dtype=self.state_torch_dtype, device="cuda")

    def new_workspace(self, rows: int):
        torch = _torch()
        return torch.empty(self.workspace_bytes(rows), dtype=torch.uint8, device="cuda")

    def decode_step(self, B, pos, tok_in, state, tok_out, logits=None, hidden=None, workspace=None,
                    stream=None, temperature=None, seed=0, top_p=None):
        """srm_decode_step; srm_decode_step_sampled when a temperature is given; srm_decode_step_topp
        when top_p is given too."""
        torch = _torch()
        p_in = _dev(tok_in, torch.int32, B, "tok_in")
        p_st = _dev(state, self.state_torch_dtype, self.L * B * self.sd, "state")
        if state.numel() != self.L * B * self.sd:
            raise ValueError("state: must be exactly [L][B][d]")
        p_out = _dev(tok_out, torch.int32, B, "tok_out")
        p_lg = None if logits is None else _dev(logits, torch.float32, B * self.vocab, "logits")
        p_hd = None if hidden is None else _dev(hidden, torch.float32, B * self.d, "hidden")
        p_ws = _dev(workspace, torch.uint8, 1, "workspace")
        if temperature is None:
            _check(lib().srm_decode_step(self._h, B, pos, p_in, p_st, p_out, p_lg, p_hd, p_ws,
                                         workspace.numel(), _stream(stream)))
        elif top_p is None:
            _check(lib().srm_decode_step_sampled(self._h, B, pos, p_in, p_st, p_out, temperature, seed, p_lg,
                                                 p_hd, p_ws, workspace.numel(), _stream(stream)))
        else:
            _check(lib().srm_decode_step_topp(self._h, B, pos, p_in, p_st, p_out, temperature, top_p, seed, p_lg,
                                              p_hd, p_ws, workspace.numel(), _stream(stream)))

    def generate(self, B, pos0, G, tok, state, tokens_out, workspace=None, stream=None, temperature=0.0, seed=0,
                 top_p=None, logits=None):
        torch = _torch()
        p_tk = _dev(tok, torch.int32, B, "tok")
        p_st = _dev(state, self.state_torch_dtype, self.L * B * self.sd, "state")
        if state.numel() != self.L * B * self.sd:
            raise ValueError("state: must be exactly [L][B][d]")
        p_out = _dev(tokens_out, torch.int32, G * B, "tokens_out")
        p_ws = _dev(workspace, torch.uint8, 1, "workspace")
        if top_p is None:
            _check(lib().srm_generate(self._h, B, pos0, G, p_tk, p_st, p_out, temperature, seed, p_ws,
                                      workspace.numel(), _stream(stream)))
        else:
            p_lg = None if logits is None else _dev(logits, torch.float32, B * self.vocab, "logits")
            _check(lib().srm_generate_topp(self._h, B, pos0, G, p_tk, p_st, p_out, temperature, top_p, seed, p_lg,
                                           p_ws, workspace.numel(), _stream(stream)))

    def prefill(self, prompts, fanout_k, state, next_tok, logits=None, workspace=None, stream=None):
        torch = _torch()
        N, P = prompts.shape
        Bt = N * fanout_k
        p_pr = _dev(prompts, torch.int32, N * P, "prompts")
        p_st = _dev(state, self.state_torch_dtype, self.L * Bt * self.sd, "state")
        if state.numel() != self.L * Bt * self.sd:
            raise ValueError("state: must be exactly [L][N*k][d]")
        p_nt = _dev(next_tok, torch.int32, Bt, "next_tok")
        p_lg = None if logits is None else _dev(logits, torch.float32, N * self.vocab, "logits")
        p_ws = _dev(workspace, torch.uint8, 1, "workspace")
        _check(lib().srm_prefill(self._h, p_pr, N, P, fanout_k, p_st, p_nt, p_lg, p_ws,
                                 workspace.numel(), _stream(stream)))

    def decode_step_ragged(self, B, pos, tok_in, state, tok_out, advance=True, temperature=0.0, seed=0,
                           logits=None, workspace=None, stream=None, top_p=1.0):
        """One step with per-sample positions pos[B] (device int32, advanced in place if asked)."""
        torch = _torch()
        p_pos = _dev(pos, torch.int32, B, "pos")
        p_in = _dev(tok_in, torch.int32, B, "tok_in")
        p_st = _dev(state, self.state_torch_dtype, self.L * B * self.sd, "state")
        if state.numel() != self.L * B * self.sd:
            raise ValueError("state: must be exactly [L][B][d]")
        p_out = _dev(tok_out, torch.int32, B, "tok_out")
        p_lg = None if logits is None else _dev(logits, torch.float32, B * self.vocab, "logits")
        p_ws = _dev(workspace, torch.uint8, 1, "workspace")
        _check(lib().srm_decode_step_ragged(self._h, B, p_pos, 1 if advance else 0, p_in, p_st, p_out,
                                            float(temperature), float(top_p), int(seed), p_lg, p_ws,
                                            workspace.numel(), _stream(stream)))

    def generate_ragged(self, B, G, pos, tok, state, tokens_out, eos_id=-1, temperature=0.0, top_p=1.0, seed=0,
                        logits=None, workspace=None, stream=None):
        """G ragged steps on the device; a sample that emits eos_id goes idle (position -1)."""
        torch = _torch()
        p_pos = _dev(pos, torch.int32, B, "pos")
        p_tk = _dev(tok, torch.int32, B, "tok")
        p_st = _dev(state, self.state_torch_dtype, self.L * B * self.sd, "state")
        if state.numel() != self.L * B * self.sd:
            raise ValueError("state: must be exactly [L][B][d]")
        p_out = _dev(tokens_out, torch.int32, G * B, "tokens_out")
        p_lg = None if logits is None else _dev(logits, torch.float32, B * self.vocab, "logits")
        p_ws = _dev(workspace, torch.uint8, 1, "workspace")
        _check(lib().srm_generate_ragged(self._h, B, G, p_pos, p_tk, p_st, p_out, int(eos_id), float(temperature),
                                         float(top_p), int(seed), p_lg, p_ws, workspace.numel(), _stream(stream)))

    def prefill_ragged(self, tokens, offsets, state, next_tok, fanout_k=1, slot=None, pos=None, logits=None,
                       workspace=None, stream=None):
        """Packed prompts of different lengths; offsets: host int32 sequence of N + 1 boundaries."""
        import numpy as np
        torch = _torch()
        h_off = np.ascontiguousarray(offsets, dtype=np.int32)
        N = h_off.size - 1
        if N < 1:
            raise ValueError("offsets: need at least two boundaries")
        d_off = torch.from_numpy(h_off).to(tokens.device)
        Bt = state.numel() // (self.L * self.sd)
        if state.numel() != self.L * Bt * self.sd:
            raise ValueError("state: must be [L][state_batch][d]")
        p_tk = _dev(tokens, torch.int32, int(h_off[-1]), "tokens")
        p_st = _dev(state, self.state_torch_dtype, self.L * Bt * self.sd, "state")
        p_nt = _dev(next_tok, torch.int32, Bt, "next_tok")
        p_sl = None if slot is None else _dev(slot, torch.int32, N, "slot")
        p_pos = None if pos is None else _dev(pos, torch.int32, Bt, "pos")
        p_lg = None if logits is None else _dev(logits, torch.float32, N * self.vocab, "logits")
        p_ws = _dev(workspace, torch.uint8, 1, "workspace")
        _check(lib().srm_prefill_ragged(self._h, p_tk, h_off.ctypes.data, _dev(d_off, torch.int32, N + 1, "offsets"),
                                        N, fanout_k, p_sl, Bt, p_st, p_nt, p_pos, p_lg, p_ws, workspace.numel(),
                                        _stream(stream)))
        return d_off      # kept alive by the caller until the stream has run the call

    def parallel_forward(self, tok, hidden, logits=None, workspace=None, stream=None):
        torch = _torch()
        B, T = tok.shape
        p_tk = _dev(tok, torch.int32, B * T, "tok")
        p_hd = _dev(hidden, torch.float32, B * T * self.d, "hidden")
        p_lg = None if logits is None else _dev(logits, torch.float32, B * T * self.vocab, "logits")
        p_ws = _dev(workspace, torch.uint8, 1, "workspace")
        _check(lib().srm_parallel_forward(self._h, p_tk, B, T, p_hd, p_lg, p_ws, workspace.numel(),
                                          _stream(stream)))

    def mixer_update(self, layer, pos, B, u, state_layer, m, stream=None):
        torch = _torch()
        n = B * self.sd
        p_u = _dev(u, self.act_dtype, n, "u")
        p_s = _dev(state_layer, self.state_torch_dtype, n, "state_layer")
        p_m = _dev(m, self.act_dtype, n, "m")
        _check(lib().srm_mixer_update(self._h, layer, pos, B, p_u, p_s, p_m, _stream(stream)))

    def mixer_project_update(self, layer, pos, B, a, state_layer, m, stream=None):
        n = B * self.sd
        p_a = _dev(a, self.act_dtype, B * self.d, "a")
        p_s = _dev(state_layer, self.state_torch_dtype, n, "state_layer")
        p_m = _dev(m, self.act_dtype, n, "m")
        _check(lib().srm_mixer_project_update(self._h, layer, pos, B, p_a, p_s, p_m, _stream(stream)))

    def mixer_block(self, layer, pos, B, x, state_layer, norm_out, pos_rows=None, slabs=None, stream=None):
        """srm_mixer_block: x [B][d] fp32 (updated), state_layer [B][d] (updated), norm_out [B][d] bf16 (written);
        pos_rows: int32 [B] device tensor of per-row positions instead of `pos`; slabs: fp32 scratch of
        (d / 128) * B * d elements (allocated here if not given)."""
        torch = _torch()
        n = B * self.d
        if slabs is None:
            slabs = torch.empty((self.d // 128) * n, dtype=torch.float32, device=x.device)
        p_x = _dev(x, torch.float32, n, "x")
        p_s = _dev(state_layer, self.state_torch_dtype, n, "state_layer")
        p_o = _dev(norm_out, self.act_dtype, n, "norm_out")
        p_l = _dev(slabs, torch.float32, (self.d // 128) * n, "slabs")
        p_p = None if pos_rows is None else _dev(pos_rows, torch.int32, B, "pos_rows")
        _check(lib().srm_mixer_block(self._h, layer, pos, p_p, B, p_x, p_s, p_o, p_l, _stream(stream)))


def sample_logits(logits, temperature, top_p, seed, pos, tok_out, stream=None):
    """srm_sample_logits on a torch tensor logits [rows][vocab] (fp32)."""
    torch = _torch()
    rows, V = logits.shape
    _check(lib().srm_sample_logits(_dev(logits, torch.float32, rows * V, "logits"), rows, V, float(temperature),
                                   float(top_p), int(seed), int(pos), _dev(tok_out, torch.int32, rows, "tok_out"),
                                   _stream(stream)))


def probe_copy(dst, src, streaming=True, stream=None):
    """srm_probe_copy: dst = src (same-sized contiguous torch tensors); returns the HBM bytes moved."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes or not (src.is_cuda and dst.is_cuda):
        raise ValueError("probe_copy: dst and src must be device tensors of one size")
    if not (src.is_contiguous() and dst.is_contiguous()):
        raise ValueError("probe_copy: tensors must be contiguous")
    _check(lib().srm_probe_copy(dst.data_ptr(), src.data_ptr(), nbytes, int(bool(streaming)), _stream(stream)))
    return 2 * nbytes


def probe_mfma(out, blocks: int, iters: int, random_operands: bool = False, stream=None) -> float:
    """srm_probe_mfma into out (fp32, blocks * 256 elements); returns the launch's flop count."""
    flop = C.c_double(0.0)
    _check(lib().srm_probe_mfma(_dev(out, _torch().float32, blocks * 256, "out"), int(blocks), int(iters),
                                1 if random_operands else 0, C.byref(flop), _stream(stream)))
    return flop.value


def linear_timeline_probe(buf, blocks: int = 0) -> None:
    """srm_linear_timeline_probe: buf = int64 CUDA tensor of 8 * blocks elements, or None to clear."""
    torch = _torch()
    if buf is None:
        lib().srm_linear_timeline_probe(None, 0)
    else:
        lib().srm_linear_timeline_probe(_dev(buf, torch.int64, 8 * blocks, "timeline probe"), int(blocks))


def linear_argmax_noalloc(dtype, A, W, bias, argmax, stream=None):
    """srm_linear_argmax_noalloc on torch tensors A [M][K], W [N][K] -> argmax [M] int32."""
    torch = _torch()
    M, K = A.shape
    N, K2 = W.shape
    if K != K2:
        raise ValueError("A and W disagree on K")
    t = torch.bfloat16 if dtype == SRM_BF16 else torch.float32
    _check(lib().srm_linear_argmax_noalloc(dtype, _dev(A, t, M * K, "A"), _dev(W, t, N * K, "W"),
                                           None if bias is None else _dev(bias, torch.float32, N, "bias"),
                                           M, N, K, _dev(argmax, torch.int32, M, "argmax"), _stream(stream)))


def linear_argmax_noalloc_max_bytes() -> int:
    return lib().srm_linear_argmax_noalloc_max_bytes()


def linear_scratch_bytes(M: int, N: int) -> int:
    return lib().srm_linear_scratch_bytes(M, N)


def linear(dtype, epilogue, A, W, bias, out=None, argmax=None, scratch=None, stream=None, tile=None):
    """srm_linear on torch tensors A [M][K], W [N][K].  tile (0|1|2) pins the
    bf16 tile shape for sweeps."""
    torch = _torch()
    M, K = A.shape
    N, K2 = W.shape
    if K != K2:
        raise ValueError("A and W disagree on K")
    t = torch.bfloat16 if dtype == SRM_BF16 else torch.float32
    p_a = _dev(A, t, M * K, "A")
    p_w = _dev(W, t, N * K, "W")
    p_b = None if bias is None else _dev(bias, torch.float32, N, "bias")
    epi = epilogue % 100
    out_t = torch.float32 if epi in (2, 3, 4) else t
    p_o = None if out is None else _dev(out, out_t, M * N, "out")
    p_am = None if argmax is None else _dev(argmax, torch.int32, M, "argmax")
    p_sc = None
    if epi == 3:
        p_sc = _dev(scratch, torch.uint8, linear_scratch_bytes(M, N), "scratch")
    code = epilogue if tile is None else (tile + 1) * 100 + epi
    _check(lib().srm_linear(dtype, code, p_a, p_w, p_b, M, N, K, p_o, p_am, p_sc, _stream(stream)))

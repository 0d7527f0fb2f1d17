"""ctypes front end of the plain-C SRM oracle (oracle/srm_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's cpu_baseline leg.  The HIP library and its Python binding never
import this module, and this module never imports them.

Two builds of the same source are loaded on demand: "f64" (truth; parity tests
compare against it) and "f32" (the plain fp32 program that is timed as the CPU
baseline).  Arrays cross in numpy, dtype = the build's real type.
"""
from __future__ import annotations

import ctypes as C
import os
import sys
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "srm_oracle.c")
_LAYER_TENSORS = ("ln1_g", "ln1_b", "w_in", "b_in", "alpha", "beta", "lam",
                  "w_out", "b_out", "ln2_g", "ln2_b", "w_up", "b_up", "w_down", "b_down")
_LIBS = {}


def lib_path(kind: str) -> str:
    return os.path.join(_HERE, f"libsrm_oracle_{kind}.so")


def build(force: bool = False) -> None:
    """Compile both builds with gcc (plain -O2, OpenMP over samples only)."""
    for kind, real in (("f64", "double"), ("f32", "float")):
        out = lib_path(kind)
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(_SRC):
            continue
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               f"-DREAL={real}", _SRC, "-o", out, "-lm"]
        subprocess.run(cmd, check=True)


def _load(kind: str):
    if kind not in _LIBS:
        build()
        lib = C.CDLL(lib_path(kind))
        lib.orc_create.restype = C.c_void_p
        lib.orc_create.argtypes = [C.c_int] * 6 + [C.c_double, C.POINTER(C.c_void_p)]
        lib.orc_create_layout.restype = C.c_void_p
        lib.orc_create_layout.argtypes = [C.c_int] * 6 + [C.c_double, C.c_int, C.POINTER(C.c_void_p)]
        lib.orc_create_kernel.restype = C.c_void_p
        lib.orc_create_kernel.argtypes = [C.c_int] * 6 + [C.c_double, C.c_int, C.POINTER(C.c_void_p)]
        lib.orc_state_width.restype = C.c_int
        lib.orc_state_width.argtypes = [C.c_void_p]
        lib.orc_destroy.argtypes = [C.c_void_p]
        lib.orc_count_params.restype = C.c_longlong
        lib.orc_count_params.argtypes = [C.c_int] * 7
        lib.orc_uniform.restype = C.c_double
        lib.orc_uniform.argtypes = [C.c_uint32] * 4
        lib.orc_gumbel.restype = C.c_double
        lib.orc_gumbel.argtypes = [C.c_uint32] * 4
        lib.orc_pick.restype = C.c_int
        lib.orc_pick.argtypes = [C.c_void_p, C.c_int, C.c_double, C.c_uint32, C.c_int, C.c_int, C.c_void_p]
        lib.orc_nucleus.restype = C.c_int
        lib.orc_nucleus.argtypes = [C.c_void_p, C.c_int, C.c_double, C.c_double, C.c_void_p, C.c_void_p]
        lib.orc_pick_topp.restype = C.c_int
        lib.orc_pick_topp.argtypes = [C.c_void_p, C.c_int, C.c_double, C.c_double, C.c_uint32, C.c_int, C.c_int,
                                      C.c_void_p, C.c_void_p]
        lib.orc_generate_topp.restype = C.c_int
        lib.orc_generate_topp.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.c_void_p, C.c_void_p, C.c_double, C.c_uint32, C.c_int, C.c_double,
                                          C.c_void_p]
        lib.orc_set_state_half.restype = None
        lib.orc_set_state_half.argtypes = [C.c_void_p, C.c_int]
        lib.orc_round_half.restype = C.c_double if kind == "f64" else C.c_float
        lib.orc_round_half.argtypes = [C.c_double if kind == "f64" else C.c_float]
        lib.orc_set_projections.restype = None
        lib.orc_set_projections.argtypes = [C.c_void_p, C.c_int]
        lib.orc_generate.restype = C.c_int
        lib.orc_generate.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_void_p, C.c_void_p, C.c_double, C.c_uint32, C.c_int]
        lib.orc_gelu.restype = C.c_double if kind == "f64" else C.c_float
        lib.orc_gelu.argtypes = [C.c_double if kind == "f64" else C.c_float]
        _LIBS[kind] = lib
    return _LIBS[kind]


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def uniform(seed, pos, b, v) -> float:
    return float(_load("f64").orc_uniform(seed, pos, b, v))


def gumbel(seed, pos, b, v) -> float:
    return float(_load("f64").orc_gumbel(seed, pos, b, v))


def pick(logits, temperature, seed, pos, b, kind="f64") -> int:
    real = np.float64 if kind == "f64" else np.float32
    lg = np.ascontiguousarray(logits, dtype=real)
    return int(_load(kind).orc_pick(_p(lg), lg.size, float(temperature), seed, pos, b, None))


def nucleus(logits, temperature, top_p, kind="f64"):
    """(keep mask [V] of bool, mass margin) of the top-p truncation of softmax(logits / temperature)."""
    real = np.float64 if kind == "f64" else np.float32
    lg = np.ascontiguousarray(logits, dtype=real)
    keep = np.zeros(lg.size, np.uint8)
    mm = C.c_double(0.0)
    _load(kind).orc_nucleus(_p(lg), lg.size, float(temperature), float(top_p), _p(keep), C.byref(mm))
    return keep.astype(bool), mm.value


def pick_topp(logits, temperature, top_p, seed, pos, b, kind="f64", want_margins=False):
    real = np.float64 if kind == "f64" else np.float32
    lg = np.ascontiguousarray(logits, dtype=real)
    mg = (C.c_double if kind == "f64" else C.c_float)(0.0)
    mm = C.c_double(0.0)
    tok = int(_load(kind).orc_pick_topp(_p(lg), lg.size, float(temperature), float(top_p), seed, pos, b,
                                        C.byref(mg), C.byref(mm)))
    return (tok, float(mg.value), mm.value) if want_margins else tok


def round_half(v: float) -> float:
    return float(_load("f64").orc_round_half(float(v)))


LAYOUTS = {"mixed": 0, "row": 1, "column": 2, "combined": 3}


def count_params(vocab, d, L, H=4, e=4, n_ctx=512, with_projections=True) -> int:
    return int(_load("f64").orc_count_params(vocab, d, L, H, e, n_ctx, int(with_projections)))


class Oracle:
    """One model instance in one precision ("f64" or "f32")."""

    def __init__(self, cfg, weights: dict, kind: str = "f64", n_ctx: Optional[int] = None):
        self.lib = _load(kind)
        self.kind = kind
        self.real = np.float64 if kind == "f64" else np.float32
        assert self.lib.orc_real_bytes() == np.dtype(self.real).itemsize
        self.V, self.d, self.L, self.H, self.e = (cfg.vocab, cfg.d_model, cfg.n_layers,
                                                  cfg.n_heads, cfg.mlp_expansion)
        self.n_ctx = cfg.n_ctx if n_ctx is None else n_ctx
        tensors = [weights["embed"], weights["head"], weights["lnf_g"], weights["lnf_b"]]
        for lw in weights["layers"]:
            tensors += [lw[n] for n in _LAYER_TENSORS]
        self._keep = [np.ascontiguousarray(t, dtype=np.float32) for t in tensors]
        arr = (C.c_void_p * len(self._keep))(*[t.ctypes.data for t in self._keep])
        self.layout = LAYOUTS[getattr(cfg, "head_layout", "mixed")]
        self.kmix = int(getattr(cfg, "mixer_kernel", 1))
        if self.kmix > 1:
            if self.layout != LAYOUTS["column"]:
                raise ValueError("a mixer with k filters is built from column-repeat matrices: head_layout 'column'")
            self.h = self.lib.orc_create_kernel(self.V, self.d, self.L, self.H, self.e, self.n_ctx,
                                                float(cfg.ln_eps), self.kmix, arr)
        else:
            self.h = self.lib.orc_create_layout(self.V, self.d, self.L, self.H, self.e, self.n_ctx,
                                                float(cfg.ln_eps), self.layout, arr)
        if not self.h:
            raise ValueError("orc_create rejected the configuration")
        self.sd = int(self.lib.orc_state_width(C.c_void_p(self.h)))
        self._keep = None  # the C side copied everything
        if not getattr(cfg, "use_projections", True):
            self.lib.orc_set_projections(C.c_void_p(self.h), 0)
        if getattr(cfg, "state_dtype", "fp32") == "fp16":
            self.lib.orc_set_state_half(C.c_void_p(self.h), 1)

    def close(self):
        if getattr(self, "h", None):
            self.lib.orc_destroy(C.c_void_p(self.h))
            self.h = None

    def __del__(self):
        if sys.is_finalizing():      # module globals are going away: the process frees the handle
            return
        self.close()

    # -- pieces -----------------------------------------------------------
    def _r(self, a):
        return np.ascontiguousarray(a, dtype=self.real)

    def layernorm(self, x, g, b, eps=1e-5):
        x, g, b = self._r(x), self._r(g), self._r(b)
        out = np.empty_like(x)
        self.lib.orc_layernorm(_p(x), _p(g), _p(b), C.c_int(x.size), C.c_double(eps), _p(out))
        return out

    def linear(self, W, bias, a):
        W, a = self._r(W), self._r(a)
        bias = None if bias is None else self._r(bias)
        y = np.empty(W.shape[0], dtype=self.real)
        self.lib.orc_linear(_p(W), _p(bias), _p(a), C.c_int(W.shape[0]), C.c_int(W.shape[1]), _p(y))
        return y

    def gelu(self, x: float) -> float:
        return float(self.lib.orc_gelu(x))

    def mixer_step(self, S, u, alpha_t, beta_t, lam):
        """In-place on S (must be an ndarray of the build's dtype); returns m."""
        assert S.dtype == self.real and S.flags.c_contiguous
        u, alpha_t, beta_t, lam = map(self._r, (u, alpha_t, beta_t, lam))
        m = np.empty_like(u)
        self.lib.orc_mixer_step(_p(S), _p(u), _p(alpha_t), _p(beta_t), _p(lam),
                                C.c_int(lam.size), C.c_int(u.size), _p(m))
        return m

    def mixer_step_layout(self, S, u, alpha_t, beta_t, lam, H, layout, half=False):
        """orc_mixer_step_layout: in place on S ([d], or [2d] for "combined"); returns m."""
        assert S.dtype == self.real and S.flags.c_contiguous
        u, alpha_t, beta_t, lam = map(self._r, (u, alpha_t, beta_t, lam))
        m = np.empty_like(u)
        self.lib.orc_mixer_step_layout(_p(S), _p(u), _p(alpha_t), _p(beta_t), _p(lam), C.c_int(H),
                                       C.c_int(u.size), C.c_int(LAYOUTS[layout]), C.c_int(int(half)), _p(m))
        return m

    def mixer_step_kernel(self, S, u, alpha_t, beta_t, lam, H, k, half=False):
        """orc_mixer_step_kernel: in place on S [k*d]; returns m [d]."""
        assert S.dtype == self.real and S.flags.c_contiguous
        u, alpha_t, beta_t, lam = map(self._r, (u, alpha_t, beta_t, lam))
        m = np.empty_like(u)
        self.lib.orc_mixer_step_kernel(_p(S), _p(u), _p(alpha_t), _p(beta_t), _p(lam), C.c_int(H), C.c_int(u.size),
                                       C.c_int(k), C.c_int(int(half)), _p(m))
        return m

    def mixer_parallel_kernel(self, U, alpha, beta, lam, H, k, pos0=0):
        U, alpha, beta, lam = map(self._r, (U, alpha, beta, lam))
        T, d = U.shape
        Y = np.empty_like(U)
        self.lib.orc_mixer_parallel_kernel(_p(U), _p(alpha), _p(beta), _p(lam), C.c_int(H), C.c_int(d), C.c_int(k),
                                           C.c_int(T), C.c_int(alpha.shape[1]), C.c_int(pos0), _p(Y))
        return Y

    def mixer_parallel_layout(self, U, alpha, beta, lam, H, layout, pos0=0):
        U, alpha, beta, lam = map(self._r, (U, alpha, beta, lam))
        T, d = U.shape
        Y = np.empty_like(U)
        self.lib.orc_mixer_parallel_layout(_p(U), _p(alpha), _p(beta), _p(lam), C.c_int(H), C.c_int(d), C.c_int(T),
                                           C.c_int(alpha.shape[1]), C.c_int(pos0), C.c_int(LAYOUTS[layout]), _p(Y))
        return Y

    def mixer_parallel(self, U, alpha, beta, lam, pos0=0):
        U, alpha, beta, lam = map(self._r, (U, alpha, beta, lam))
        T, d = U.shape
        Y = np.empty_like(U)
        self.lib.orc_mixer_parallel(_p(U), _p(alpha), _p(beta), _p(lam), C.c_int(lam.size),
                                    C.c_int(d), C.c_int(T), C.c_int(alpha.shape[1]),
                                    C.c_int(pos0), _p(Y))
        return Y

    def mixer_closed_form(self, U, alpha, beta, lam):
        U, alpha, beta, lam = map(self._r, (U, alpha, beta, lam))
        T, d = U.shape
        Y = np.empty_like(U)
        self.lib.orc_mixer_closed_form(_p(U), _p(alpha), _p(beta), _p(lam), C.c_int(lam.size),
                                       C.c_int(d), C.c_int(T), C.c_int(alpha.shape[1]), _p(Y))
        return Y

    # -- whole model --------------------------------------------------------
    def new_state(self, B):
        return np.zeros((B, self.L, self.sd), dtype=self.real)

    def recurrent_forward(self, tokens, pos0=0, state=None, want_hidden=True,
                          want_logits=True, want_greedy=False):
        tokens = np.ascontiguousarray(tokens, dtype=np.int32)
        B, T = tokens.shape
        if state is None:
            state = self.new_state(B)
        assert state.dtype == self.real and state.shape == (B, self.L, self.sd)
        hidden = np.empty((B, T, self.d), self.real) if want_hidden else None
        logits = np.empty((B, T, self.V), self.real) if want_logits else None
        greedy = np.empty((B, T), np.int32) if want_greedy else None
        rc = self.lib.orc_recurrent_forward(C.c_void_p(self.h), B, T, _p(tokens), pos0,
                                            _p(state), _p(hidden), _p(logits), _p(greedy))
        if rc:
            raise ValueError("orc_recurrent_forward: bad argument")
        return {"state": state, "hidden": hidden, "logits": logits, "greedy": greedy}

    def greedy(self, prompts, G, want_logits=False, temperature=0.0, seed=0, b0=0, top_p=1.0):
        """Generate G tokens per prompt: greedy, or sampled when temperature > 0 (from the
        top-p nucleus when top_p < 1)."""
        prompts = np.ascontiguousarray(prompts, dtype=np.int32)
        B, P = prompts.shape
        state = self.new_state(B)
        toks = np.empty((B, G), np.int32)
        logits = np.empty((B, G, self.V), self.real) if want_logits else None
        margin = np.empty((B, G), self.real)
        mass = np.ones((B, G), np.float64)
        rc = self.lib.orc_generate_topp(C.c_void_p(self.h), B, P, G, _p(prompts), _p(state), _p(toks),
                                        _p(logits), _p(margin), float(temperature), seed, b0, float(top_p),
                                        _p(mass))
        if rc:
            raise ValueError("orc_generate: bad argument")
        return {"tokens": toks, "logits": logits, "margin": margin, "state": state, "mass_margin": mass}

    def parallel_forward(self, tokens, want_logits=True):
        tokens = np.ascontiguousarray(tokens, dtype=np.int32)
        B, T = tokens.shape
        hidden = np.empty((B, T, self.d), self.real)
        logits = np.empty((B, T, self.V), self.real) if want_logits else None
        rc = self.lib.orc_parallel_forward(C.c_void_p(self.h), B, T, _p(tokens), _p(hidden),
                                           _p(logits))
        if rc:
            raise ValueError("orc_parallel_forward: bad argument")
        return {"hidden": hidden, "logits": logits}

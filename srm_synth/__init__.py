"""Seeded synthetic inputs for the SRM decode path: configs, weights, prompts.

This module only draws random numbers and rounds storage formats.  It holds
none of the model's arithmetic, so both the CPU oracle's tests and the HIP
library's tests may import it without sharing any method code.

Tensor order, distributions and seeds are the recipe this build fixes for the
five benchmark configurations (tiny fp32, parallel-vs-recurrent, mid bf16,
large bf16, concurrency sweep).  The paper's workloads (trained models on text
prompts, Tables 1, 2, 11) are not available; throughput does not depend on
the values, so random tensors of the same shapes stand in for them.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List

import numpy as np

N_HEADS = 4          # four heads per layer, mixed row/column (MAX model details)
MLP_EXPANSION = 4    # channel mixer expansion; fixed by the printed parameter counts
LN_EPS = 1e-5

LAYER_TENSORS = (
    "ln1_g", "ln1_b", "w_in", "b_in", "alpha", "beta", "lam",
    "w_out", "b_out", "ln2_g", "ln2_b", "w_up", "b_up", "w_down", "b_down",
)
GLOBAL_TENSORS = ("embed", "head", "lnf_g", "lnf_b")
# Matrices stored in bf16 on the device when weight_dtype == "bf16".
BF16_TENSORS = ("embed", "head", "w_in", "w_out", "w_up", "w_down")


@dataclass(frozen=True)
class SRMConfig:
    name: str
    vocab: int
    d_model: int
    n_layers: int
    weight_dtype: str       # "fp32" | "bf16"
    weight_seed: int
    prompt_seed: int
    batch: int              # decode batch (for C5: number of distinct prompts)
    prompt_len: int
    gen_len: int
    n_heads: int = N_HEADS
    mlp_expansion: int = MLP_EXPANSION
    ln_eps: float = LN_EPS
    fanout: tuple = (1,)
    n_ctx_fixed: int = 0    # 0: prompt_len + gen_len rounded up to a multiple of 64
    use_projections: bool = True   # False: non-projected mixer layers (w_in / w_out are drawn but unused)
    state_dtype: str = "fp32"      # "fp16": recurrent cache and decay constants in half precision
    head_layout: str = "mixed"     # "mixed" | "row" | "column" | "combined" (two matrices per head, twice the cache)
    mixer_kernel: int = 1          # k > 1: k column-repeat filters along the hidden dimension (head_layout "column")

    @property
    def n_ctx(self) -> int:
        if self.n_ctx_fixed:
            return self.n_ctx_fixed
        n = self.prompt_len + self.gen_len
        return (n + 63) // 64 * 64

    @property
    def d_head(self) -> int:
        return self.d_model // self.n_heads

    @property
    def d_ff(self) -> int:
        return self.d_model * self.mlp_expansion

    @property
    def head_slots(self) -> int:
        """Rows of alpha / beta (entries of lam) per layer."""
        return self.n_heads * (self.mixer_kernel if self.mixer_kernel > 1 else 2 if self.head_layout == "combined" else 1)

    @property
    def state_width(self) -> int:
        """Cache values per layer per sample."""
        return self.d_model * (self.mixer_kernel if self.mixer_kernel > 1 else 2 if self.head_layout == "combined" else 1)


CONFIGS: Dict[str, SRMConfig] = {
    # C1 and C2 are one model (seed 0): both carry C2's 256 positions.
    "C1": SRMConfig("C1", 4096, 256, 4, "fp32", 0, 1, 8, 16, 32, n_ctx_fixed=256),
    # parallel-vs-recurrent: 256 teacher-forced positions, nothing generated
    "C2": SRMConfig("C2", 4096, 256, 4, "fp32", 0, 2, 4, 256, 0),
    "C3": SRMConfig("C3", 32000, 512, 8, "bf16", 3, 1003, 1024, 64, 256),
    "C4": SRMConfig("C4", 32000, 1024, 16, "bf16", 4, 1004, 16384, 128, 512),
    # C5 runs C4's model (seed 4), so it keeps C4's 640 positions.
    "C5": SRMConfig("C5", 32000, 1024, 16, "bf16", 4, 1005, 256, 128, 256,
                    fanout=(64, 256, 1024), n_ctx_fixed=640),
}


def tiny_config(name="T", vocab=32, d_model=8, n_layers=2, n_heads=2, n_ctx=16,
                weight_dtype="fp32", seed=7, mlp_expansion=4, use_projections=True,
                state_dtype="fp32", head_layout="mixed", mixer_kernel=1) -> SRMConfig:
    """A brute-force sized config for unit tests."""
    return SRMConfig(name, vocab, d_model, n_layers, weight_dtype, seed, seed + 1,
                     2, n_ctx, 0, n_heads=n_heads, mlp_expansion=mlp_expansion,
                     n_ctx_fixed=n_ctx, use_projections=use_projections, state_dtype=state_dtype,
                     head_layout=head_layout, mixer_kernel=mixer_kernel)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result stays fp32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32).astype(np.uint64)
    lsb = (bits >> 16) & 1
    rounded = ((bits + 0x7FFF + lsb) >> 16) << 16
    out = rounded.astype(np.uint32).view(np.float32).reshape(a.shape)
    nan = np.isnan(a)
    if nan.any():
        out = np.where(nan, a, out)
    return out


def tensor_shapes(cfg: SRMConfig, n_ctx: int | None = None):
    d, ff, H, V = cfg.d_model, cfg.d_ff, cfg.head_slots, cfg.vocab
    n = cfg.n_ctx if n_ctx is None else n_ctx
    layer = {
        "ln1_g": (d,), "ln1_b": (d,), "w_in": (d, d), "b_in": (d,),
        "alpha": (H, n), "beta": (cfg.n_heads if cfg.mixer_kernel > 1 else H, n), "lam": (H,),
        "w_out": (d, d), "b_out": (d,), "ln2_g": (d,), "ln2_b": (d,),
        "w_up": (ff, d), "b_up": (ff,), "w_down": (d, ff), "b_down": (d,),
    }
    glob = {"embed": (V, d), "head": (V, d), "lnf_g": (d,), "lnf_b": (d,)}
    return layer, glob


def make_weights(cfg: SRMConfig, stress: bool = False, n_ctx: int | None = None) -> dict:
    """Draw every tensor, in a fixed order, from numpy's default_rng(weight_seed).

    Returns {"embed","head","lnf_g","lnf_b": ndarray, "layers": [ {name: ndarray} ]},
    all float32, row-major [out][in] for matrices.  With stress=True the mixer
    coefficients are O(1) (alpha ~ N(0,1)) and the decays reach down to 0.9001,
    so that mixer mistakes cannot hide behind small coefficients.
    """
    rng = np.random.default_rng(cfg.weight_seed)
    lshape, gshape = tensor_shapes(cfg, n_ctx)

    def normal(shape, scale=0.02):
        return (scale * rng.standard_normal(shape, dtype=np.float32)).astype(np.float32)

    w = {"embed": normal(gshape["embed"])}
    layers: List[dict] = []
    for _ in range(cfg.n_layers):
        lw = {}
        for name in LAYER_TENSORS:
            shape = lshape[name]
            if name == "lam":
                u = rng.random(shape, dtype=np.float32)
                span = np.float32(0.0999) if stress else np.float32(0.1)
                lw[name] = (np.float32(1.0) - span * u).astype(np.float32)
            elif name in ("ln1_g", "ln2_g"):
                lw[name] = (np.float32(1.0) + normal(shape)).astype(np.float32)
            elif name in ("alpha", "beta") and stress:
                lw[name] = normal(shape, 1.0 if name == "alpha" else 0.5)
            else:
                lw[name] = normal(shape)
        layers.append(lw)
    w["lnf_g"] = (np.float32(1.0) + normal(gshape["lnf_g"])).astype(np.float32)
    w["lnf_b"] = normal(gshape["lnf_b"])
    w["head"] = normal(gshape["head"])
    w["layers"] = layers
    if cfg.weight_dtype == "bf16":
        for name in ("embed", "head"):
            w[name] = round_to_bf16(w[name])
        for lw in layers:
            for name in ("w_in", "w_out", "w_up", "w_down"):
                lw[name] = round_to_bf16(lw[name])
    return w


def make_prompts(cfg: SRMConfig, batch: int | None = None, length: int | None = None,
                 seed: int | None = None) -> np.ndarray:
    """int32 [batch][length] tokens uniform in [0, vocab)."""
    rng = np.random.default_rng(cfg.prompt_seed if seed is None else seed)
    b = cfg.batch if batch is None else batch
    p = cfg.prompt_len if length is None else length
    return rng.integers(0, cfg.vocab, size=(b, p), dtype=np.int32)


def subset(cfg: SRMConfig, **kw) -> SRMConfig:
    return replace(cfg, **kw)

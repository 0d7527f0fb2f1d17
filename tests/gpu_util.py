"""Shared helpers of the GPU parity tests (no method arithmetic here)."""
import numpy as np
import torch


def to_dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t if dtype is None else t.to(dtype)


def rel_err_rows(got, ref):
    """max over rows of max|got-ref| / max|ref| along the last axis."""
    ref = np.asarray(ref, dtype=np.float64)
    scale = np.abs(ref).max(axis=-1, keepdims=True)
    return float((np.abs(np.asarray(got, dtype=np.float64) - ref) / scale).max())


def check_tokens(got, ref_tokens, ref_margin, ref_logits_absmax, rtol=1e-4):
    """Greedy tokens must equal the oracle's, except where the oracle's own top-2
    margin is below rtol * max|logit| (a tolerated near tie).  Returns the number
    of tolerated ties."""
    got = np.asarray(got); ref_tokens = np.asarray(ref_tokens)
    bad = got != ref_tokens
    tie = ref_margin < rtol * ref_logits_absmax
    assert not (bad & ~tie).any(), f"{int((bad & ~tie).sum())} tokens differ from the oracle"
    return int((bad & tie).sum())


class Generator:
    """Greedy generation loop over the C ABI (prefill + decode steps), with
    optional teacher forcing of the first rows."""

    def __init__(self, model, batch, prefill_rows):
        self.m = model
        self.B = batch
        self.state = model.new_state(batch)
        self.ws = model.new_workspace(max(batch, prefill_rows))
        self.tok = torch.empty(batch, dtype=torch.int32, device="cuda")

    def prefill(self, prompts_dev, fanout=1, logits=None):
        self.m.prefill(prompts_dev, fanout, self.state, self.tok, logits=logits, workspace=self.ws)

    def step(self, pos, logits=None, hidden=None):
        self.m.decode_step(self.B, pos, self.tok, self.state, self.tok, logits=logits, hidden=hidden,
                           workspace=self.ws)

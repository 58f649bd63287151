"""Seeded synthetic inputs for a Chimera worker: the five workload configurations,
the stage weights and the per-micro-batch activations / upstream gradients.

This module holds none of the method's arithmetic.  It only draws random
tensors (numpy, host) with a fixed recipe so that the library, the tests and
the CPU oracle all see the same numbers.  The paper trains on Wikipedia and
WikiText-2 (appendix); a mid-pipeline stage never sees tokens, only hidden
states, so N(0,1) tensors of the right shape stand in for them.

Recipe: linear weights and biases ~ N(0, 0.02); LayerNorm gain = 1 + N(0, 0.02),
LayerNorm bias ~ N(0, 0.02) (so their gradients are not trivial); incoming
activation X_g and upstream gradient dY_g ~ N(0, 1).  `qk_gain` multiplies the
Q and K columns of the fused QKV weight: with 0.02-scale weights the softmax is
almost uniform, which would hide masking and scaling mistakes, so the parity
tests also run with a gain that gives peaked attention.  For bf16 workloads all
values are rounded to the nearest bf16 (ties to even) and returned as float32.
Every tensor has its own stream derived from (seed, role, stage, layer, index),
so tensors do not change when others are added or skipped.
"""
from dataclasses import dataclass

import numpy as np

PARAM_ORDER = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
               "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")


@dataclass(frozen=True)
class WorkerConfig:
    name: str
    D: int            # pipeline stages
    N: int            # micro-batches per worker and iteration
    layers: int       # Transformer blocks per stage
    hidden: int
    heads: int
    seq: int
    microbatch: int   # B, sequences per micro-batch
    causal: bool
    dtype: str        # "f32" or "bf16"

    @property
    def tokens(self):
        return self.seq * self.microbatch

    @property
    def head_dim(self):
        return self.hidden // self.heads


CONFIGS = {
    "tiny-gpt2-f32": WorkerConfig("tiny-gpt2-f32", 4, 4, 2, 128, 4, 64, 2, True, "f32"),
    "bert48-bf16": WorkerConfig("bert48-bf16", 4, 4, 12, 1024, 16, 512, 8, False, "bf16"),
    "gpt2-1p3b-bf16": WorkerConfig("gpt2-1p3b-bf16", 8, 8, 6, 1600, 25, 1024, 4, True, "bf16"),
    "gpt2-1p3b-n32-bf16": WorkerConfig("gpt2-1p3b-n32-bf16", 8, 32, 6, 1600, 25, 1024, 2, True, "bf16"),
    "gpt2-deep-bf16": WorkerConfig("gpt2-deep-bf16", 32, 32, 2, 2048, 16, 2048, 1, True, "bf16"),
}


def param_shapes(hidden):
    H = hidden
    return {
        "ln1_g": (H,), "ln1_b": (H,), "w_qkv": (H, 3 * H), "b_qkv": (3 * H,),
        "w_o": (H, H), "b_o": (H,), "ln2_g": (H,), "ln2_b": (H,),
        "w_fc1": (H, 4 * H), "b_fc1": (4 * H,), "w_fc2": (4 * H, H), "b_fc2": (H,),
    }


def layer_param_count(hidden):
    return sum(int(np.prod(s)) for s in param_shapes(hidden).values())


def round_to_bf16(a):
    """Nearest-even rounding of float32 values to bf16 precision (kept as float32)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def _rng(seed, role, *idx):
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, role, *idx])))


def _finish(a, dtype):
    a = a.astype(np.float32)
    return round_to_bf16(a) if dtype == "bf16" else a


def qk_gain_for(hidden, score_std=2.0):
    """Gain on the Q and K weights that gives attention scores of about this
    standard deviation (q, k ~ N(0, gain^2 0.02^2 hidden), score = q.k / sqrt(d))."""
    return float(np.sqrt(score_std / (0.02 * 0.02 * hidden)))


def make_stage_params(hidden, layers, stage_id, seed=0, dtype="f32", qk_gain=1.0):
    """Weights of one pipeline stage: list (per block) of dicts keyed by PARAM_ORDER."""
    shapes = param_shapes(hidden)
    out = []
    for layer in range(layers):
        p = {}
        for i, name in enumerate(PARAM_ORDER):
            a = _rng(seed, 1, stage_id, layer, i).standard_normal(shapes[name]) * 0.02
            if name in ("ln1_g", "ln2_g"):
                a = 1.0 + a
            if name == "w_qkv" and qk_gain != 1.0:
                a[:, :2 * hidden] *= qk_gain
            p[name] = _finish(a, dtype)
        out.append(p)
    return out


def make_microbatch(tokens, hidden, mb, seed=0, dtype="f32"):
    """(X_g, dY_g) for micro-batch id `mb`, each [tokens, hidden]."""
    x = _rng(seed, 2, mb).standard_normal((tokens, hidden))
    dy = _rng(seed, 3, mb).standard_normal((tokens, hidden))
    return _finish(x, dtype), _finish(dy, dtype)


def flatten_params(params):
    """Flat float32 vector in the library's parameter order (block after block)."""
    return np.concatenate([layer[k].reshape(-1) for layer in params for k in PARAM_ORDER])

"""Seeded synthetic inputs for the LoCoCo segment step.

This module only draws random tensors of the shapes and value distributions
of the measured workloads and rounds them once to the storage type.  It holds
none of the method's arithmetic and is the one piece of code that both the
HIP path's tests and the CPU oracle's tests are fed from.

Every (tensor, batch, head) slab has its own counter-based stream (Philox
keyed by seed and slab id), so a single chain of a large workload can be
regenerated on its own and is identical to that chain inside the full tensor.

Layouts (row-major, last index contiguous):
    q, o      [batch, n_q_heads,  L, head_dim]
    k, v      [batch, n_kv_heads, L, head_dim]
    conv_w    [M, C, conv_width]   (C = head_dim, or 2*head_dim when conv_in=1)
    conv_b    [M]
"""
from __future__ import annotations

import dataclasses
import math
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

_TENSOR_ID = {"q": 1, "k": 2, "v": 3, "conv_w": 4, "conv_b": 5, "tok_scale": 6}


@dataclasses.dataclass(frozen=True)
class Workload:
    """One synthetic workload: shapes, storage type and value recipe."""

    name: str
    dtype: str              # "f32" or "bf16": storage type of every tensor
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    L: int                  # sequence length
    B: int                  # block (segment) length
    M: int                  # cache slots
    conv_width: int         # odd
    conv_in: int = 0        # 0: keys only (C = d); 1: [K;V] stacked (C = 2d)
    norm: int = 0           # 0: softmax over positions; 1: relu + sum; 2: relu on the conv input, plain sum
    per_head_filters: bool = False
    qk_gain: float = 1.0    # multiplies Q and K ("sharpened" variants use > 1)
    conv_gain: float = 1.0  # multiplies the conv weights
    tok_lognormal_sigma: float = 0.0  # per-token norm scale ~ LogNormal(0, sigma)
    bias_sigma: float = 0.0
    filter_abs: bool = False          # |weights|, |bias|: keeps the signed row sums of norm = 2 away from zero
    seed: int = 0

    @property
    def C(self) -> int:
        return self.head_dim * (2 if self.conv_in else 1)

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    def replace(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


# The five configurations the benchmark description names, in its order.
CFG1 = Workload("cfg1_tiny_f32", "f32", 1, 1, 1, 64, 256, 16, 16, 3)
CFG2 = Workload("cfg2_llama7b_3p5k_M128", "bf16", 1, 32, 32, 128, 3584, 128, 128, 15)
CFG3 = Workload("cfg3_llama7b_32k_M512", "bf16", 1, 32, 32, 128, 32768, 512, 512, 15)
CFG4 = Workload("cfg4_batched_8k_M128", "bf16", 16, 32, 32, 128, 8192, 64, 128, 15,
                tok_lognormal_sigma=0.5)
CFG5 = Workload("cfg5_gqa_16k_M256", "bf16", 2, 32, 8, 128, 16384, 256, 256, 15)
CONFIGS = {w.name.split("_")[0]: w for w in (CFG1, CFG2, CFG3, CFG4, CFG5)}


def _stream(seed: int, tensor: str, b: int = 0, h: int = 0) -> np.random.Generator:
    slab = (_TENSOR_ID[tensor] << 48) | (b << 24) | h
    return np.random.Generator(np.random.Philox(key=[seed & (2**64 - 1), slab]))


def _store(x: np.ndarray, dtype: torch.dtype) -> torch.Tensor:
    return torch.from_numpy(x).to(dtype)


def chain_slab(w: Workload, tensor: str, b: int, h: int, L: int | None = None) -> torch.Tensor:
    """One [L, head_dim] slab of q, k or v for batch b, head h, in storage dtype.

    The slab's first L rows do not depend on L (the stream is consumed row by
    row), so a truncated sequence is a prefix of the full one.
    """
    L = w.L if L is None else L
    d = w.head_dim
    x = _stream(w.seed, tensor, b, h).standard_normal((L, d), dtype=np.float32)
    gain = (w.qk_gain if tensor in ("q", "k") else 1.0) / math.sqrt(d)
    x *= np.float32(gain)
    if w.tok_lognormal_sigma > 0.0:
        z = _stream(w.seed, "tok_scale", b, (_TENSOR_ID[tensor] << 16) | h)
        s = np.exp(np.float32(w.tok_lognormal_sigma)
                   * z.standard_normal((L, 1), dtype=np.float32))
        x *= s
    return _store(x, w.torch_dtype)


def qkv(w: Workload, L: int | None = None, workers: int = 8):
    """Full q [b,Hq,L,d], k, v [b,Hkv,L,d] tensors (CPU, storage dtype)."""
    L = w.L if L is None else L
    out = {
        "q": torch.empty((w.batch, w.n_q_heads, L, w.head_dim), dtype=w.torch_dtype),
        "k": torch.empty((w.batch, w.n_kv_heads, L, w.head_dim), dtype=w.torch_dtype),
        "v": torch.empty((w.batch, w.n_kv_heads, L, w.head_dim), dtype=w.torch_dtype),
    }
    jobs = [(t, b, h) for t in ("q", "k", "v") for b in range(w.batch)
            for h in range(out[t].shape[1])]

    def fill(job):
        t, b, h = job
        out[t][b, h] = chain_slab(w, t, b, h, L)

    if workers > 1 and len(jobs) > 8:
        with ThreadPoolExecutor(workers) as ex:
            list(ex.map(fill, jobs))
    else:
        for j in jobs:
            fill(j)
    return out["q"], out["k"], out["v"]


def conv_filters(w: Workload):
    """conv_w [M, C, k] (or [Hkv, M, C, k] with per-head banks) and conv_b [M].

    Weights ~ N(0, variance 1/(C*k)) times conv_gain; bias ~ N(0, bias_sigma^2)
    (zero by default, as in every measured configuration).
    """
    banks = w.n_kv_heads if w.per_head_filters else 1
    shape = (banks, w.M, w.C, w.conv_width)
    g = _stream(w.seed, "conv_w")
    x = g.standard_normal(shape, dtype=np.float32)
    x *= np.float32(w.conv_gain / math.sqrt(w.C * w.conv_width))
    if w.filter_abs:
        x = np.abs(x)
    cw = _store(x if w.per_head_filters else x[0], w.torch_dtype)
    bshape = (banks, w.M) if w.per_head_filters else (w.M,)
    if w.bias_sigma > 0.0:
        bz = _stream(w.seed, "conv_b").standard_normal(bshape, dtype=np.float32)
        cb = _store((np.abs(bz) if w.filter_abs else bz) * np.float32(w.bias_sigma), w.torch_dtype)
    else:
        cb = torch.zeros(bshape, dtype=w.torch_dtype)
    return cw, cb


def chain_inputs(w: Workload, b: int, kvh: int, L: int | None = None):
    """q [g,L,d], k [L,d], v [L,d] of one (batch, kv-head) chain."""
    g = w.group
    q = torch.stack([chain_slab(w, "q", b, kvh * g + i, L) for i in range(g)])
    return q, chain_slab(w, "k", b, kvh, L), chain_slab(w, "v", b, kvh, L)

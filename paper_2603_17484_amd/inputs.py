"""Seeded synthetic inputs for the L2A conditional-attention layer.

This module only draws random tensors and routing masks.  It holds none of the
layer's arithmetic, so both the CPU oracle's tests and the HIP path may use it
to obtain *identical* inputs.  Everything is numpy on the host.

The paper's kernel benchmark (App. D.1) uses the Qwen2.5-7B head configuration
with synthetic sparsity levels; its tensors are not published, and real router
masks would need trained models, so every workload here is a stand-in: i.i.d.
N(0,1) activations and either i.i.d. Bernoulli routing (the "context-free"
routing of the ablation in Sec. 5) or a bursty two-state Markov chain.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Optional, Sequence, Union

import numpy as np

__all__ = [
    "Workload", "WORKLOADS", "workload", "f32_to_bf16_bits", "bf16_bits_to_f32",
    "round_to_bf16", "normal_tensor", "mask_bernoulli", "mask_markov",
    "make_mask", "make_inputs",
]


# --------------------------------------------------------------------------
# bf16 <-> fp32 bit conversions (round-to-nearest-even), numpy only
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 array -> uint16 array of bf16 bit patterns (RNE; inputs finite)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> fp32 array holding exactly those values."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 array whose every value is exactly representable in bf16."""
    return bf16_bits_to_f32(f32_to_bf16_bits(x))


# --------------------------------------------------------------------------
# workloads
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    T: int
    Hq: int
    Hkv: int
    D: int
    W: int
    dtype: str                       # "bf16" | "fp32"
    mask_kind: str                   # "bernoulli" | "markov" | "dense" | "none"
    mask_heads: int                  # 1, Hkv or Hq
    routed_fraction: Union[float, tuple] = 0.2   # scalar, or (lo, hi) drawn per mask head
    burst: int = 32                  # mean run of routed tokens (markov)
    force_first: bool = False        # force d_0 = 1
    backward: bool = True
    note: str = ""

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def softmax_scale(self) -> float:
        return 1.0 / float(np.sqrt(self.D))


WORKLOADS = {
    # tiny fp32 case: the oracle finishes in seconds
    "tiny_fp32": Workload("tiny_fp32", 1, 2048, 1, 1, 64, 256, "fp32", "bernoulli", 1, 0.2,
                          force_first=True),
    # Qwen2.5-7B-shaped single layer, forward
    "qwen25_7b_32k": Workload("qwen25_7b_32k", 1, 32768, 28, 4, 128, 4096, "bf16", "bernoulli", 1, 0.2,
                              backward=False),
    # long prefill, bursty shared routing, forward
    "prefill_128k": Workload("prefill_128k", 1, 131072, 28, 4, 128, 4096, "bf16", "markov", 1, 0.2,
                             backward=False),
    # training step, per-head i.i.d. routing (fraction swept by the caller)
    "train_64k": Workload("train_64k", 1, 65536, 28, 4, 128, 4096, "bf16", "bernoulli", 28, 0.2),
    # Qwen3-8B-shaped long-context training, per-head bursty routing
    "qwen3_8b_128k": Workload("qwen3_8b_128k", 1, 131072, 32, 8, 128, 4096, "bf16", "markov", 32,
                              (0.05, 0.3)),
    # headline: training-step shape at 128K, 80 % of tokens skip Global attention
    "train_128k": Workload("train_128k", 1, 131072, 28, 4, 128, 4096, "bf16", "bernoulli", 28, 0.2),
}


def workload(name: str, **overrides) -> Workload:
    return replace(WORKLOADS[name], **overrides)


# --------------------------------------------------------------------------
# tensors
# --------------------------------------------------------------------------
def normal_tensor(shape: Sequence[int], seed: int, stream: int, dtype: str) -> np.ndarray:
    """i.i.d. N(0,1) fp32 array; for dtype "bf16" every value is rounded once to bf16."""
    rng = np.random.Generator(np.random.PCG64([int(seed), int(stream)]))
    x = rng.standard_normal(size=tuple(shape), dtype=np.float32)
    if dtype == "bf16":
        x = round_to_bf16(x)
    elif dtype != "fp32":
        raise ValueError(f"dtype {dtype!r}")
    return x


# --------------------------------------------------------------------------
# routing masks  d[B, Hm, T] in {0,1}
# --------------------------------------------------------------------------
def _fractions(fraction, n: int, rng: np.random.Generator) -> np.ndarray:
    if isinstance(fraction, (tuple, list)):
        lo, hi = fraction
        return rng.uniform(lo, hi, size=n)
    return np.full(n, float(fraction))


def mask_bernoulli(B: int, Hm: int, T: int, fraction, seed: int, force_first: bool = False) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64([int(seed), 101]))
    f = _fractions(fraction, B * Hm, rng).reshape(B, Hm, 1)
    d = (rng.random(size=(B, Hm, T)) < f).astype(np.uint8)
    if force_first:
        d[:, :, 0] = 1
    return d


def mask_markov(B: int, Hm: int, T: int, fraction, burst: int, seed: int,
                force_first: bool = False) -> np.ndarray:
    """Two-state Markov chain per (b, head): P(1->0) = 1/burst, P(0->1) chosen so the
    stationary routed fraction is `fraction`; the first state is drawn from the stationary
    law.  Run lengths of such a chain are geometric, which is how the chain is drawn."""
    rng = np.random.Generator(np.random.PCG64([int(seed), 202]))
    fr = _fractions(fraction, B * Hm, rng)
    d = np.zeros((B * Hm, T), dtype=np.uint8)
    for i in range(B * Hm):
        f = float(fr[i])
        if f >= 1.0:
            d[i] = 1
            continue
        if f <= 0.0:
            continue
        p10 = 1.0 / float(burst)
        p01 = min(1.0, f / (1.0 - f) * p10)
        state = 1 if rng.random() < f else 0
        # enough alternating runs to cover T with overwhelming probability
        mean_pair = 1.0 / p10 + 1.0 / p01
        n_pairs = int(T / mean_pair * 1.5) + 64
        filled = 0
        pieces = []
        while filled < T:
            on = rng.geometric(p10, size=n_pairs)
            off = rng.geometric(p01, size=n_pairs)
            runs = np.empty(2 * n_pairs, dtype=np.int64)
            vals = np.empty(2 * n_pairs, dtype=np.uint8)
            if state == 1:
                runs[0::2], runs[1::2] = on, off
                vals[0::2], vals[1::2] = 1, 0
            else:
                runs[0::2], runs[1::2] = off, on
                vals[0::2], vals[1::2] = 0, 1
            pieces.append(np.repeat(vals, runs))
            filled += int(runs.sum())
            # 2*n_pairs runs: the next run starts in the same state as the first one
        d[i] = np.concatenate(pieces)[:T]
    d = d.reshape(B, Hm, T)
    if force_first:
        d[:, :, 0] = 1
    return d


def make_mask(w: Workload, seed: int) -> Optional[np.ndarray]:
    if w.mask_kind == "bernoulli":
        return mask_bernoulli(w.B, w.mask_heads, w.T, w.routed_fraction, seed, w.force_first)
    if w.mask_kind == "markov":
        return mask_markov(w.B, w.mask_heads, w.T, w.routed_fraction, w.burst, seed, w.force_first)
    if w.mask_kind == "dense":
        return np.ones((w.B, w.mask_heads, w.T), dtype=np.uint8)
    if w.mask_kind == "none":
        return np.zeros((w.B, w.mask_heads, w.T), dtype=np.uint8)
    raise ValueError(w.mask_kind)


@dataclass
class Inputs:
    w: Workload
    seed: int
    q: np.ndarray      # [B,T,Hq,D]  fp32 values (bf16-representable when w.dtype == "bf16")
    k: np.ndarray      # [B,T,Hkv,D]
    v: np.ndarray      # [B,T,Hkv,D]
    dO: Optional[np.ndarray]   # [B,T,Hq,D]
    mask: np.ndarray   # [B,Hm,T] uint8


def make_inputs(w: Workload, seed: int = 0, with_dO: Optional[bool] = None) -> Inputs:
    """The same arrays go to the oracle and, after upload, to the GPU."""
    if with_dO is None:
        with_dO = w.backward
    q = normal_tensor((w.B, w.T, w.Hq, w.D), seed, 1, w.dtype)
    k = normal_tensor((w.B, w.T, w.Hkv, w.D), seed, 2, w.dtype)
    v = normal_tensor((w.B, w.T, w.Hkv, w.D), seed, 3, w.dtype)
    dO = normal_tensor((w.B, w.T, w.Hq, w.D), seed, 4, w.dtype) if with_dO else None
    return Inputs(w, seed, q, k, v, dO, make_mask(w, seed))

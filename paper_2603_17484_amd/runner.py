"""Buffer management around the three C-ABI calls: upload, allocate, call, download.

Nothing here computes a step of the layer; it strings l2a_route_compact, l2a_attn_fwd and
l2a_attn_bwd together the way a framework integration would, for the tests, the smoke check
and the benchmark.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

from . import binding as B
from .inputs import f32_to_bf16_bits


def to_device(x: np.ndarray, dtype: str, device="cuda") -> torch.Tensor:
    """fp32 host array -> device tensor of the workload's element type (bf16 values must be exact)."""
    if dtype == "bf16":
        bits = torch.from_numpy(f32_to_bf16_bits(x).view(np.int16))
        return bits.to(device).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(device)


def to_host(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


class GuardedAllocator:
    """torch.empty with a guard band of a known byte pattern on both sides of every buffer.  The tests
    allocate all outputs and workspaces of a layer through one of these and call check() after the
    kernels ran: a store outside a buffer's bounds shows as a changed guard byte."""
    BAND = 4096          # bytes on each side; keeps the 256-byte alignment of what torch returns
    PATTERN = 0xA5

    def __init__(self):
        self.bands = []  # (name, raw uint8 buffer, payload bytes)

    def __call__(self, shape, dtype=torch.float32, device="cuda"):
        shape = (shape,) if isinstance(shape, int) else tuple(shape)
        n = 1
        for d in shape:
            n *= int(d)
        nbytes = n * torch.empty((), dtype=dtype).element_size()
        pad = (-nbytes) % 256
        raw = torch.full((self.BAND + nbytes + pad + self.BAND,), self.PATTERN, dtype=torch.uint8, device=device)
        self.bands.append((f"buffer {len(self.bands)} {shape} {dtype}", raw, nbytes))
        return raw[self.BAND:self.BAND + nbytes].view(dtype).view(shape)

    def check(self):
        """Raises if any guard byte differs from the pattern."""
        for name, raw, nbytes in self.bands:
            lo, hi = raw[:self.BAND], raw[self.BAND + nbytes:]
            if not (bool((lo == self.PATTERN).all()) and bool((hi == self.PATTERN).all())):
                nlo, nhi = int((lo != self.PATTERN).sum()), int((hi != self.PATTERN).sum())
                raise AssertionError(f"{name}: {nlo} guard bytes before and {nhi} after the buffer were overwritten")
        return len(self.bands)


@dataclass
class Layer:
    """Device buffers of one layer call."""
    p: B.l2a_params
    q: torch.Tensor
    k: torch.Tensor
    v: torch.Tensor
    mask: Optional[torch.Tensor]
    qg: Optional[torch.Tensor] = None
    kg: Optional[torch.Tensor] = None
    vg: Optional[torch.Tensor] = None
    alloc: Optional[GuardedAllocator] = None   # tests: every output and workspace between guard bands

    def __post_init__(self):
        p, dev = self.p, self.q.device
        self.qg = self.q if self.qg is None else self.qg
        self.kg = self.k if self.kg is None else self.kg
        self.vg = self.v if self.vg is None else self.vg
        self.dense = bool(p.flags & B.L2A_FLAG_DENSE)
        if self.dense:
            self.row_idx = self.count = self.first = self.route_ws = None
        else:
            self.row_idx, self.count, self.first, self.route_ws = B.alloc_route(p, dev, self.alloc)
        self.O, self.lse_l, self.lse_g, self.S, self.A = B.alloc_fwd(p, dev, alloc=self.alloc)
        self.fwd_ws = B.alloc_fwd_workspace(p, dev, self.alloc)
        self.dq = self.dk = self.dv = self.bwd_ws = None
        self.dqg = self.dkg = self.dvg = None
        self.delta_g = None

    # ---- the hot path, in order
    def route(self):
        if not self.dense:
            B.l2a_route_compact(self.p, self.mask, self.row_idx, self.count, self.first, self.route_ws)

    def forward(self, save_branches: bool = True):
        B.l2a_attn_fwd(self.p, self.q, self.k, self.v, self.qg, self.kg, self.vg, self.row_idx, self.count,
                       self.first, self.O, self.lse_l, self.lse_g, self.S if save_branches else None,
                       self.A if save_branches else None, self.fwd_ws)

    def backward(self, dO: torch.Tensor, separate: bool = False, want_delta: bool = False):
        if self.dq is None:
            self.dq, self.dk, self.dv, self.bwd_ws = B.alloc_bwd(self.p, self.q.device, self.alloc)
            if separate:
                self.dqg, self.dkg, self.dvg, _ = B.alloc_bwd(self.p, self.q.device, self.alloc)
            if want_delta:
                self.delta_g = (self.alloc or torch.empty)(tuple(self.lse_g.shape), dtype=torch.float32,
                                                           device=self.q.device)
        g = (self.dqg, self.dkg, self.dvg) if separate else (self.dq, self.dk, self.dv)
        B.l2a_attn_bwd(self.p, dO, self.q, self.k, self.v, self.qg, self.kg, self.vg, self.row_idx, self.count,
                       self.first, self.S, self.A, self.lse_l, self.lse_g, self.dq, self.dk, self.dv, g[0], g[1],
                       g[2], self.delta_g, self.bwd_ws)


def layer_from_numpy(q, k, v, mask, W, dtype="bf16", flags=0, scale=None, qg=None, kg=None, vg=None,
                     device="cuda", guard: bool = False) -> Layer:
    Bn, T, Hq, D = q.shape
    Hkv = k.shape[2]
    Hm = 1 if mask is None else mask.shape[1]
    p = B.make_params(Bn, T, Hq, Hkv, D, W, Hm, B.L2A_BF16 if dtype == "bf16" else B.L2A_FP32, flags, scale)
    up = lambda x: None if x is None else to_device(x, dtype, device)
    m = None if mask is None else torch.from_numpy(np.array(mask, dtype=np.uint8, order="C", copy=True)).to(device)
    return Layer(p, up(q), up(k), up(v), m, up(qg), up(kg), up(vg), GuardedAllocator() if guard else None)

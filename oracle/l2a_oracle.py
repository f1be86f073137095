"""numpy front-end of the CPU oracle (oracle/l2a_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
cpu_baseline leg; never by the product package.  It shares no code with the HIP path.

All tensors are numpy arrays: q [B,T,Hq,D], k/v [B,T,Hkv,D] float32 (values may be
bf16-representable), mask [B,Hm,T] uint8.  Results are float64.

Parity pins (tests/test_oracle_*.py): explicit masked-matrix softmax in numpy, PyTorch
CPU scaled_dot_product_attention and autograd in fp64, central finite differences, closed
forms (uniform weights, W=0, t=0, constant V) and the layer's invariants.  No function in
this file is "parity unpinned".
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "l2a_oracle.c")
_LIB = os.path.join(_HERE, "libl2a_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (host only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"]
        subprocess.check_call(cmd)
    return _LIB


class _Dims(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("T", ctypes.c_int32), ("Hq", ctypes.c_int32),
                ("Hkv", ctypes.c_int32), ("D", ctypes.c_int32), ("W", ctypes.c_int32),
                ("Hm", ctypes.c_int32), ("scale", ctypes.c_double)]


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        assert _lib.l2a_oracle_abi() == 1
    return _lib


def threads() -> int:
    """OpenMP threads the oracle's loops use."""
    return int(_load().l2a_oracle_threads())


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


@dataclass
class Problem:
    """Shapes + inputs of one layer call; the global-branch q/k/v default to the local ones."""
    q: np.ndarray
    k: np.ndarray
    v: np.ndarray
    mask: np.ndarray
    W: int
    scale: Optional[float] = None
    qg: Optional[np.ndarray] = None
    kg: Optional[np.ndarray] = None
    vg: Optional[np.ndarray] = None

    def __post_init__(self):
        self.q, self.k, self.v = _f32(self.q), _f32(self.k), _f32(self.v)
        self.qg = self.q if self.qg is None else _f32(self.qg)
        self.kg = self.k if self.kg is None else _f32(self.kg)
        self.vg = self.v if self.vg is None else _f32(self.vg)
        self.mask = np.ascontiguousarray(self.mask, dtype=np.uint8)
        self.B, self.T, self.Hq, self.D = self.q.shape
        self.Hkv = self.k.shape[2]
        assert self.k.shape == (self.B, self.T, self.Hkv, self.D) == self.v.shape
        assert self.Hq % self.Hkv == 0
        self.G = self.Hq // self.Hkv
        self.Hm = self.mask.shape[1]
        assert self.mask.shape == (self.B, self.Hm, self.T) and self.Hm in (1, self.Hkv, self.Hq)
        if self.scale is None:
            self.scale = 1.0 / float(np.sqrt(self.D))

    @property
    def dims(self) -> _Dims:
        return _Dims(self.B, self.T, self.Hq, self.Hkv, self.D, int(self.W), self.Hm, float(self.scale))

    def mask_per_head(self) -> np.ndarray:
        """d broadcast to [B,Hq,T]."""
        if self.Hm == 1:
            return np.broadcast_to(self.mask, (self.B, self.Hq, self.T)) != 0
        if self.Hm == self.Hq:
            return self.mask != 0
        return np.repeat(self.mask, self.G, axis=1) != 0

    def all_rows(self) -> np.ndarray:
        b, t, h = np.meshgrid(np.arange(self.B), np.arange(self.T), np.arange(self.Hq), indexing="ij")
        return np.stack([b, h, t], axis=-1).reshape(-1, 3).astype(np.int32)

    def all_keys(self) -> np.ndarray:
        b, t, h = np.meshgrid(np.arange(self.B), np.arange(self.T), np.arange(self.Hkv), indexing="ij")
        return np.stack([b, h, t], axis=-1).reshape(-1, 3).astype(np.int32)


# ------------------------------------------------------------------------------------
# compaction  (Sec. 3.2; App. C, Alg. 1 step 1)
# ------------------------------------------------------------------------------------
def route_compact(mask: np.ndarray, Hq: int, Hkv: int):
    """-> row_idx [B,Hkv,T*G] int32 (tail -1), count [B,Hkv], kblk_first_row [B,Hkv,ceil(T/64)+1]."""
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    B, Hm, T = mask.shape
    G = Hq // Hkv
    nkb = (T + 63) // 64
    row_idx = np.empty((B, Hkv, T * G), dtype=np.int32)
    count = np.empty((B, Hkv), dtype=np.int32)
    first = np.empty((B, Hkv, nkb + 1), dtype=np.int32)
    d = _Dims(B, T, Hq, Hkv, 0, 0, Hm, 0.0)
    _load().l2a_oracle_route_compact(ctypes.byref(d), _p(mask), _p(row_idx), _p(count), _p(first))
    return row_idx, count, first


# ------------------------------------------------------------------------------------
# router  (Sec. 3.1 Eq. 3)
# ------------------------------------------------------------------------------------
def router(x: np.ndarray, w: np.ndarray, bias: float = 0.0, tau: float = 0.5):
    """x [B,T,C], w [C] -> logit, dhat [B,T] float64 and d [B,1,T] uint8 (a mask shared by all heads)."""
    x = _f32(x)
    B, T, C = x.shape
    w = np.ascontiguousarray(w, dtype=np.float64)
    assert w.shape == (C,) and 0.0 < tau < 1.0
    logit = np.empty((B, T)); dhat = np.empty((B, T)); d = np.empty((B, T), dtype=np.uint8)
    _load().l2a_oracle_router(ctypes.c_int32(B), ctypes.c_int32(T), ctypes.c_int32(C), _p(x), _p(w),
                              ctypes.c_double(bias), ctypes.c_double(tau), _p(logit), _p(dhat), _p(d))
    return logit, dhat, d.reshape(B, 1, T)


# ------------------------------------------------------------------------------------
# forward
# ------------------------------------------------------------------------------------
def fwd_rows(pr: Problem, rows: np.ndarray):
    """rows [n,3] = (b, h, t)  ->  dict S, A, O [n,D], lse_l, lse_g [n]."""
    rows = np.ascontiguousarray(rows, dtype=np.int32).reshape(-1, 3)
    n = rows.shape[0]
    S = np.empty((n, pr.D)); A = np.empty((n, pr.D)); O = np.empty((n, pr.D))
    ll = np.empty(n); lg = np.empty(n)
    d = pr.dims
    _load().l2a_oracle_fwd_rows(ctypes.byref(d), _p(pr.q), _p(pr.k), _p(pr.v), _p(pr.qg), _p(pr.kg),
                                _p(pr.vg), _p(pr.mask), ctypes.c_int64(n), _p(rows), _p(S), _p(A), _p(O),
                                _p(ll), _p(lg))
    return {"S": S, "A": A, "O": O, "lse_l": ll, "lse_g": lg}


def layer_fwd(pr: Problem):
    """Whole layer: S, A, O [B,T,Hq,D]; lse_l, lse_g [B,Hq,T]."""
    r = fwd_rows(pr, pr.all_rows())
    shp = (pr.B, pr.T, pr.Hq, pr.D)
    out = {k: r[k].reshape(shp) for k in ("S", "A", "O")}
    for k in ("lse_l", "lse_g"):
        out[k] = np.ascontiguousarray(r[k].reshape(pr.B, pr.T, pr.Hq).transpose(0, 2, 1))
    return out


# ------------------------------------------------------------------------------------
# backward
# ------------------------------------------------------------------------------------
def bwd_dq_rows(pr: Problem, dO: np.ndarray, rows: np.ndarray):
    """-> dq_l, dq_g [n,D] for rows (b,h,t)."""
    rows = np.ascontiguousarray(rows, dtype=np.int32).reshape(-1, 3)
    dO = _f32(dO)
    n = rows.shape[0]
    dql = np.empty((n, pr.D)); dqg = np.empty((n, pr.D))
    d = pr.dims
    _load().l2a_oracle_bwd_dq_rows(ctypes.byref(d), _p(pr.q), _p(pr.k), _p(pr.v), _p(pr.qg), _p(pr.kg),
                                   _p(pr.vg), _p(pr.mask), _p(dO), ctypes.c_int64(n), _p(rows), _p(dql),
                                   _p(dqg))
    return dql, dqg


def row_deltas(dO: np.ndarray, S: np.ndarray, A: np.ndarray):
    """delta_l = <dO_t, s_t>, delta_g = <dO_t, a_t>, each [B,Hq,T] (inputs [B,T,Hq,D])."""
    dO = np.asarray(dO, dtype=np.float64)
    dl = np.einsum("bthd,bthd->bht", dO, S)
    dg = np.einsum("bthd,bthd->bht", dO, A)
    return np.ascontiguousarray(dl), np.ascontiguousarray(dg)


def bwd_dkdv_keys(pr: Problem, dO: np.ndarray, keys: np.ndarray, lse_l, delta_l, lse_g, delta_g):
    """keys [n,3] = (b, hk, j); statistics are [B,Hq,T] float64 -> dk_l, dv_l, dk_g, dv_g [n,D]."""
    keys = np.ascontiguousarray(keys, dtype=np.int32).reshape(-1, 3)
    dO = _f32(dO)
    n = keys.shape[0]
    outs = [np.empty((n, pr.D)) for _ in range(4)]
    st = [np.ascontiguousarray(x, dtype=np.float64) for x in (lse_l, delta_l, lse_g, delta_g)]
    for x in st:
        assert x.shape == (pr.B, pr.Hq, pr.T)
    d = pr.dims
    _load().l2a_oracle_bwd_dkdv_keys(ctypes.byref(d), _p(pr.q), _p(pr.k), _p(pr.v), _p(pr.qg), _p(pr.kg),
                                     _p(pr.vg), _p(pr.mask), _p(dO), _p(st[0]), _p(st[1]), _p(st[2]),
                                     _p(st[3]), ctypes.c_int64(n), _p(keys), *[_p(o) for o in outs])
    return tuple(outs)


def layer_bwd(pr: Problem, dO: np.ndarray, fwd: Optional[dict] = None):
    """Whole-layer gradients per branch, plus their sums (what shared Q/K/V receive)."""
    if fwd is None:
        fwd = layer_fwd(pr)
    dql, dqg = bwd_dq_rows(pr, dO, pr.all_rows())
    dl, dg = row_deltas(dO, fwd["S"], fwd["A"])
    dkl, dvl, dkg, dvg = bwd_dkdv_keys(pr, dO, pr.all_keys(), fwd["lse_l"], dl, fwd["lse_g"], dg)
    qs = (pr.B, pr.T, pr.Hq, pr.D)
    ks = (pr.B, pr.T, pr.Hkv, pr.D)
    out = {"dq_l": dql.reshape(qs), "dq_g": dqg.reshape(qs), "dk_l": dkl.reshape(ks), "dv_l": dvl.reshape(ks),
           "dk_g": dkg.reshape(ks), "dv_g": dvg.reshape(ks), "delta_l": dl, "delta_g": dg}
    out["dq"] = out["dq_l"] + out["dq_g"]
    out["dk"] = out["dk_l"] + out["dk_g"]
    out["dv"] = out["dv_l"] + out["dv_g"]
    return out

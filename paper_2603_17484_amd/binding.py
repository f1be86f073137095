"""ctypes binding of libl2a.so: argument marshalling only.

The three calls have the names and argument order of the C ABI (include/l2a.h).  Tensors are
torch tensors on the GPU (torch is used for device memory and streams only); every step of
the layer runs inside the HIP library.  There is no fallback: if the library is missing or a
call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libl2a.so")

L2A_BF16, L2A_FP32 = 0, 1
L2A_FLAG_DENSE, L2A_FLAG_SKIP_LOCAL, L2A_FLAG_SKIP_GLOBAL = 1, 2, 4
L2A_FLAG_SEQUENTIAL = 8
L2A_FLAG_RING_CACHE = 16
L2A_FLAG_SCALAR = 1 << 16

EXPORTS = ("l2a_version", "l2a_strerror", "l2a_route_workspace_bytes", "l2a_attn_workspace_bytes",
           "l2a_kblk_entries", "l2a_route_compact", "l2a_route_compact_static", "l2a_router_decide", "l2a_attn_fwd", "l2a_attn_bwd",
           "l2a_decode_workspace_bytes", "l2a_attn_decode",
           "l2a_profile_enable", "l2a_profile_read")


class l2a_params(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("T", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
                ("D", ctypes.c_int32), ("W", ctypes.c_int32), ("mask_heads", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("flags", ctypes.c_int32), ("softmax_scale", ctypes.c_float)]


class L2AError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where} failed with {code}: {lib().l2a_strerror(code).decode()}")


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded HIP library; raises if it has not been built (python -m paper_2603_17484_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: build it with `python -m paper_2603_17484_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32p = ctypes.c_void_p, ctypes.c_void_p
        pp = ctypes.POINTER(l2a_params)
        L.l2a_version.restype = ctypes.c_int
        L.l2a_strerror.restype = ctypes.c_char_p
        L.l2a_strerror.argtypes = [ctypes.c_int]
        L.l2a_route_workspace_bytes.restype = ctypes.c_size_t
        L.l2a_route_workspace_bytes.argtypes = [pp]
        L.l2a_attn_workspace_bytes.restype = ctypes.c_size_t
        L.l2a_attn_workspace_bytes.argtypes = [pp, ctypes.c_int]
        L.l2a_kblk_entries.restype = ctypes.c_int32
        L.l2a_kblk_entries.argtypes = [ctypes.c_int32]
        L.l2a_route_compact.restype = ctypes.c_int
        L.l2a_route_compact.argtypes = [pp, vp, i32p, i32p, i32p, vp, ctypes.c_size_t, vp]
        L.l2a_route_compact_static.restype = ctypes.c_int
        L.l2a_route_compact_static.argtypes = [pp, vp, i32p, i32p, i32p, vp]
        L.l2a_router_decide.restype = ctypes.c_int
        L.l2a_router_decide.argtypes = [pp, ctypes.c_int32, vp, vp, ctypes.c_float, ctypes.c_float, vp, vp, vp, vp]
        L.l2a_decode_workspace_bytes.restype = ctypes.c_size_t
        L.l2a_decode_workspace_bytes.argtypes = [pp]
        L.l2a_attn_decode.restype = ctypes.c_int
        L.l2a_attn_decode.argtypes = [pp] + [vp] * 10 + [vp, ctypes.c_size_t, vp]
        L.l2a_attn_fwd.restype = ctypes.c_int
        L.l2a_attn_fwd.argtypes = [pp] + [vp] * 6 + [i32p] * 3 + [vp] * 5 + [vp, ctypes.c_size_t, vp]
        L.l2a_attn_bwd.restype = ctypes.c_int
        L.l2a_attn_bwd.argtypes = [pp] + [vp] * 7 + [i32p] * 3 + [vp] * 4 + [vp] * 6 + [vp] + [vp, ctypes.c_size_t, vp]
        _lib = L
    return _lib


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors must be contiguous GPU tensors")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def make_params(B, T, Hq, Hkv, D, W, mask_heads=1, dtype=L2A_BF16, flags=0, softmax_scale=None) -> l2a_params:
    if softmax_scale is None:
        softmax_scale = float(D) ** -0.5
    return l2a_params(B, T, Hq, Hkv, D, W, mask_heads, dtype, flags, softmax_scale)


def torch_dtype(p: l2a_params):
    return torch.bfloat16 if p.dtype == L2A_BF16 else torch.float32


def _ws(nbytes: int, device, alloc=None) -> Optional[torch.Tensor]:
    return (alloc or torch.empty)(max(nbytes, 16), dtype=torch.uint8, device=device) if nbytes else None


# ------------------------------------------------------------------------------------------
# the three calls
# ------------------------------------------------------------------------------------------
def l2a_route_compact(p: l2a_params, mask: torch.Tensor, row_idx: torch.Tensor, count: torch.Tensor,
                      kblk_first_row: torch.Tensor, workspace: Optional[torch.Tensor] = None) -> None:
    if workspace is None:
        workspace = _ws(lib().l2a_route_workspace_bytes(ctypes.byref(p)), mask.device)
    rc = lib().l2a_route_compact(ctypes.byref(p), _ptr(mask), _ptr(row_idx), _ptr(count), _ptr(kblk_first_row),
                                 _ptr(workspace), workspace.numel() if workspace is not None else 0, _stream())
    if rc != 0:
        raise L2AError(rc, "l2a_route_compact")


def l2a_route_compact_static(p: l2a_params, mask: torch.Tensor, row_idx: torch.Tensor, count: torch.Tensor,
                             kblk_first_row: torch.Tensor) -> None:
    """l2a_route_compact with the library's static scratch: no workspace, nothing allocated."""
    rc = lib().l2a_route_compact_static(ctypes.byref(p), _ptr(mask), _ptr(row_idx), _ptr(count),
                                        _ptr(kblk_first_row), _stream())
    if rc != 0:
        raise L2AError(rc, "l2a_route_compact_static")


def l2a_router_decide(p: l2a_params, x: torch.Tensor, w: torch.Tensor, bias: float, tau: float, mask: torch.Tensor,
                      dhat: Optional[torch.Tensor] = None, logit: Optional[torch.Tensor] = None) -> None:
    rc = lib().l2a_router_decide(ctypes.byref(p), int(x.shape[-1]), _ptr(x), _ptr(w), float(bias), float(tau),
                                 _ptr(logit), _ptr(dhat), _ptr(mask), _stream())
    if rc != 0:
        raise L2AError(rc, "l2a_router_decide")


def l2a_attn_decode(p: l2a_params, q, k_cache, v_cache, pos, mask, O, lse_local=None, lse_global=None, S_opt=None,
                    A_opt=None, workspace=None) -> None:
    if workspace is None:
        workspace = _ws(lib().l2a_decode_workspace_bytes(ctypes.byref(p)), q.device)
    rc = lib().l2a_attn_decode(ctypes.byref(p), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(pos), _ptr(mask), _ptr(O),
                               _ptr(lse_local), _ptr(lse_global), _ptr(S_opt), _ptr(A_opt), _ptr(workspace),
                               workspace.numel() if workspace is not None else 0, _stream())
    if rc != 0:
        raise L2AError(rc, "l2a_attn_decode")


def l2a_attn_fwd(p: l2a_params, q_loc, k_loc, v_loc, q_glb, k_glb, v_glb, row_idx, count, kblk_first_row, O,
                 lse_local, lse_global, S_opt=None, A_opt=None, workspace=None) -> None:
    rc = lib().l2a_attn_fwd(ctypes.byref(p), _ptr(q_loc), _ptr(k_loc), _ptr(v_loc), _ptr(q_glb), _ptr(k_glb),
                            _ptr(v_glb), _ptr(row_idx), _ptr(count), _ptr(kblk_first_row), _ptr(O),
                            _ptr(lse_local), _ptr(lse_global), _ptr(S_opt), _ptr(A_opt), _ptr(workspace),
                            workspace.numel() if workspace is not None else 0, _stream())
    if rc != 0:
        raise L2AError(rc, "l2a_attn_fwd")


def l2a_attn_bwd(p: l2a_params, dO, q_loc, k_loc, v_loc, q_glb, k_glb, v_glb, row_idx, count, kblk_first_row,
                 S, A, lse_local, lse_global, dq_loc, dk_loc, dv_loc, dq_glb, dk_glb, dv_glb,
                 delta_glb_opt=None, workspace=None) -> None:
    if workspace is None:
        workspace = _ws(lib().l2a_attn_workspace_bytes(ctypes.byref(p), 1), dO.device)
    rc = lib().l2a_attn_bwd(ctypes.byref(p), _ptr(dO), _ptr(q_loc), _ptr(k_loc), _ptr(v_loc), _ptr(q_glb),
                            _ptr(k_glb), _ptr(v_glb), _ptr(row_idx), _ptr(count), _ptr(kblk_first_row), _ptr(S),
                            _ptr(A), _ptr(lse_local), _ptr(lse_global), _ptr(dq_loc), _ptr(dk_loc), _ptr(dv_loc),
                            _ptr(dq_glb), _ptr(dk_glb), _ptr(dv_glb), _ptr(delta_glb_opt), _ptr(workspace),
                            workspace.numel() if workspace is not None else 0, _stream())
    if rc != 0:
        raise L2AError(rc, "l2a_attn_bwd")


class l2a_kernel_time(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char_p), ("ms", ctypes.c_float)]


def profile_enable(on: bool) -> None:
    lib().l2a_profile_enable(1 if on else 0)


def profile_read(max_records: int = 4096):
    """-> [(kernel name, milliseconds)] in launch order since the last read; synchronises."""
    buf = (l2a_kernel_time * max_records)()
    L = lib()
    L.l2a_profile_read.restype = ctypes.c_int
    n = L.l2a_profile_read(buf, max_records)
    return [(buf[i].name.decode(), float(buf[i].ms)) for i in range(min(n, max_records))]


# ------------------------------------------------------------------------------------------
# buffer helpers (allocation only)
# ------------------------------------------------------------------------------------------
# `alloc` has torch.empty's signature (shape, dtype=, device=); the tests pass one that surrounds every
# buffer with guard bands.
def alloc_route(p: l2a_params, device="cuda", alloc=None):
    e = alloc or torch.empty
    G = p.Hq // p.Hkv
    row_idx = e((p.B, p.Hkv, p.T * G), dtype=torch.int32, device=device)
    count = e((p.B, p.Hkv), dtype=torch.int32, device=device)
    first = e((p.B, p.Hkv, lib().l2a_kblk_entries(p.T)), dtype=torch.int32, device=device)
    ws = _ws(lib().l2a_route_workspace_bytes(ctypes.byref(p)), device, alloc)
    return row_idx, count, first, ws


def alloc_fwd(p: l2a_params, device="cuda", branches=True, alloc=None):
    e = alloc or torch.empty
    dt = torch_dtype(p)
    shape = (p.B, p.T, p.Hq, p.D)
    O = e(shape, dtype=dt, device=device)
    lse_l = e((p.B, p.Hq, p.T), dtype=torch.float32, device=device)
    lse_g = e((p.B, p.Hq, p.T), dtype=torch.float32, device=device)
    S = e(shape, dtype=dt, device=device) if branches else None
    A = e(shape, dtype=dt, device=device) if branches else None
    return O, lse_l, lse_g, S, A


def alloc_fwd_workspace(p: l2a_params, device="cuda", alloc=None):
    return _ws(lib().l2a_attn_workspace_bytes(ctypes.byref(p), 0), device, alloc)


def alloc_bwd(p: l2a_params, device="cuda", alloc=None):
    e = alloc or torch.empty
    dt = torch_dtype(p)
    dq = e((p.B, p.T, p.Hq, p.D), dtype=dt, device=device)
    dk = e((p.B, p.T, p.Hkv, p.D), dtype=dt, device=device)
    dv = e((p.B, p.T, p.Hkv, p.D), dtype=dt, device=device)
    ws = _ws(lib().l2a_attn_workspace_bytes(ctypes.byref(p), 1), device, alloc)
    return dq, dk, dv, ws

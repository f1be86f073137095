"""Host-side checks of the C-ABI library (no GPU work): it loads, exports every function the
header declares, and turns bad arguments into error codes before anything is launched."""
import ctypes
import os
import re

import pytest

from paper_2603_17484_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2603_17484_amd.build import build_lib
        build_lib()
    return B.lib()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "l2a.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(l2a_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert set(B.EXPORTS) == set(names), (names, B.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None
    assert lib.l2a_version() == 1
    assert lib.l2a_strerror(0) == b"ok" and b"NULL" in lib.l2a_strerror(-1)


def test_params_struct_layout_matches_header():
    assert ctypes.sizeof(B.l2a_params) == 40
    assert [f[0] for f in B.l2a_params._fields_] == ["B", "T", "Hq", "Hkv", "D", "W", "mask_heads", "dtype",
                                                     "flags", "softmax_scale"]


def test_workspace_queries(lib):
    p = B.make_params(1, 131072, 28, 4, 128, 4096, 28)
    Bn, T, Hq, Hkv, D, G = 1, 131072, 28, 4, 128, 7
    up = lambda x, m: (x + m - 1) // m * m
    kv_copy = Bn * Hkv * D * up(T, 64) * 2            # token-minor copy of K or V, bf16
    redo = up(4 * up(up(T * G, 256) // 256, 8) * Bn * Hkv, 256)   # tiles per (b, KV head): a multiple of 8
    delta = up(4 * Bn * Hq * T, 256)
    cap = up(T * G, 64)
    packed = 2 * (Bn * Hkv * cap * D * 2) + 3 * up(Bn * Hkv * cap * 4, 256)   # Q, dO rows + 3 statistics
    assert lib.l2a_attn_workspace_bytes(ctypes.byref(p), 0) == 2 * kv_copy + redo
    assert lib.l2a_attn_workspace_bytes(ctypes.byref(p), 1) == 2 * delta + 2 * packed
    # short sequences run both branches in one launch: the flags twice and a buffer for A in fp32
    T = 4096
    ps = B.make_params(1, T, 28, 4, 128, 4096, 1)
    kv_copy_s = Bn * Hkv * D * up(T, 64) * 2
    redo_s = up(4 * up(up(T * G, 256) // 256, 8) * Bn * Hkv, 256)
    assert lib.l2a_attn_workspace_bytes(ctypes.byref(ps), 0) == 2 * kv_copy_s + 2 * redo_s + Bn * T * Hq * D * 4
    # ... and the backward shares each key block's row tiles between 4 workgroups (32 blocks x 4 heads x 4 = 512)
    delta_s, cap_s = up(4 * Bn * Hq * T, 256), up(T * G, 64)
    packed_s = 2 * (Bn * Hkv * cap_s * D * 2) + 3 * up(Bn * Hkv * cap_s * 4, 256)
    assert lib.l2a_attn_workspace_bytes(ctypes.byref(ps), 1) == 2 * delta_s + 2 * packed_s + 4 * 2 * Bn * T * Hkv * D * 4
    for flag in (B.L2A_FLAG_SEQUENTIAL, B.L2A_FLAG_DENSE, B.L2A_FLAG_SKIP_GLOBAL, B.L2A_FLAG_SKIP_LOCAL):
        ps.flags = flag
        assert lib.l2a_attn_workspace_bytes(ctypes.byref(ps), 0) == 2 * kv_copy_s + redo_s
    p.flags = B.L2A_FLAG_SCALAR   # scalar kernels: only the two delta arrays
    assert lib.l2a_attn_workspace_bytes(ctypes.byref(p), 0) == 0
    assert lib.l2a_attn_workspace_bytes(ctypes.byref(p), 1) == 2 * delta
    p.flags = 0
    assert lib.l2a_route_workspace_bytes(ctypes.byref(p)) == 4 * 4 * (131072 // 2048)
    assert lib.l2a_route_workspace_bytes(ctypes.byref(B.make_params(2, 5000, 28, 4, 128, 4096, 1))) == 4 * 2 * 4 * 20  # chunks of 256
    assert lib.l2a_kblk_entries(131072) == 2049 and lib.l2a_kblk_entries(65) == 3
    p.flags = B.L2A_FLAG_DENSE
    assert lib.l2a_route_workspace_bytes(ctypes.byref(p)) == 0


BAD = [
    (dict(B=0), -2), (dict(T=0), -2), (dict(Hq=6, Hkv=4), -2), (dict(W=-1), -2), (dict(mask_heads=3), -2),
    (dict(D=96), -3), (dict(dtype=7), -3), (dict(flags=B.L2A_FLAG_SKIP_LOCAL | B.L2A_FLAG_SKIP_GLOBAL), -3),
    (dict(softmax_scale=0.0), -2), (dict(Hq=64, Hkv=2), -3),
    (dict(D=64), -3),      # bf16 runs on the matrix cores, built for D = 128 ...
]


def test_bf16_head_size_64_only_through_the_scalar_kernels(lib):
    """... and is accepted with L2A_FLAG_SCALAR (workspace queries answer 0 for parameters they reject)."""
    p = B.make_params(1, 256, 4, 2, 64, 16, 1, B.L2A_BF16, 0)
    assert lib.l2a_attn_workspace_bytes(ctypes.byref(p), 1) == 0
    p.flags = B.L2A_FLAG_SCALAR
    assert lib.l2a_attn_workspace_bytes(ctypes.byref(p), 1) == 2 * 4 * 4 * 256     # the two delta arrays
    pf = B.make_params(1, 256, 4, 2, 64, 16, 1, B.L2A_FP32, 0)
    assert lib.l2a_attn_workspace_bytes(ctypes.byref(pf), 1) == 2 * 4 * 4 * 256


@pytest.mark.parametrize("change,code", BAD)
def test_bad_params_are_rejected_before_launch(lib, change, code):
    kw = dict(B=1, T=256, Hq=4, Hkv=2, D=128, W=16, mask_heads=1, dtype=B.L2A_BF16, flags=0, softmax_scale=0.1)
    kw.update(change)
    p = B.l2a_params(*[kw[f[0]] for f in B.l2a_params._fields_])
    fake = ctypes.c_void_p(0x1000)   # never dereferenced: validation fails first
    assert lib.l2a_route_compact(ctypes.byref(p), fake, fake, fake, fake, fake, 1 << 20, None) == code
    assert lib.l2a_attn_fwd(ctypes.byref(p), *([fake] * 14), None, 0, None) == code
    assert lib.l2a_attn_bwd(ctypes.byref(p), *([fake] * 20), None, fake, 1 << 30, None) == code


def test_null_alignment_and_workspace_errors(lib):
    p = B.make_params(1, 256, 4, 2, 128, 16)
    ok = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1004)
    pp = ctypes.byref(p)
    assert lib.l2a_route_compact(None, ok, ok, ok, ok, ok, 64, None) == -1
    assert lib.l2a_route_compact(pp, None, ok, ok, ok, ok, 64, None) == -1
    assert lib.l2a_route_compact(pp, ok, ok, ok, ok, None, 0, None) == -4
    assert lib.l2a_route_compact(pp, ok, ok, ok, ok, ok, 1, None) == -4
    assert lib.l2a_route_compact(pp, ok, odd, ok, ok, ok, 64, None) == -5
    fwd = [ok] * 14
    assert lib.l2a_attn_fwd(pp, *(fwd[:9] + [None] + fwd[10:]), None, 0, None) == -1          # O missing
    assert lib.l2a_attn_fwd(pp, *(fwd[:6] + [None] + fwd[7:]), None, 0, None) == -1           # row_idx missing
    assert lib.l2a_attn_fwd(pp, *([odd] + fwd[1:]), None, 0, None) == -5
    bwd = [ok] * 20
    assert lib.l2a_attn_bwd(pp, *bwd, None, None, 0, None) == -4
    assert lib.l2a_attn_bwd(pp, *bwd, None, ok, 8, None) == -4
    assert lib.l2a_attn_bwd(pp, *([None] + bwd[1:]), None, ok, 1 << 30, None) == -1
    # gradient buffers that alias only partly, or alias while the inputs differ, are refused
    a, b2 = ctypes.c_void_p(0x2000), ctypes.c_void_p(0x3000)
    part = bwd[:14] + [a, a, a, a, b2, b2]
    assert lib.l2a_attn_bwd(pp, *part, None, ok, 1 << 30, None) == -3
    diff_in = [ok, ok, ok, ok, a, a, a] + bwd[7:14] + [b2] * 6
    assert lib.l2a_attn_bwd(pp, *diff_in, None, ok, 1 << 30, None) == -3
    # dense mode needs no index arrays and no compaction work
    p.flags = B.L2A_FLAG_DENSE
    assert lib.l2a_route_compact(ctypes.byref(p), None, None, None, None, None, 0, None) == 0


def test_static_scratch_entry_point_argument_errors(lib):
    """l2a_route_compact_static: the checks of l2a_route_compact minus the workspace, plus the fixed
    array's limit of 65536 chunk counters -- all answered before anything touches a GPU."""
    ok, odd = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1004)
    p = B.make_params(1, 256, 4, 2, 128, 16)
    pp = ctypes.byref(p)
    assert lib.l2a_route_compact_static(None, ok, ok, ok, ok, None) == -1
    assert lib.l2a_route_compact_static(pp, None, ok, ok, ok, None) == -1
    assert lib.l2a_route_compact_static(pp, ok, odd, ok, ok, None) == -5
    bad = B.make_params(1, 0, 4, 2, 128, 16)
    assert lib.l2a_route_compact_static(ctypes.byref(bad), ok, ok, ok, ok, None) == -2
    # 64 x 32 (batch, KV head) pairs x 64 chunks of 256 positions = 131072 counters
    big = B.make_params(64, 16384, 32, 32, 128, 16)
    assert lib.l2a_route_workspace_bytes(ctypes.byref(big)) == 4 * 131072
    assert lib.l2a_route_compact_static(ctypes.byref(big), ok, ok, ok, ok, None) == -7
    assert b"static scratch" in lib.l2a_strerror(-7)
    # exactly at the limit the size check passes (what follows needs a GPU, so only the dense no-op is called here)
    p.flags = B.L2A_FLAG_DENSE
    assert lib.l2a_route_compact_static(ctypes.byref(p), None, None, None, None, None) == 0


def test_router_argument_errors(lib):
    p = B.make_params(1, 128, 4, 2, 128, 16)
    x = ctypes.c_void_p(0x1000)
    call = lambda C, xp, wp, tau, mp: lib.l2a_router_decide(ctypes.byref(p), C, xp, wp, ctypes.c_float(0.0),
                                                           ctypes.c_float(tau), None, None, mp, None)
    assert call(12, x, x, 0.5, x) == -2          # C not a multiple of 8
    assert call(0, x, x, 0.5, x) == -2
    assert call(64, x, x, 0.0, x) == -2 and call(64, x, x, 1.0, x) == -2   # tau outside (0, 1)
    assert call(64, None, x, 0.5, x) == -1 and call(64, x, None, 0.5, x) == -1 and call(64, x, x, 0.5, None) == -1
    assert call(64, ctypes.c_void_p(0x1004), x, 0.5, x) == -5


def test_decode_argument_errors_and_workspace(lib):
    p = B.make_params(2, 5000, 28, 4, 128, 4096, 1)
    # one (max, sum, 2 unused, O[128]) partial per 512 keys, query head and branch
    assert lib.l2a_decode_workspace_bytes(ctypes.byref(p)) == 2 * 28 * 2 * ((5000 + 511) // 512) * 132 * 4
    x = ctypes.c_void_p(0x1000)
    big = ctypes.c_size_t(1 << 30)
    call = lambda q=x, k=x, v=x, pos=x, m=x, O=x, ws=x, n=big, pp=p: lib.l2a_attn_decode(
        ctypes.byref(pp), q, k, v, pos, m, O, None, None, None, None, ws, n, None)
    assert call(q=None) == -1 and call(k=None) == -1 and call(pos=None) == -1 and call(m=None) == -1 and call(O=None) == -1
    assert call(ws=None) == -4 and call(n=ctypes.c_size_t(16)) == -4
    assert call(q=ctypes.c_void_p(0x1008)) == -5
    pf = B.make_params(2, 5000, 28, 4, 128, 4096, 1, B.L2A_FP32)
    assert call(pp=pf) == -3 and lib.l2a_decode_workspace_bytes(ctypes.byref(pf)) == 0
    # a ring cache serves the Local branch alone and must hold the whole window
    assert call(pp=B.make_params(2, 5000, 28, 4, 128, 4096, 1, B.L2A_BF16, B.L2A_FLAG_RING_CACHE)) == -3
    ring = B.L2A_FLAG_RING_CACHE | B.L2A_FLAG_SKIP_GLOBAL
    assert call(pp=B.make_params(2, 4096, 28, 4, 128, 4096, 1, B.L2A_BF16, ring)) == -3      # T < W + 1
    assert call(pp=B.make_params(2, 4100, 28, 4, 128, 4096, 1, B.L2A_BF16, ring)) == -3      # not whole sub-blocks

"""The dK/dV kernel's walk over row tiles, checked on the CPU.

The kernel's arithmetic never names the tile it works on: step i trusts that the loads' cursor
fetched the right tile i steps earlier and that the mask class of the running segment fits it.  Both
orders, the three-run split of a set's tiles, the XCD-aware block map and the launch shape live in
csrc/dkdv_walk.hpp, which compiles for the host; tests/dkdv_walk_check.cpp replays them for every
key block and split of a shape and compares with brute force over (row, key) pairs from the mask
definitions (Sec. 2: causal, and the window 0 <= t - j <= W).  Checked: every tile with a pair that
counts is visited exactly once, loads and arithmetic agree on set and order, no tile that needs a
mask runs in an unmasked segment, the cursor parks on the last tile, the block map is a bijection.
"""
import ctypes
import os
import subprocess

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "dkdv_walk_check.cpp")
HDR = os.path.join(HERE, "..", "paper_2603_17484_amd", "csrc", "dkdv_walk.hpp")
LIB = os.path.join(HERE, "libdkdv_walk_check.so")

LOCAL, DENSE, LIST = 0, 1, 2


@pytest.fixture(scope="module")
def chk():
    if not os.path.exists(LIB) or os.path.getmtime(LIB) < max(os.path.getmtime(SRC), os.path.getmtime(HDR)):
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-shared", "-fPIC", "-o", LIB, SRC])
    L = ctypes.CDLL(LIB)
    L.walk_check.restype = ctypes.c_int
    L.walk_check.argtypes = [ctypes.c_int] * 6 + [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p,
                                                  ctypes.c_char_p, ctypes.c_int]
    L.walk_launch_shape.argtypes = [ctypes.c_int, ctypes.c_longlong, ctypes.c_void_p]
    return L


def routed_positions(T, G, f, per_head, seed):
    """Positions of the routed rows of one KV group, ascending by row code pos * G + g."""
    rng = np.random.default_rng(seed)
    d = rng.random((T, G)) < f if per_head else np.repeat(rng.random((T, 1)) < f, G, axis=1)
    return np.ascontiguousarray(np.argwhere(d)[:, 0], dtype=np.int32)   # argwhere is row-major: (pos, g) ascending


def check(chk, T, G, W, chunk, nsplit, kinds, pos=None):
    kinds_a = np.asarray(kinds, dtype=np.int32)
    pos = np.zeros(0, np.int32) if pos is None else pos
    msg = ctypes.create_string_buffer(512)
    stats = np.zeros(2, dtype=np.int64)
    rc = chk.walk_check(T, G, W, chunk, nsplit, len(kinds), kinds_a.ctypes.data, pos.ctypes.data, len(pos),
                        stats.ctypes.data, msg, 512)
    assert rc == 0, f"T={T} G={G} W={W} chunk={chunk} nsplit={nsplit} sets={kinds}: {msg.value.decode()}"
    return stats


def launch_shape(chk, T, bh):
    out = np.zeros(4, dtype=np.int32)
    chk.walk_launch_shape(T, bh, out.ctypes.data)
    return dict(nblk=int(out[0]), chunk=int(out[1]), nsplit=int(out[2]), grid_x=int(out[3]))


def test_launch_shape_of_the_benchmark_configurations(chk):
    assert launch_shape(chk, 131072, 4) == dict(nblk=1024, chunk=32, nsplit=1, grid_x=1024)
    assert launch_shape(chk, 65536, 4) == dict(nblk=512, chunk=16, nsplit=1, grid_x=512)
    assert launch_shape(chk, 32768, 4) == dict(nblk=256, chunk=8, nsplit=1, grid_x=256)
    assert launch_shape(chk, 8192, 4) == dict(nblk=64, chunk=2, nsplit=1, grid_x=64)      # the mid-size whole-tensor case
    assert launch_shape(chk, 4096, 4) == dict(nblk=32, chunk=1, nsplit=4, grid_x=32)
    assert launch_shape(chk, 3000, 4) == dict(nblk=24, chunk=1, nsplit=8, grid_x=24)
    assert launch_shape(chk, 1, 1) == dict(nblk=1, chunk=1, nsplit=8, grid_x=8)


SHAPES = [  # (T, G, W): lengths around tile and block edges, windows from 0 to beyond the sequence
    (1, 1, 0), (31, 3, 5), (128, 1, 0), (129, 7, 40), (300, 4, 63), (513, 2, 64), (700, 7, 127), (1000, 8, 128),
    (1100, 4, 300), (1537, 1, 1536), (1200, 7, 5000), (2049, 2, 1),
]


@pytest.mark.parametrize("T,G,W", SHAPES)
def test_walk_visits_every_tile_once_in_step_with_the_loads(chk, T, G, W):
    nblk = (T + 127) // 128
    for chunk in sorted({1, 2, 3, max(1, nblk // 2), 32}):
        for nsplit in (1, 2, 8):
            pos = routed_positions(T, G, 0.3, per_head=(T % 2 == 0), seed=T + G)
            # the layer's own combinations: both branches on shared inputs, each alone, dense mode with and without Local
            check(chk, T, G, W, chunk, nsplit, [LOCAL, LIST], pos)
            check(chk, T, G, W, chunk, nsplit, [LOCAL])
            check(chk, T, G, W, chunk, nsplit, [LIST], pos)
            check(chk, T, G, W, chunk, nsplit, [LOCAL, DENSE])
            check(chk, T, G, W, chunk, nsplit, [DENSE])


@pytest.mark.parametrize("f", [0.0, 0.02, 1.0])
def test_walk_with_degenerate_row_lists(chk, f):
    """No routed row, a handful (key blocks with an empty list range), all rows routed."""
    T, G, W = 900, 4, 100
    pos = routed_positions(T, G, f, per_head=True, seed=5)
    for chunk in (1, 4):
        check(chk, T, G, W, chunk, 1, [LOCAL, LIST], pos)
        check(chk, T, G, W, chunk, 2, [LIST], pos)
    last = np.array([T - 1] * G, dtype=np.int32)             # only the last position routed
    check(chk, T, G, W, 2, 1, [LOCAL, LIST], last)
    first_ = np.array([0] * G, dtype=np.int32)               # only position 0 routed
    check(chk, T, G, W, 2, 1, [LOCAL, LIST], first_)


def test_walk_at_the_mid_size_whole_tensor_shape(chk):
    """T = 8192, G = 7, W = 1024 with the launch shape the host picks for Hkv = 4 (one workgroup per key
    block, chunks of 2): the rotated Local walk and the reversed Global walk of the long configurations."""
    T, G, W = 8192, 7, 1024
    shape = launch_shape(chk, T, 4)
    assert shape["nsplit"] == 1 and shape["chunk"] == 2
    pos = routed_positions(T, G, 0.2, per_head=True, seed=61)
    stats = check(chk, T, G, W, shape["chunk"], shape["nsplit"], [LOCAL, LIST], pos)
    assert stats[0] > 64 * (W * G // 32)           # every key block walks at least its window's tiles
    check(chk, T, G, W, shape["chunk"], shape["nsplit"], [LOCAL, DENSE])


def test_walk_with_long_chunks_and_a_wide_window(chk):
    """Chunks of 32 key blocks as at 128K tokens, window of several key blocks: shorter stand-in lengths."""
    pos = routed_positions(6000, 7, 0.2, per_head=True, seed=9)
    check(chk, 6000, 7, 2000, 32, 1, [LOCAL, LIST], pos)
    check(chk, 6000, 7, 2000, 16, 1, [LOCAL, DENSE])

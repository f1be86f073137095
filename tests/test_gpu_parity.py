"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element, on
seeded inputs small enough for the oracle yet spanning several tiles and a ragged tail, and at the
benchmark's full sizes on sampled rows, sampled keys and whole KV groups.

Bars (stated once, in tests/tolerance.py): compaction bit-exact; fp32 max-abs <= 1e-4; log-sum-exp
1e-2 (bf16) / 1e-5 (fp32); bf16 max-abs <= 2e-2 on O, S, A, dQ, dK, dV -- held strictly on every
gradient row (token, head) whose largest reference element is <= 1, and widened only where bf16
storage or the bf16 operands of the matrix cores cannot hold it: outputs max(2e-2, 2^-8 |ref|),
gradient rows with larger elements 2e-2 + 2^-7 max_c |ref|.  Every comparison prints the raw max-abs
error and the number of elements above a flat 2e-2.

Every output and workspace buffer of the whole-layer cases sits between guard bands that are checked
after the kernels ran.
"""
import numpy as np
import pytest
import torch

from paper_2603_17484_amd import binding as B
from paper_2603_17484_amd import inputs as gen
from paper_2603_17484_amd.runner import layer_from_numpy, to_device, to_host
from tests.gpu_helpers import assert_close, assert_lse, make_case, run_and_check

pytestmark = pytest.mark.gpu


# ------------------------------------------------------------------------------------------
# compaction
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("T", [1, 63, 64, 65, 2047, 2048, 2049, 5000])
@pytest.mark.parametrize("Hm", ["shared", "kv", "q"])
def test_route_compact_bit_exact(oracle, T, Hm):
    Hq, Hkv = 14, 2
    hm = {"shared": 1, "kv": Hkv, "q": Hq}[Hm]
    for f, seed in ((0.0, 0), (1.0, 1), (0.2, 2), (0.9, 3)):
        mask = (np.random.default_rng(seed * 7919 + T).random((2, hm, T)) < f).astype(np.uint8) * 3
        p = B.make_params(2, T, Hq, Hkv, 128, 16, hm)
        row_idx, count, first, ws = B.alloc_route(p)
        row_idx.fill_(12345); first.fill_(-7)
        B.l2a_route_compact(p, torch.from_numpy(mask).cuda(), row_idx, count, first, ws)
        torch.cuda.synchronize()
        r, c, k = oracle.route_compact(mask, Hq, Hkv)
        assert np.array_equal(count.cpu().numpy(), c)
        assert np.array_equal(first.cpu().numpy(), k)
        assert np.array_equal(row_idx.cpu().numpy(), r)


@pytest.mark.parametrize("name", ["prefill_128k", "qwen3_8b_128k"])
def test_route_compact_full_size(oracle, name):
    w = gen.workload(name)
    mask = gen.make_mask(w, 0)
    p = B.make_params(w.B, w.T, w.Hq, w.Hkv, w.D, w.W, w.mask_heads)
    row_idx, count, first, ws = B.alloc_route(p)
    B.l2a_route_compact(p, torch.from_numpy(mask).cuda(), row_idx, count, first, ws)
    torch.cuda.synchronize()
    r, c, k = oracle.route_compact(mask, w.Hq, w.Hkv)
    assert np.array_equal(count.cpu().numpy(), c) and np.array_equal(first.cpu().numpy(), k)
    assert np.array_equal(row_idx.cpu().numpy(), r)


# ------------------------------------------------------------------------------------------
# the tiny fp32 configuration, whole layer forward + backward
# ------------------------------------------------------------------------------------------
def test_tiny_fp32_config(oracle):
    x = gen.make_inputs(gen.workload("tiny_fp32"), seed=0)
    assert x.mask[0, 0, 0] == 1
    run_and_check(oracle, x)


@pytest.mark.parametrize("D", [64, 128])
def test_fp32_gqa_per_head_mask(oracle, D):
    run_and_check(oracle, make_case(B_=2, T=333, Hq=6, Hkv=2, D=D, W=40, dtype="fp32", Hm=6, f=0.3, seed=4))


def test_fp32_separate_branch_inputs(oracle):
    run_and_check(oracle, make_case(T=200, Hq=4, Hkv=2, D=64, W=17, dtype="fp32", Hm=2, seed=5), separate=True,
                  scale=0.2)


# ------------------------------------------------------------------------------------------
# bf16 (matrix-core kernels)
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("order", [0, B.L2A_FLAG_SEQUENTIAL])
@pytest.mark.parametrize("Hm", ["shared", "q"])
def test_bf16_layer_several_tiles_ragged(oracle, Hm, order):
    """order: both branches in one launch (short sequences) / one after the other."""
    Hq, Hkv = 14, 2
    x = make_case(B_=1, T=1037, Hq=Hq, Hkv=Hkv, W=300, Hm=1 if Hm == "shared" else Hq, f=0.3, seed=6)
    run_and_check(oracle, x, flags=order)


def test_bf16_batch_and_kv_mask(oracle):
    run_and_check(oracle, make_case(B_=2, T=515, Hq=8, Hkv=2, W=64, Hm=2, f=0.5, seed=7))


def test_bf16_dense_mode(oracle):
    run_and_check(oracle, make_case(T=700, Hq=4, Hkv=1, W=128, seed=8), flags=B.L2A_FLAG_DENSE)


def test_bf16_branch_flags(oracle):
    x = make_case(T=450, Hq=4, Hkv=2, W=50, f=0.4, seed=9)
    run_and_check(oracle, x, flags=B.L2A_FLAG_SKIP_LOCAL)
    run_and_check(oracle, x, flags=B.L2A_FLAG_SKIP_GLOBAL)
    run_and_check(oracle, x, flags=B.L2A_FLAG_SKIP_LOCAL | B.L2A_FLAG_DENSE)


@pytest.mark.parametrize("order", [0, B.L2A_FLAG_SEQUENTIAL])
def test_bf16_forward_without_branch_outputs(oracle, order):
    """Inference: S_opt and A_opt are NULL; with both branches in one launch a then lives in the workspace."""
    x = make_case(T=900, Hq=8, Hkv=2, W=100, f=0.4, seed=12)
    ref = oracle.layer_fwd(oracle.Problem(x.q, x.k, x.v, x.mask, x.w.W))
    lay = layer_from_numpy(x.q, x.k, x.v, x.mask, x.w.W, "bf16", order)
    lay.route()
    lay.forward(save_branches=False)
    torch.cuda.synchronize()
    assert_close("O", to_host(lay.O), ref["O"], "bf16")
    assert_lse("lse_local", to_host(lay.lse_l), ref["lse_l"], "bf16")
    assert_lse("lse_global", to_host(lay.lse_g), ref["lse_g"], "bf16")


def test_bf16_one_launch_equals_sequential_bit_for_bit():
    """Short sequences: both branches in one launch and o = s + d a formed afterwards from the fp32 a --
    the same bits as the Global kernel adding its result to the stored s."""
    x = make_case(T=2000, Hq=14, Hkv=2, W=300, Hm=14, f=0.3, seed=13)
    outs = []
    for order in (0, B.L2A_FLAG_SEQUENTIAL):
        lay = layer_from_numpy(x.q, x.k, x.v, x.mask, x.w.W, "bf16", order)
        lay.route()
        lay.forward()
        torch.cuda.synchronize()
        outs.append({n: getattr(lay, n).clone() for n in ("O", "S", "A", "lse_l", "lse_g")})
    for n in outs[0]:
        assert torch.equal(outs[0][n], outs[1][n]), n


@pytest.mark.parametrize("order", [0, B.L2A_FLAG_SEQUENTIAL])
def test_bf16_workspaces_may_hold_anything(order):
    """The workspaces are scratch: filled with 0xFF bytes (NaN patterns, negative integers) before
    the calls, they must give the same bits as before."""
    x = make_case(T=1100, Hq=14, Hkv=2, W=200, Hm=14, f=0.3, seed=14)
    lay = layer_from_numpy(x.q, x.k, x.v, x.mask, x.w.W, "bf16", order)
    dO = to_device(x.dO, "bf16")
    names = ("O", "S", "A", "lse_l", "lse_g", "dq", "dk", "dv")

    def step():
        lay.route(); lay.forward(); lay.backward(dO)
        torch.cuda.synchronize()
        return {n: getattr(lay, n).clone() for n in names}

    first = step()
    for ws in (lay.route_ws, lay.fwd_ws, lay.bwd_ws):
        ws.view(torch.uint8).fill_(0xFF)
    second = step()
    for n in names:
        assert not torch.isnan(second[n].float()).any(), n
        assert torch.equal(first[n], second[n]), n


def test_bf16_separate_branch_inputs(oracle):
    run_and_check(oracle, make_case(T=390, Hq=4, Hkv=2, W=33, f=0.4, seed=10), separate=True)


@pytest.mark.parametrize("W", [0, 1, 63, 64, 100000])
def test_bf16_window_edges(oracle, W):
    run_and_check(oracle, make_case(T=300, Hq=2, Hkv=1, W=W, f=0.3, seed=11 + W % 7))


def test_bf16_degenerate_masks(oracle):
    T = 260
    none = np.zeros((1, 1, T), np.uint8)
    run_and_check(oracle, make_case(T=T, Hq=2, Hkv=1, W=20, mask=none, seed=20))         # n_c = 0: O = S
    one = none.copy(); one[0, 0, 200] = 1
    run_and_check(oracle, make_case(T=T, Hq=2, Hkv=1, W=20, mask=one, seed=21))          # a single routed token
    first = none.copy(); first[0, 0, 0] = 1
    run_and_check(oracle, make_case(T=T, Hq=2, Hkv=1, W=20, mask=first, seed=22))        # only token 0
    run_and_check(oracle, make_case(T=1, Hq=2, Hkv=1, W=4, f=1.0, seed=23))              # T = 1
    run_and_check(oracle, make_case(T=64, Hq=7, Hkv=1, W=4096, f=1.0, seed=24))          # one block exactly


def test_bf16_scalar_kernels_agree(oracle):
    """The scalar-FMA kernels on bf16 storage are a second GPU implementation of the same layer."""
    run_and_check(oracle, make_case(T=300, Hq=4, Hkv=2, W=40, f=0.3, seed=30), flags=B.L2A_FLAG_SCALAR)


def test_bf16_custom_scale(oracle):
    run_and_check(oracle, make_case(T=300, Hq=4, Hkv=2, W=40, f=0.3, seed=31), scale=0.05)


# ------------------------------------------------------------------------------------------
# forward softmax reference: scores that grow along the sequence
# ------------------------------------------------------------------------------------------
def growing_scores_case(top, T=900, Hq=4, Hkv=2, W=200, seed=40):
    """Keys whose score against every query grows linearly with the position up to `top` (natural
    log units): the latest key dominates every row, far above the scores of a row's first blocks."""
    x = make_case(T=T, Hq=Hq, Hkv=Hkv, W=W, f=0.5, seed=seed)
    D = x.q.shape[-1]
    x.q[...] = gen.round_to_bf16(1.0 + 0.05 * x.q)
    ramp = (np.arange(T, dtype=np.float64) / T * top * np.sqrt(D) / D).astype(np.float32)
    x.k[...] = gen.round_to_bf16(ramp[None, :, None, None] + 0.02 * x.k)
    return x


def redo_flags(lay):
    """Flags of the tiles the pipelined forward kernel left to the fix-up kernel: they sit behind the two
    token-minor V copies in the forward workspace -- those of the last branch run, or of both branches
    when one launch carried both (short sequences without L2A_FLAG_SEQUENTIAL)."""
    p = lay.p
    up = lambda x, m: (x + m - 1) // m * m
    kv_copy = p.B * p.Hkv * p.D * up(p.T, 64) * 2
    n = up(up(p.T * (p.Hq // p.Hkv), 256) // 256, 8) * p.B * p.Hkv   # flags of one branch
    both = lay.fwd_ws.numel() > 2 * kv_copy + up(4 * n, 256)
    return lay.fwd_ws[2 * kv_copy:2 * kv_copy + (2 if both else 1) * 4 * n].view(torch.int32).cpu().numpy()


SEQ = [0, B.L2A_FLAG_SEQUENTIAL]   # short sequences: both branches in one launch / one after the other


@pytest.mark.parametrize("order", SEQ)
def test_bf16_scores_above_reference_without_overflow(oracle, order):
    """Scores exceed the fixed reference by up to e^40: sums stay in range, no tile is redone."""
    lay, _ = run_and_check(oracle, growing_scores_case(40.0), flags=order)
    assert not redo_flags(lay).any()


@pytest.mark.parametrize("order", SEQ)
def test_bf16_scores_overflow_reference_fixup_kernel(oracle, order):
    """Scores exceed the reference by up to e^300: row sums overflow, the fix-up kernel takes over.
    Forward only: keys this large (|k| ~ 26 in every channel) multiply the rounding of the saved
    bf16 outputs, through delta = <dO, out>, into dQ = scale sum_j p (dp - delta) k_j beyond any
    fixed tolerance -- a property of bf16 storage of the outputs, not of the kernels."""
    lay, _ = run_and_check(oracle, growing_scores_case(300.0), flags=order, backward=False)
    assert redo_flags(lay).any()


@pytest.mark.parametrize("order", SEQ)
def test_bf16_large_values_overflow_the_accumulators_not_the_row_sums(oracle, order):
    """Scores exceed a row's fixed reference by up to e^55 in the Global branch (the reference is the largest
    score among the tile's first 128 keys, ~64 * 128 / 900 here) and by up to e^64 in the Local branch (rows
    none of whose keys lie in their tile's first blocks take 0) -- row sums of 1e25 and 1e29, inside the
    range the pipelined kernel accepts -- while the values are of magnitude 1e15: the products overflow the
    fp32 output accumulators although no row sum does.  The tile must be handed to the fix-up kernel (the
    running-maximum algorithm of App. C Alg. 1, whose weights never exceed one).  The layer is linear in
    V, so results are compared after dividing by the values' scale."""
    scale_v = 2.0 ** 50            # 1.1e15, a power of two: the scaled values are bf16 numbers as well
    x = growing_scores_case(64.0)
    ref = oracle.layer_fwd(oracle.Problem(x.q, x.k, x.v, x.mask, x.w.W))     # with values of magnitude one
    lay = layer_from_numpy(x.q, x.k, x.v * np.float32(scale_v), x.mask, x.w.W, "bf16", order)
    unit = layer_from_numpy(x.q, x.k, x.v, x.mask, x.w.W, "bf16", order)
    for l_ in (lay, unit):
        l_.route(); l_.forward()
    torch.cuda.synchronize()
    print("tiles handed to the fix-up kernel: values of magnitude one", np.flatnonzero(redo_flags(unit)),
          "scaled values", np.flatnonzero(redo_flags(lay)), flush=True)
    assert not redo_flags(unit).any(), "with values of magnitude one nothing overflows"
    assert redo_flags(lay).any(), "overflowing accumulators must send the tile to the fix-up kernel"
    for n in ("O", "S", "A"):
        got = to_host(getattr(lay, n))
        assert np.isfinite(got).all(), n
        assert_close(n, got / scale_v, ref[n], "bf16")
    assert_lse("lse_global", to_host(lay.lse_g), ref["lse_g"], "bf16")


def test_bf16_scores_falling_along_sequence(oracle):
    run_and_check(oracle, growing_scores_case(-300.0), backward=False)
    run_and_check(oracle, growing_scores_case(-40.0))


@pytest.mark.parametrize("T,Hq,Hkv", [(129, 7, 1), (193, 3, 1), (2049, 2, 2), (4100, 14, 2), (300, 16, 1)])
def test_bf16_ragged_tiles(oracle, T, Hq, Hkv):
    """Row counts and key counts just past tile boundaries; T * G not a multiple of the row tile."""
    for order in (0, B.L2A_FLAG_SEQUENTIAL):
        run_and_check(oracle, make_case(T=T, Hq=Hq, Hkv=Hkv, W=70, f=0.35, seed=50 + T % 13), flags=order)


def _random_shape(i):
    """Seeded draw of a small layer: lengths around tile and block edges, every head layout and mask
    granularity, windows from 0 to beyond the sequence, routed fractions from none to all."""
    rng = np.random.default_rng(7000 + i)
    Hkv = int(rng.choice([1, 2, 3]))
    G = int(rng.choice([1, 2, 4, 7, 8]))
    base = int(rng.choice([1, 31, 64, 127, 128, 256, 300, 512, 1000, 1537, 2304]))
    T = max(1, base + int(rng.integers(-2, 3)))
    W = int(rng.choice([0, 1, 5, 63, 64, 65, 200, 511, T - 1 if T > 1 else 0, T + 7]))
    Hm = int(rng.choice([1, Hkv, Hkv * G]))
    f = float(rng.choice([0.0, 0.05, 0.2, 0.5, 0.9, 1.0]))
    Bn = int(rng.choice([1, 1, 2]))
    return dict(B_=Bn, T=T, Hq=Hkv * G, Hkv=Hkv, W=W, Hm=Hm, f=f, seed=7100 + i)


@pytest.mark.parametrize("i", range(16))
def test_bf16_random_shapes(oracle, i):
    """Whole tensors, forward and backward, on shapes nobody picked by hand."""
    cfg = _random_shape(i)
    order = B.L2A_FLAG_SEQUENTIAL if i % 2 else 0   # half of them with the branches one after the other
    print("case", cfg, "flags", order, flush=True)
    run_and_check(oracle, make_case(**cfg), flags=order)


# ------------------------------------------------------------------------------------------
# training variant with Global attention for every token (Sec. 3.3), composed from the same calls
# ------------------------------------------------------------------------------------------
def test_global_for_all_training_variant(oracle):
    """With a small probability a training step computes Global attention for all tokens, still
    merges o = s + d a with the router's decisions, and back-propagates <dO_t, a_t> to the router for
    every token (Sec. 3.3, Eq. 7).  Composition: a dense Global-only forward gives a_t and its
    log-sum-exp for all t; the normal sparse forward gives O and S; the backward call takes the
    dense A and log-sum-exp with the sparse row lists, so q/k/v gradients still come from routed
    rows only while delta_glb is <dO_t, a_t> for every t."""
    x = make_case(T=700, Hq=6, Hkv=2, W=90, Hm=6, f=0.3, seed=70)
    w = x.w
    pr = oracle.Problem(x.q, x.k, x.v, x.mask, w.W)
    pr_all = oracle.Problem(x.q, x.k, x.v, np.ones_like(x.mask), w.W)
    ref, ref_all = oracle.layer_fwd(pr), oracle.layer_fwd(pr_all)
    g = oracle.layer_bwd(pr, x.dO, ref)

    sparse = layer_from_numpy(x.q, x.k, x.v, x.mask, w.W, w.dtype)
    dense = layer_from_numpy(x.q, x.k, x.v, x.mask, w.W, w.dtype, flags=B.L2A_FLAG_DENSE | B.L2A_FLAG_SKIP_LOCAL)
    sparse.route(); sparse.forward()
    dense.forward()
    torch.cuda.synchronize()
    assert_close("O", to_host(sparse.O), ref["S"] + ref["A"], w.dtype)          # forward unchanged
    assert_close("A", to_host(dense.A), ref_all["A"], w.dtype)                  # a_t for every token
    sparse.A, sparse.lse_g = dense.A, dense.lse_g                               # hand the dense branch to the backward
    sparse.backward(to_device(x.dO, w.dtype), want_delta=True)
    torch.cuda.synchronize()
    assert_close("dq", to_host(sparse.dq), g["dq_l"] + g["dq_g"], w.dtype)
    assert_close("dk", to_host(sparse.dk), g["dk_l"] + g["dk_g"], w.dtype)
    assert_close("dv", to_host(sparse.dv), g["dv_l"] + g["dv_g"], w.dtype)
    delta_all = np.einsum("bthd,bthd->bht", x.dO.astype(np.float64), ref_all["A"])
    err = np.abs(to_host(sparse.delta_g) - delta_all).max()
    assert err <= 3e-2, f"router-gradient factor <dO, a> max err {err}"


# ------------------------------------------------------------------------------------------
# router front-end (Sec. 3.1 Eq. 3)
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,C,T", [("bf16", 3584, 1000), ("fp32", 512, 333), ("bf16", 8, 5), ("bf16", 1032, 4097)])
@pytest.mark.parametrize("tau", [0.5, 0.2])
def test_router_decide(oracle, dtype, C, T, tau):
    """Scores against the fp64 oracle; decisions must agree wherever the fp64 logit is not within the
    fp32 accumulation error of the threshold (there either answer is a correct fp32 decision)."""
    rng = np.random.default_rng(C + T)
    Bn = 2
    x = rng.standard_normal((Bn, T, C)).astype(np.float32)
    if dtype == "bf16":
        x = gen.round_to_bf16(x)
    w = (rng.standard_normal(C) / np.sqrt(C)).astype(np.float32)
    bias = 0.1
    lg, dhat, d = oracle.router(x, w.astype(np.float64), bias, tau)
    p = B.make_params(Bn, T, 4, 2, 128, 16, 1, B.L2A_BF16 if dtype == "bf16" else B.L2A_FP32)
    xd = to_device(x, dtype)
    wd = torch.from_numpy(w).cuda()
    mask = torch.full((Bn, 1, T), 7, dtype=torch.uint8, device="cuda")
    dh = torch.empty((Bn, T), dtype=torch.float32, device="cuda")
    lo = torch.empty((Bn, T), dtype=torch.float32, device="cuda")
    B.l2a_router_decide(p, xd, wd, bias, tau, mask, dh, lo)
    torch.cuda.synchronize()
    got_lg, got_dh, got_d = lo.cpu().numpy().astype(np.float64), dh.cpu().numpy().astype(np.float64), mask.cpu().numpy()
    # fp32 sum of C products of O(1/sqrt(C)) terms: a few 1e-7 per unit of |logit| ~ 1
    assert np.abs(got_lg - lg).max() <= 2e-5
    assert np.abs(got_dh - dhat).max() <= 1e-5
    thr = np.log(tau / (1 - tau))
    sure = np.abs(lg - thr) > 2e-5
    assert sure.mean() > 0.99
    assert np.array_equal(got_d[:, 0][sure], d[:, 0][sure])
    assert set(np.unique(got_d)) <= {0, 1}
    # the mask feeds the compaction as a shared one
    row_idx, count, first, ws = B.alloc_route(p)
    B.l2a_route_compact(p, mask, row_idx, count, first, ws)
    torch.cuda.synchronize()
    r, c, k = oracle.route_compact(got_d, 4, 2)
    assert np.array_equal(row_idx.cpu().numpy(), r) and np.array_equal(count.cpu().numpy(), c)


# ------------------------------------------------------------------------------------------
# decode step (Sec. 3.4): one new token per sequence against the KV cache
# ------------------------------------------------------------------------------------------
def decode_case(oracle, Bn, Tcap, Hq, Hkv, W, pos, Hm, f, seed, flags=0, pos_given=None, poison=False):
    """The oracle is the layer's definition at row t = pos[b]: whatever the cache holds beyond pos is
    out of reach of a causal row, so the same K/V arrays serve as the cache."""
    rng = np.random.default_rng(seed)
    D = 128
    k = gen.normal_tensor((Bn, Tcap, Hkv, D), seed, 1, "bf16")
    v = gen.normal_tensor((Bn, Tcap, Hkv, D), seed, 2, "bf16")
    qn = gen.normal_tensor((Bn, Hq, D), seed, 3, "bf16")
    d = (rng.random((Bn, Hm)) < f).astype(np.uint8)
    pos = np.asarray(pos, dtype=np.int32)
    dense = bool(flags & B.L2A_FLAG_DENSE)
    # oracle: a [B,T,Hq,D] query tensor that is zero except at each sequence's own position
    qfull = np.zeros((Bn, Tcap, Hq, D), np.float32)
    mfull = np.zeros((Bn, Hm, Tcap), np.uint8)
    for b in range(Bn):
        qfull[b, pos[b]] = qn[b]
        mfull[b, :, pos[b]] = 1 if dense else d[b]
    pr = oracle.Problem(qfull, k, v, mfull, W)
    rows = np.array([(b, h, pos[b]) for b in range(Bn) for h in range(Hq)], dtype=np.int32)
    ref = oracle.fwd_rows(pr, rows)

    p = B.make_params(Bn, Tcap, Hq, Hkv, D, W, Hm, B.L2A_BF16, flags)
    out = {n: torch.full((Bn, Hq, D), 7.0, dtype=torch.bfloat16, device="cuda") for n in ("O", "S", "A")}
    lse_l = torch.zeros((Bn, Hq), dtype=torch.float32, device="cuda")
    lse_g = torch.zeros((Bn, Hq), dtype=torch.float32, device="cuda")
    kd, vd = to_device(k, "bf16"), to_device(v, "bf16")
    if poison:   # cache rows behind the new token are not written yet: they may hold anything
        for b in range(Bn):
            kd[b, pos[b] + 1:] = float("nan")
            vd[b, pos[b] + 1:] = float("nan")
    B.l2a_attn_decode(p, to_device(qn, "bf16"), kd, vd,
                      torch.from_numpy(pos if pos_given is None else np.asarray(pos_given, dtype=np.int32)).cuda(),
                      None if dense else torch.from_numpy(d).cuda(), out["O"], lse_l, lse_g,
                      out["S"], out["A"])
    torch.cuda.synchronize()
    skip_l, skip_g = bool(flags & B.L2A_FLAG_SKIP_LOCAL), bool(flags & B.L2A_FLAG_SKIP_GLOBAL)
    rs = 0 * ref["S"] if skip_l else ref["S"]
    ra = 0 * ref["A"] if skip_g else ref["A"]
    shp = (Bn, Hq, D)
    assert_close("S", to_host(out["S"]), rs.reshape(shp), "bf16")
    assert_close("A", to_host(out["A"]), ra.reshape(shp), "bf16")
    assert_close("O", to_host(out["O"]), (rs + ra).reshape(shp), "bf16")
    if not skip_l:
        assert_lse("lse_local", lse_l.cpu().numpy().astype(np.float64), ref["lse_l"].reshape(Bn, Hq), "bf16")
    if not skip_g:
        assert_lse("lse_global", lse_g.cpu().numpy().astype(np.float64), ref["lse_g"].reshape(Bn, Hq), "bf16")
    return d


@pytest.mark.parametrize("Hq,Hkv,Hm", [(28, 4, 1), (8, 2, 8), (4, 4, 4), (16, 1, 1)])
def test_decode_matches_layer_row(oracle, Hq, Hkv, Hm):
    hm = {1: 1}.get(Hm, Hm)
    d = decode_case(oracle, Bn=3, Tcap=3000, Hq=Hq, Hkv=Hkv, W=700, pos=[2999, 1234, 5], Hm=hm, f=0.5, seed=80 + Hq)
    assert d.shape == (3, hm)


@pytest.mark.parametrize("pos", [[0], [1], [31], [32], [511], [512], [513], [1023], [1500]])
def test_decode_positions_at_tile_edges(oracle, pos):
    decode_case(oracle, Bn=1, Tcap=1501, Hq=14, Hkv=2, W=100, pos=pos, Hm=1, f=1.0, seed=90 + pos[0])


@pytest.mark.parametrize("W", [0, 31, 100000])
def test_decode_window_edges(oracle, W):
    decode_case(oracle, Bn=2, Tcap=1100, Hq=8, Hkv=2, W=W, pos=[1099, 700], Hm=8, f=0.6, seed=95)


def test_decode_flags_and_unrouted(oracle):
    decode_case(oracle, Bn=2, Tcap=900, Hq=8, Hkv=2, W=64, pos=[899, 10], Hm=1, f=0.0, seed=96)    # nobody routed: O = S
    decode_case(oracle, Bn=2, Tcap=900, Hq=8, Hkv=2, W=64, pos=[899, 10], Hm=8, f=0.5, seed=97, flags=B.L2A_FLAG_DENSE)
    decode_case(oracle, Bn=2, Tcap=900, Hq=8, Hkv=2, W=64, pos=[899, 10], Hm=8, f=0.5, seed=98, flags=B.L2A_FLAG_SKIP_LOCAL)
    decode_case(oracle, Bn=2, Tcap=900, Hq=8, Hkv=2, W=64, pos=[899, 10], Hm=8, f=0.5, seed=99, flags=B.L2A_FLAG_SKIP_GLOBAL)


def test_decode_positions_outside_the_cache_are_clamped(oracle):
    """pos lives in device memory, so the host cannot reject it: the kernels clamp it into 0..T-1."""
    decode_case(oracle, Bn=3, Tcap=777, Hq=8, Hkv=2, W=64, pos=[776, 0, 776], Hm=1, f=1.0, seed=100,
                pos_given=[777, -5, 2 ** 31 - 1])


@pytest.mark.parametrize("pos", [[0, 5], [31, 32], [100, 513], [1022, 700]])
def test_decode_rows_behind_the_new_token_are_never_used(oracle, pos):
    """NaN in every cache row after pos: a zero weight would not keep it out of the sums."""
    decode_case(oracle, 2, 1024, 8, 2, 300, pos, 8, 0.6, seed=95, poison=True)


@pytest.mark.parametrize("Tring,W,pos", [(320, 300, [5, 299]), (320, 300, [319, 320]), (320, 300, [1000, 4000]),
                                          (512, 300, [511, 512]), (640, 100, [90, 5000]), (32, 31, [31, 32]),
                                          (64, 31, [63, 100]), (4128, 4096, [4127, 9000])])
def test_decode_local_ring_cache(oracle, Tring, W, pos):
    """A Local module of its own keeps a ring of Tring >= W + 1 slots, token j in slot j mod Tring; the
    result is the Local attention of the layer's definition at the token's position in the whole sequence."""
    Bn, Hq, Hkv, D, Tfull = 2, 8, 2, 128, max(pos) + 1
    k = gen.normal_tensor((Bn, Tfull, Hkv, D), 96, 1, "bf16")
    v = gen.normal_tensor((Bn, Tfull, Hkv, D), 96, 2, "bf16")
    qn = gen.normal_tensor((Bn, Hq, D), 96, 3, "bf16")
    pos = np.asarray(pos, dtype=np.int32)
    qfull = np.zeros((Bn, Tfull, Hq, D), np.float32)
    for b in range(Bn):
        qfull[b, pos[b]] = qn[b]
    pr = oracle.Problem(qfull, k, v, np.zeros((Bn, 1, Tfull), np.uint8), W)
    rows = np.array([(b, h, pos[b]) for b in range(Bn) for h in range(Hq)], dtype=np.int32)
    ref = oracle.fwd_rows(pr, rows)
    # the ring as the module would have written it: every token up to pos in its slot, later ones overwrite
    kr = torch.full((Bn, Tring, Hkv, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    vr = torch.full((Bn, Tring, Hkv, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    kd, vd = to_device(k, "bf16"), to_device(v, "bf16")
    for b in range(Bn):
        first = max(0, int(pos[b]) - Tring + 1)
        j = torch.arange(first, int(pos[b]) + 1, device="cuda")
        kr[b, j % Tring] = kd[b, j]
        vr[b, j % Tring] = vd[b, j]
    p = B.make_params(Bn, Tring, Hq, Hkv, D, W, 1, B.L2A_BF16, B.L2A_FLAG_SKIP_GLOBAL | B.L2A_FLAG_RING_CACHE)
    O = torch.full((Bn, Hq, D), 7.0, dtype=torch.bfloat16, device="cuda")
    lse_l = torch.zeros((Bn, Hq), dtype=torch.float32, device="cuda")
    B.l2a_attn_decode(p, to_device(qn, "bf16"), kr, vr, torch.from_numpy(pos).cuda(),
                      torch.zeros((Bn, 1), dtype=torch.uint8, device="cuda"), O, lse_l, None)
    torch.cuda.synchronize()
    assert_close("O", to_host(O), ref["S"].reshape(Bn, Hq, D), "bf16")
    assert_lse("lse_local", lse_l.cpu().numpy().astype(np.float64), ref["lse_l"].reshape(Bn, Hq), "bf16")


@pytest.mark.timeout(600)
def test_decode_full_length_cache(oracle):
    """Qwen2.5-7B head layout, 128K cache, a routed and an unrouted sequence; the cache rows behind
    each new token hold NaN."""
    rng = np.random.default_rng(5)
    Bn, T, Hq, Hkv, D, W = 2, 131072, 28, 4, 128, 4096
    k = gen.normal_tensor((Bn, T, Hkv, D), 5, 1, "bf16")
    v = gen.normal_tensor((Bn, T, Hkv, D), 5, 2, "bf16")
    qn = gen.normal_tensor((Bn, Hq, D), 5, 3, "bf16")
    pos = np.array([T - 1, 100000], dtype=np.int32)
    d = np.array([[1], [0]], dtype=np.uint8)
    qfull = np.zeros((Bn, T, Hq, D), np.float32)
    mfull = np.zeros((Bn, 1, T), np.uint8)
    for b in range(Bn):
        qfull[b, pos[b]] = qn[b]
        mfull[b, 0, pos[b]] = d[b, 0]
    pr = oracle.Problem(qfull, k, v, mfull, W)
    rows = np.array([(b, h, pos[b]) for b in range(Bn) for h in range(Hq)], dtype=np.int32)
    ref = oracle.fwd_rows(pr, rows)
    p = B.make_params(Bn, T, Hq, Hkv, D, W, 1)
    O = torch.empty((Bn, Hq, D), dtype=torch.bfloat16, device="cuda")
    lse_g = torch.zeros((Bn, Hq), dtype=torch.float32, device="cuda")
    kd, vd = to_device(k, "bf16"), to_device(v, "bf16")
    for b in range(Bn):
        kd[b, pos[b] + 1:] = float("nan")
        vd[b, pos[b] + 1:] = float("nan")
    B.l2a_attn_decode(p, to_device(qn, "bf16"), kd, vd, torch.from_numpy(pos).cuda(),
                      torch.from_numpy(d).cuda(), O, None, lse_g)
    torch.cuda.synchronize()
    assert_close("O", to_host(O), (ref["S"] + ref["A"]).reshape(Bn, Hq, D), "bf16")
    assert_lse("lse_global", lse_g.cpu().numpy().astype(np.float64), ref["lse_g"].reshape(Bn, Hq), "bf16")


# ------------------------------------------------------------------------------------------
# HIP graph capture of the whole step
# ------------------------------------------------------------------------------------------
def test_step_replays_from_a_hip_graph(oracle):
    """route_compact + forward + backward captured once and replayed: the library allocates nothing,
    clears scratch with fill kernels, and every kernel is deterministic, so each replay must
    reproduce the eager results bit for bit -- also after the inputs changed in place."""
    x = make_case(T=1500, Hq=14, Hkv=2, W=300, Hm=14, f=0.3, seed=110)
    lay = layer_from_numpy(x.q, x.k, x.v, x.mask, x.w.W, "bf16")
    dO = to_device(x.dO, "bf16")

    def step():
        lay.route(); lay.forward(); lay.backward(dO)

    step()                       # eager: allocates the gradient buffers and workspaces
    torch.cuda.synchronize()
    names = ("O", "S", "A", "lse_l", "lse_g", "dq", "dk", "dv")
    eager = {n: getattr(lay, n).clone() for n in names}
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                   # warm-up on the capturing stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        for n in names:
            getattr(lay, n).fill_(3.0)            # eager work between the replays
        graph.replay()
        torch.cuda.synchronize()
        for n in names:
            assert torch.equal(getattr(lay, n), eager[n]), f"replay {rep}: {n} differs from the eager result"
    # new inputs in the same buffers: the replay must follow them
    x2 = make_case(T=1500, Hq=14, Hkv=2, W=300, Hm=14, f=0.5, seed=111)
    lay.q.copy_(to_device(x2.q, "bf16")); lay.k.copy_(to_device(x2.k, "bf16")); lay.v.copy_(to_device(x2.v, "bf16"))
    lay.mask.copy_(torch.from_numpy(x2.mask).cuda()); dO.copy_(to_device(x2.dO, "bf16"))
    graph.replay()
    torch.cuda.synchronize()
    pr = oracle.Problem(x2.q, x2.k, x2.v, x2.mask, x2.w.W)
    ref = oracle.layer_fwd(pr)
    g = oracle.layer_bwd(pr, x2.dO, ref)
    assert_close("O", to_host(lay.O), ref["O"], "bf16")
    assert_close("dq", to_host(lay.dq), g["dq_l"] + g["dq_g"], "bf16")
    assert_close("dk", to_host(lay.dk), g["dk_l"] + g["dk_g"], "bf16")
    assert_close("dv", to_host(lay.dv), g["dv_l"] + g["dv_g"], "bf16")

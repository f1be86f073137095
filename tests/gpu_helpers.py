"""Helpers shared by the GPU parity tests: one whole-layer comparison against the oracle."""
import numpy as np
import torch

from paper_2603_17484_amd import binding as B
from paper_2603_17484_amd import inputs as gen
from paper_2603_17484_amd.runner import layer_from_numpy, to_device, to_host
from tests.tolerance import LSE_BF16, LSE_FP32, compare as assert_close, error_bands


def assert_lse(name, got, ref, dtype):
    fin = np.isfinite(ref)
    assert np.array_equal(np.isneginf(got), ~fin), f"{name}: -inf pattern differs"
    if fin.any():
        err = np.abs(got[fin] - ref[fin]).max()
        assert err <= (LSE_FP32 if dtype == "fp32" else LSE_BF16), f"{name}: max err {err:.3e}"


def make_case(B_=1, T=600, Hq=4, Hkv=2, D=128, W=100, dtype="bf16", Hm=1, f=0.3, seed=0, mask=None, scale=None):
    w = gen.Workload("case", B_, T, Hq, Hkv, D, W, dtype, "bernoulli", Hm, f)
    x = gen.make_inputs(w, seed, with_dO=True)
    if mask is not None:
        x.mask = np.ascontiguousarray(np.broadcast_to(mask, x.mask.shape), dtype=np.uint8)
    return x


def run_and_check(oracle, x, flags=0, backward=True, separate=False, scale=None, check_branches=True, kv_heads=None,
                  twice=False, bands=False):
    """One layer call on the GPU, every element of every output against the oracle.
    kv_heads: compare only these KV heads and their query heads (heads are independent, so the oracle
    then runs on the sub-problem made of them; the GPU still computes all heads).
    twice: run the backward a second time and require the same bits (the kernels are deterministic;
    a result read before its matrix instruction has finished would show as a difference).
    bands: print the largest gradient error per band of the row's largest reference element."""
    w = x.w
    G = w.Hq // w.Hkv
    qg = kg = vg = None
    if separate:
        qg = gen.normal_tensor(x.q.shape, x.seed, 11, w.dtype)
        kg = gen.normal_tensor(x.k.shape, x.seed, 12, w.dtype)
        vg = gen.normal_tensor(x.v.shape, x.seed, 13, w.dtype)
    dense = bool(flags & B.L2A_FLAG_DENSE)
    omask = np.ones_like(x.mask) if dense else x.mask
    ksel = list(range(w.Hkv)) if kv_heads is None else list(kv_heads)
    qsel = [hk * G + g_ for hk in ksel for g_ in range(G)]
    msel = {1: [0], w.Hkv: ksel}.get(omask.shape[1], qsel)
    sub = lambda a, sel: None if a is None else np.ascontiguousarray(a[:, :, sel])
    pr = oracle.Problem(sub(x.q, qsel), sub(x.k, ksel), sub(x.v, ksel), np.ascontiguousarray(omask[:, msel]), w.W, scale,
                        sub(qg, qsel), sub(kg, ksel), sub(vg, ksel))
    ref = oracle.layer_fwd(pr)
    hq = lambda t: to_host(t[:, :, qsel])       # [B,T,Hq,D] tensors
    hk_ = lambda t: to_host(t[:, :, ksel])      # [B,T,Hkv,D]
    hs = lambda t: to_host(t[:, qsel])          # [B,Hq,T] statistics

    lay = layer_from_numpy(x.q, x.k, x.v, x.mask, w.W, w.dtype, flags, scale, qg, kg, vg, guard=True)
    lay.route()
    lay.forward()
    torch.cuda.synchronize()
    assert lay.alloc.check() >= 5, "guard bands around the forward's outputs and workspaces"
    skip_l = bool(flags & B.L2A_FLAG_SKIP_LOCAL)
    skip_g = bool(flags & B.L2A_FLAG_SKIP_GLOBAL)
    if not dense:
        rows, cnt, first = oracle.route_compact(x.mask, w.Hq, w.Hkv)
        assert np.array_equal(lay.row_idx.cpu().numpy(), rows)
        assert np.array_equal(lay.count.cpu().numpy(), cnt)
        assert np.array_equal(lay.first.cpu().numpy(), first)
    expect_O = (0 if skip_l else ref["S"]) + (0 if skip_g else ref["A"])
    assert_close("O", hq(lay.O), expect_O, w.dtype)
    if not skip_l:
        assert_lse("lse_local", hs(lay.lse_l), ref["lse_l"], w.dtype)
        if check_branches:
            assert_close("S", hq(lay.S), ref["S"], w.dtype)
    if not skip_g:
        assert_lse("lse_global", hs(lay.lse_g), ref["lse_g"], w.dtype)
        if check_branches:
            A = hq(lay.A)
            assert_close("A", A, ref["A"], w.dtype)
            d = pr.mask_per_head().transpose(0, 2, 1)
            assert np.all(A[~d] == 0.0), "global output of unrouted tokens must be exactly zero"
    if not backward:
        return lay, ref
    dO_np = sub(x.dO, qsel)
    g = oracle.layer_bwd(pr, dO_np, ref)
    dO = to_device(x.dO, w.dtype)
    lay.backward(dO, separate=separate, want_delta=True)
    torch.cuda.synchronize()
    lay.alloc.check()
    zero = lambda k: 0 * g[k]
    loc = {k: (zero(k) if skip_l else g[k]) for k in ("dq_l", "dk_l", "dv_l")}
    glb = {k: (zero(k) if skip_g else g[k]) for k in ("dq_g", "dk_g", "dv_g")}
    if separate:
        for name, got, r in (("dq_loc", hq(lay.dq), loc["dq_l"]), ("dk_loc", hk_(lay.dk), loc["dk_l"]),
                             ("dv_loc", hk_(lay.dv), loc["dv_l"]), ("dq_glb", hq(lay.dqg), glb["dq_g"]),
                             ("dk_glb", hk_(lay.dkg), glb["dk_g"]), ("dv_glb", hk_(lay.dvg), glb["dv_g"])):
            assert_close(name, got, r, w.dtype)
    else:
        assert_close("dq", hq(lay.dq), loc["dq_l"] + glb["dq_g"], w.dtype)
        assert_close("dk", hk_(lay.dk), loc["dk_l"] + glb["dk_g"], w.dtype)
        assert_close("dv", hk_(lay.dv), loc["dv_l"] + glb["dv_g"], w.dtype)
    if bands and not separate:
        for n, got in (("dq", hq(lay.dq)), ("dk", hk_(lay.dk)), ("dv", hk_(lay.dv))):
            print(f"largest error by the row's largest |ref|, {n}:", flush=True)
            for lo, hi, nrows, mx, over in error_bands(got, loc[n[0] + n[1] + "_l"] + glb[n[0] + n[1] + "_g"]):
                print(f"  ({lo:5.2f}, {hi:5.2f}]  rows {nrows:8d}  max err {mx:.4f}  elements over 2e-2: {over}", flush=True)
    if not skip_g:
        err = np.abs(hs(lay.delta_g) - g["delta_g"]).max()
        assert err <= (1e-4 if w.dtype == "fp32" else 3e-2), f"delta_g max err {err}"
    if twice:
        names = ("dq", "dk", "dv") + (("dqg", "dkg", "dvg") if separate else ())
        first_bits = {n: getattr(lay, n).clone() for n in names}
        for n in names:
            getattr(lay, n).fill_(3.0)
        lay.backward(dO, separate=separate, want_delta=True)
        torch.cuda.synchronize()
        for n in names:
            assert torch.equal(first_bits[n], getattr(lay, n)), f"{n}: second backward differs from the first"
    return lay, ref

"""Pins for the oracle's backward pass (CPU only).

The paper states only that gradients are taken for the active queries with the saved
log-sum-exp (Sec. 3.2), so the oracle's hand-written formulas are pinned against things
that do not share them: PyTorch fp64 autograd of a naive dense expression of the layer
(Sec. 3.1 Eqs. 4-5 on top of Sec. 2 Eq. Attn), central finite differences of that layer's
own forward, and identities that follow from rows of P summing to one.
"""
import numpy as np
import pytest
import torch


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape).astype(np.float32)


def _make(oracle, B=1, T=24, Hq=4, Hkv=2, D=8, W=4, Hm=1, f=0.4, seed=0, separate=False, scale=None):
    q, k, v = _rand((B, T, Hq, D), seed), _rand((B, T, Hkv, D), seed + 1), _rand((B, T, Hkv, D), seed + 2)
    dO = _rand((B, T, Hq, D), seed + 4)
    mask = (np.random.default_rng(seed + 3).random((B, Hm, T)) < f).astype(np.uint8)
    if separate:
        qg, kg, vg = _rand((B, T, Hq, D), seed + 5), _rand((B, T, Hkv, D), seed + 6), _rand((B, T, Hkv, D), seed + 7)
        return oracle.Problem(q, k, v, mask, W, scale, qg, kg, vg), dO
    return oracle.Problem(q, k, v, mask, W, scale), dO


def torch_layer(ql, kl, vl, qg, kg, vg, d, W, scale, G):
    """Naive dense layer in torch fp64: o = s + d * a.  Tensors [B,T,H,D]; d [B,Hq,T] bool."""
    T = ql.shape[1]
    i = torch.arange(T)[:, None]
    j = torch.arange(T)[None, :]
    neg = torch.tensor(float("-inf"), dtype=torch.float64)

    def branch(q, k, v, allowed):
        kk = k.repeat_interleave(G, dim=2)
        vv = v.repeat_interleave(G, dim=2)
        z = torch.einsum("bihd,bjhd->bhij", q, kk) * scale
        z = torch.where(allowed, z, neg)
        return torch.einsum("bhij,bjhd->bihd", torch.softmax(z, dim=-1), vv)

    s = branch(ql, kl, vl, (i - j >= 0) & (i - j <= W))
    a = branch(qg, kg, vg, j <= i)
    return s + a * d.permute(0, 2, 1)[..., None].to(torch.float64)


def autograd_reference(pr, dO):
    t = lambda x: torch.from_numpy(np.asarray(x)).double().requires_grad_(True)
    ql, kl, vl, qg, kg, vg = (t(x) for x in (pr.q, pr.k, pr.v, pr.qg, pr.kg, pr.vg))
    d = torch.from_numpy(pr.mask_per_head().copy())
    o = torch_layer(ql, kl, vl, qg, kg, vg, d, pr.W, pr.scale, pr.G)
    (o * torch.from_numpy(dO).double()).sum().backward()
    return [x.grad.numpy() for x in (ql, kl, vl, qg, kg, vg)], o.detach().numpy()


@pytest.mark.parametrize("Hm", ["shared", "kv", "q"])
@pytest.mark.parametrize("W", [0, 3, 100])
def test_backward_matches_autograd_separate_branches(oracle, Hm, W):
    Hq, Hkv = 6, 2
    hm = {"shared": 1, "kv": Hkv, "q": Hq}[Hm]
    pr, dO = _make(oracle, B=2, T=29, Hq=Hq, Hkv=Hkv, D=8, W=W, Hm=hm, seed=31 + W, separate=True, scale=0.41)
    got = oracle.layer_bwd(pr, dO)
    (dql, dkl, dvl, dqg, dkg, dvg), o = autograd_reference(pr, dO)
    np.testing.assert_allclose(oracle.layer_fwd(pr)["O"], o, atol=1e-12)
    for name, ref in (("dq_l", dql), ("dk_l", dkl), ("dv_l", dvl), ("dq_g", dqg), ("dk_g", dkg), ("dv_g", dvg)):
        np.testing.assert_allclose(got[name], ref, rtol=1e-10, atol=1e-11, err_msg=name)


def test_backward_shared_inputs_sum_branches(oracle):
    """L2A-shared (Sec. 5): one Q/K/V feeds both branches, so their gradients add."""
    pr, dO = _make(oracle, B=1, T=200, Hq=4, Hkv=2, D=16, W=17, Hm=4, f=0.3, seed=7)
    got = oracle.layer_bwd(pr, dO)
    (dql, dkl, dvl, dqg, dkg, dvg), _ = autograd_reference(pr, dO)
    # autograd sees aliased leaves as separate tensors here, so add them by hand
    np.testing.assert_allclose(got["dq"], dql + dqg, rtol=1e-10, atol=1e-11)
    np.testing.assert_allclose(got["dk"], dkl + dkg, rtol=1e-10, atol=1e-11)
    np.testing.assert_allclose(got["dv"], dvl + dvg, rtol=1e-10, atol=1e-11)


def test_backward_finite_differences(oracle):
    """Central differences of the oracle's own forward, L = sum(O * dO), fp64 on a tiny case."""
    pr, dO = _make(oracle, B=1, T=10, Hq=2, Hkv=1, D=4, W=3, Hm=2, f=0.5, seed=13)
    got = oracle.layer_bwd(pr, dO)
    eps = 1e-3   # inputs are fp32 storage: steps must be exactly representable-ish; fp64 math inside

    def loss(q, k, v):
        return float((oracle.layer_fwd(oracle.Problem(q, k, v, pr.mask, pr.W))["O"] * dO).sum())

    rng = np.random.default_rng(0)
    for name, idx_of in (("dq", 0), ("dk", 1), ("dv", 2)):
        base = [pr.q.copy(), pr.k.copy(), pr.v.copy()]
        for _ in range(12):
            idx = tuple(rng.integers(0, s) for s in base[idx_of].shape)
            x0 = base[idx_of][idx]
            hi = np.float32(x0 + eps)
            lo = np.float32(x0 - eps)
            args_hi = [a.copy() for a in base]; args_hi[idx_of][idx] = hi
            args_lo = [a.copy() for a in base]; args_lo[idx_of][idx] = lo
            fd = (loss(*args_hi) - loss(*args_lo)) / (float(hi) - float(lo))
            assert abs(fd - got[name][idx]) < 2e-5 * max(1.0, abs(fd)), (name, idx, fd, got[name][idx])


def test_backward_identities(oracle):
    pr, dO = _make(oracle, B=1, T=150, Hq=6, Hkv=2, D=8, W=11, Hm=6, f=0.25, seed=17)
    got = oracle.layer_bwd(pr, dO)
    d = pr.mask_per_head().astype(np.float64)                                  # [B,Hq,T]
    g64 = dO.astype(np.float64)
    # rows of P sum to 1: sum_j dV_j = sum over the group's heads and tokens of the upstream gradient
    grp = lambda x: x.reshape(pr.B, pr.T, pr.Hkv, pr.G, pr.D).sum(axis=3)
    np.testing.assert_allclose(got["dv_l"].sum(axis=1), grp(g64).sum(axis=1), atol=1e-10)
    gd = g64 * d.transpose(0, 2, 1)[..., None]
    np.testing.assert_allclose(got["dv_g"].sum(axis=1), grp(gd).sum(axis=1), atol=1e-10)
    # rows of dS sum to 0, and dK_j = scale * sum_t dS_tj q_t: with all queries equal, sum_j dK_j = 0
    same_q = np.broadcast_to(pr.q[:, :1, :1], pr.q.shape).copy()
    g2 = oracle.layer_bwd(oracle.Problem(same_q, pr.k, pr.v, pr.mask, pr.W), dO)
    np.testing.assert_allclose(g2["dk_l"].sum(axis=1), 0.0, atol=1e-10)
    np.testing.assert_allclose(g2["dk_g"].sum(axis=1), 0.0, atol=1e-10)
    # all keys equal: scores do not depend on j, so dQ = scale * sum_j dS_tj k = 0
    same_k = np.broadcast_to(pr.k[:, :1], pr.k.shape).copy()
    g3 = oracle.layer_bwd(oracle.Problem(pr.q, same_k, pr.v, pr.mask, pr.W), dO)
    np.testing.assert_allclose(g3["dq"], 0.0, atol=1e-10)
    # unrouted rows receive no global-branch query gradient
    assert np.all(got["dq_g"][d.transpose(0, 2, 1) == 0] == 0.0)
    # all d = 0: only the local branch contributes
    none = oracle.layer_bwd(oracle.Problem(pr.q, pr.k, pr.v, np.zeros_like(pr.mask), pr.W), dO)
    for k in ("dq_g", "dk_g", "dv_g"):
        assert np.all(none[k] == 0.0)
    np.testing.assert_array_equal(none["dq"], got["dq_l"])


def test_backward_row_and_key_subsets(oracle):
    pr, dO = _make(oracle, B=2, T=40, Hq=4, Hkv=2, D=8, W=6, Hm=1, seed=23)
    fwd = oracle.layer_fwd(pr)
    full = oracle.layer_bwd(pr, dO, fwd)
    rows = np.array([[0, 1, 0], [1, 3, 39], [0, 0, 20]], np.int32)
    dql, dqg = oracle.bwd_dq_rows(pr, dO, rows)
    for i, (b, h, t) in enumerate(rows):
        np.testing.assert_array_equal(dql[i], full["dq_l"][b, t, h])
        np.testing.assert_array_equal(dqg[i], full["dq_g"][b, t, h])
    keys = np.array([[0, 0, 0], [1, 1, 39], [1, 0, 17]], np.int32)
    dkl, dvl, dkg, dvg = oracle.bwd_dkdv_keys(pr, dO, keys, fwd["lse_l"], full["delta_l"], fwd["lse_g"], full["delta_g"])
    for i, (b, hk, j) in enumerate(keys):
        np.testing.assert_array_equal(dkl[i], full["dk_l"][b, j, hk])
        np.testing.assert_array_equal(dvg[i], full["dv_g"][b, j, hk])

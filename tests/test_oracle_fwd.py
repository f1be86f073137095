"""Pins for the oracle's forward pass and compaction (CPU only).

Each check is independent of the oracle's own code: an explicit masked-matrix softmax in
numpy, PyTorch's CPU scaled_dot_product_attention in fp64, closed forms and the layer's
invariants (Sec. 2 Eq. Attn and the sliding-window mask; Sec. 3.1 Eqs. 4-5).
"""
import numpy as np
import pytest
import torch

from paper_2603_17484_amd import inputs as gen


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape).astype(np.float32)


def _problem(oracle, B=2, T=40, Hq=4, Hkv=2, D=8, W=5, Hm=1, f=0.4, seed=0, scale=None):
    q, k, v = _rand((B, T, Hq, D), seed), _rand((B, T, Hkv, D), seed + 1), _rand((B, T, Hkv, D), seed + 2)
    mask = (np.random.default_rng(seed + 3).random((B, Hm, T)) < f).astype(np.uint8)
    return oracle.Problem(q, k, v, mask, W, scale)


def matrix_reference(pr):
    """Whole [T,T] score matrices with additive 0/-inf masks, per (b, h): Eq. (Attn) as printed."""
    B, T, Hq, D, G = pr.B, pr.T, pr.Hq, pr.D, pr.G
    i = np.arange(T)[:, None]
    j = np.arange(T)[None, :]
    M_glb = np.where(j <= i, 0.0, -np.inf)
    M_loc = np.where((i - j >= 0) & (i - j <= pr.W), 0.0, -np.inf)
    d = pr.mask_per_head()
    out = {k: np.zeros((B, T, Hq, D)) for k in ("S", "A", "O")}
    out["lse_l"] = np.zeros((B, Hq, T))
    out["lse_g"] = np.full((B, Hq, T), -np.inf)
    for b in range(B):
        for h in range(Hq):
            K = pr.k[b, :, h // G].astype(np.float64)
            V = pr.v[b, :, h // G].astype(np.float64)
            Z = pr.q[b, :, h].astype(np.float64) @ K.T * pr.scale
            for name, M in (("S", M_loc), ("A", M_glb)):
                Zm = Z + M
                mx = Zm.max(axis=1, keepdims=True)
                E = np.exp(Zm - mx)
                P = E / E.sum(axis=1, keepdims=True)
                lse = (mx + np.log(E.sum(axis=1, keepdims=True)))[:, 0]
                if name == "S":
                    out["S"][b, :, h] = P @ V
                    out["lse_l"][b, h] = lse
                else:
                    dd = d[b, h].astype(np.float64)[:, None]
                    out["A"][b, :, h] = dd * (P @ V)
                    out["lse_g"][b, h] = np.where(d[b, h], lse, -np.inf)
            out["O"][b, :, h] = out["S"][b, :, h] + out["A"][b, :, h]
    return out


@pytest.mark.parametrize("Hm", ["shared", "kv", "q"])
@pytest.mark.parametrize("W", [0, 1, 5, 39, 1000])
def test_forward_matches_masked_matrix_softmax(oracle, Hm, W):
    Hq, Hkv = 6, 2
    hm = {"shared": 1, "kv": Hkv, "q": Hq}[Hm]
    pr = _problem(oracle, Hq=Hq, Hkv=Hkv, W=W, Hm=hm, seed=11 + W)
    got, ref = oracle.layer_fwd(pr), matrix_reference(pr)
    for k in ("S", "A", "O", "lse_l"):
        np.testing.assert_allclose(got[k], ref[k], rtol=1e-12, atol=1e-12, err_msg=k)
    fin = np.isfinite(ref["lse_g"])
    assert np.array_equal(np.isfinite(got["lse_g"]), fin)
    np.testing.assert_allclose(got["lse_g"][fin], ref["lse_g"][fin], rtol=1e-12, atol=1e-12)
    assert np.all(got["lse_g"][~fin] == -np.inf)


def test_dense_global_is_library_causal_attention(oracle):
    """All d = 1: the global branch is FA-2's full causal attention (Sec. 1; Sec. 3.1 zero-init router)."""
    pr = _problem(oracle, T=33, Hq=4, Hkv=2, D=16, W=3, f=2.0, seed=5)
    got = oracle.layer_fwd(pr)
    q = torch.from_numpy(pr.q).double().permute(0, 2, 1, 3)
    k = torch.from_numpy(pr.k).double().permute(0, 2, 1, 3).repeat_interleave(pr.G, dim=1)
    v = torch.from_numpy(pr.v).double().permute(0, 2, 1, 3).repeat_interleave(pr.G, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True).permute(0, 2, 1, 3).numpy()
    np.testing.assert_allclose(got["A"], ref, rtol=1e-11, atol=1e-12)
    # local branch = the same routine with an explicit band mask (token itself + W before it)
    i = torch.arange(pr.T)[:, None]
    j = torch.arange(pr.T)[None, :]
    band = (i - j >= 0) & (i - j <= pr.W)
    ref_l = torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=band).permute(0, 2, 1, 3).numpy()
    np.testing.assert_allclose(got["S"], ref_l, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(got["O"], ref + ref_l, rtol=1e-11, atol=1e-12)


def test_custom_scale_and_separate_global_inputs(oracle):
    """Local and Global modules may have their own projections (Sec. 3.1)."""
    B, T, Hq, Hkv, D, W = 1, 21, 2, 1, 4, 2
    pr0 = _problem(oracle, B=B, T=T, Hq=Hq, Hkv=Hkv, D=D, W=W, f=0.5, seed=3, scale=0.37)
    qg, kg, vg = _rand((B, T, Hq, D), 90), _rand((B, T, Hkv, D), 91), _rand((B, T, Hkv, D), 92)
    pr = oracle.Problem(pr0.q, pr0.k, pr0.v, pr0.mask, W, 0.37, qg, kg, vg)
    got = oracle.layer_fwd(pr)
    loc = matrix_reference(pr0)
    glb = matrix_reference(oracle.Problem(qg, kg, vg, pr0.mask, W, 0.37))
    np.testing.assert_allclose(got["S"], loc["S"], atol=1e-12)
    np.testing.assert_allclose(got["A"], glb["A"], atol=1e-12)
    np.testing.assert_allclose(got["O"], loc["S"] + glb["A"], atol=1e-12)
    # a different scale must change the result (guards against a dropped scale)
    other = oracle.layer_fwd(oracle.Problem(pr0.q, pr0.k, pr0.v, pr0.mask, W, 0.5))
    assert np.abs(other["S"] - loc["S"]).max() > 1e-3


def test_closed_forms_uniform_weights(oracle):
    """K = 0 makes every softmax uniform: outputs are running / windowed means of V."""
    B, T, Hq, Hkv, D, W = 1, 50, 2, 1, 6, 7
    q, v = _rand((B, T, Hq, D), 1), _rand((B, T, Hkv, D), 2)
    k = np.zeros((B, T, Hkv, D), np.float32)
    mask = np.ones((B, 1, T), np.uint8)
    got = oracle.layer_fwd(oracle.Problem(q, k, v, mask, W))
    V = v[0, :, 0].astype(np.float64)
    t = np.arange(T)
    run_mean = np.cumsum(V, axis=0) / (t + 1)[:, None]
    win_mean = np.stack([V[max(0, i - W): i + 1].mean(axis=0) for i in range(T)])
    for h in range(Hq):
        np.testing.assert_allclose(got["A"][0, :, h], run_mean, atol=1e-12)
        np.testing.assert_allclose(got["S"][0, :, h], win_mean, atol=1e-12)
        np.testing.assert_allclose(got["lse_g"][0, h], np.log(t + 1), atol=1e-12)
        # the window holds the token itself and the W tokens before it: W + 1 keys
        np.testing.assert_allclose(got["lse_l"][0, h], np.log(np.minimum(t + 1, W + 1)), atol=1e-12)


def test_closed_forms_special_cases(oracle):
    B, T, Hq, Hkv, D = 1, 17, 2, 2, 5
    q, k, v = _rand((B, T, Hq, D), 4), _rand((B, T, Hkv, D), 5), _rand((B, T, Hkv, D), 6)
    ones = np.ones((B, 1, T), np.uint8)
    # W = 0: only the token itself (the SWA-0 ablation, Sec. 5): s_t = v_t, lse = scale <q_t,k_t>
    g = oracle.layer_fwd(oracle.Problem(q, k, v, ones, 0))
    np.testing.assert_allclose(g["S"], v.astype(np.float64), atol=1e-12)
    z = np.einsum("bthd,bthd->bht", q.astype(np.float64), k.astype(np.float64)) / np.sqrt(D)
    np.testing.assert_allclose(g["lse_l"], z, atol=1e-12)
    # t = 0: one key for both branches
    np.testing.assert_allclose(g["A"][:, 0], v[:, 0].astype(np.float64), atol=1e-12)
    np.testing.assert_allclose(g["lse_g"][:, :, 0], z[:, :, 0], atol=1e-12)
    # all value rows equal: any convex combination returns that row
    vc = np.broadcast_to(v[:, :1], v.shape).copy()
    g = oracle.layer_fwd(oracle.Problem(q, k, vc, ones, 3))
    np.testing.assert_allclose(g["S"], np.broadcast_to(vc[:, :1].astype(np.float64), g["S"].shape), atol=1e-12)
    np.testing.assert_allclose(g["A"], g["S"], atol=1e-12)


def test_layer_invariants(oracle):
    pr = _problem(oracle, T=64, Hq=4, Hkv=2, D=8, W=9, Hm=4, f=0.3, seed=21)
    full = oracle.layer_fwd(pr)
    d = pr.mask_per_head().transpose(0, 2, 1)            # [B,T,Hq]
    # d = 0 rows: global output exactly zero, o = s, lse_g = -inf (Eq. 4, Eq. 5)
    assert np.all(full["A"][~d] == 0.0)
    assert np.array_equal(full["O"][~d], full["S"][~d])
    assert np.all(np.isneginf(full["lse_g"].transpose(0, 2, 1)[~d]))
    # routed rows do not depend on which other rows are routed
    ones = oracle.Problem(pr.q, pr.k, pr.v, np.ones_like(pr.mask), pr.W)
    dense = oracle.layer_fwd(ones)
    np.testing.assert_array_equal(full["A"][d], dense["A"][d])
    np.testing.assert_array_equal(full["S"], dense["S"])
    # all d = 0: the layer is local attention only
    none = oracle.layer_fwd(oracle.Problem(pr.q, pr.k, pr.v, np.zeros_like(pr.mask), pr.W))
    np.testing.assert_array_equal(none["O"], none["S"])
    np.testing.assert_array_equal(none["S"], full["S"])
    # W >= T-1: local = global on routed rows when both branches read the same q/k/v
    wide = oracle.layer_fwd(oracle.Problem(pr.q, pr.k, pr.v, pr.mask, pr.T - 1))
    np.testing.assert_allclose(wide["S"][d], wide["A"][d], atol=1e-13)
    np.testing.assert_allclose(wide["O"][d], 2 * wide["S"][d], atol=1e-13)
    # shifting every key by a constant vector adds <q_t, c> to all of row t's scores: no change
    c = _rand((pr.D,), 77)
    sh = oracle.layer_fwd(oracle.Problem(pr.q, pr.k + c, pr.v, pr.mask, pr.W))
    np.testing.assert_allclose(sh["O"], full["O"], atol=1e-6)
    # grouped-query heads: head h equals a single-head problem on KV head h // G
    h = 3
    one = oracle.layer_fwd(oracle.Problem(pr.q[:, :, h:h + 1], pr.k[:, :, h // pr.G:h // pr.G + 1],
                                          pr.v[:, :, h // pr.G:h // pr.G + 1], pr.mask[:, h:h + 1], pr.W))
    np.testing.assert_array_equal(one["O"][:, :, 0], full["O"][:, :, h])


def test_fwd_rows_subset_equals_full(oracle):
    pr = _problem(oracle, T=30, seed=8)
    full = oracle.layer_fwd(pr)
    rows = np.array([[0, 0, 0], [1, 3, 29], [0, 2, 7], [1, 1, 13]], np.int32)
    sub = oracle.fwd_rows(pr, rows)
    for i, (b, h, t) in enumerate(rows):
        np.testing.assert_array_equal(sub["O"][i], full["O"][b, t, h])
        assert sub["lse_l"][i] == full["lse_l"][b, h, t]
        assert sub["lse_g"][i] == full["lse_g"][b, h, t]


# ------------------------------------------------------------------------------------
# compaction
# ------------------------------------------------------------------------------------
def brute_compact(mask, Hq, Hkv):
    B, Hm, T = mask.shape
    G = Hq // Hkv
    nkb = (T + 63) // 64
    rows = -np.ones((B, Hkv, T * G), np.int32)
    cnt = np.zeros((B, Hkv), np.int32)
    first = np.zeros((B, Hkv, nkb + 1), np.int32)
    for b in range(B):
        for hk in range(Hkv):
            lst = []
            for pos in range(T):
                for g in range(G):
                    h = hk * G + g
                    mh = 0 if Hm == 1 else (h if Hm == Hq else hk)
                    if mask[b, mh, pos]:
                        lst.append(pos * G + g)
            rows[b, hk, :len(lst)] = lst
            cnt[b, hk] = len(lst)
            pos_of = np.array(lst, np.int64) // G
            for kb in range(nkb + 1):
                first[b, hk, kb] = int(np.sum(pos_of < 64 * kb))
    return rows, cnt, first


@pytest.mark.parametrize("T", [1, 63, 64, 65, 200])
@pytest.mark.parametrize("Hm", ["shared", "kv", "q"])
def test_compaction_brute_force(oracle, T, Hm):
    Hq, Hkv = 6, 2
    hm = {"shared": 1, "kv": Hkv, "q": Hq}[Hm]
    for f, seed in ((0.0, 1), (1.0, 2), (0.3, 3)):
        mask = (np.random.default_rng(seed + T).random((2, hm, T)) < f).astype(np.uint8) * 7   # any non-zero byte
        got = oracle.route_compact(mask, Hq, Hkv)
        ref = brute_compact(mask, Hq, Hkv)
        for a, b in zip(got, ref):
            np.testing.assert_array_equal(a, b)
        rows, cnt, first = got
        assert np.all(first[:, :, -1] == cnt) and np.all(np.diff(first, axis=-1) >= 0)
        # every routed (token, query head) pair appears exactly once
        assert np.array_equal(cnt.sum(axis=1), (mask != 0).sum(axis=(1, 2)) * (Hq // hm))


def test_compaction_single_bit(oracle):
    mask = np.zeros((1, 1, 130), np.uint8)
    mask[0, 0, 64] = 1
    rows, cnt, first = oracle.route_compact(mask, 3, 1)
    assert cnt[0, 0] == 3 and list(rows[0, 0, :4]) == [192, 193, 194, -1]
    assert list(first[0, 0]) == [0, 0, 3, 3]


# ------------------------------------------------------------------------------------
# input generators (no method arithmetic, but both sides depend on them)
# ------------------------------------------------------------------------------------
def test_bf16_rounding_is_exact_and_nearest_even():
    x = np.array([1.0, 1.00390625, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, -2.5, 3.14159], np.float32)
    r = gen.round_to_bf16(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(r, ref)
    big = np.random.default_rng(0).standard_normal(10000).astype(np.float32)
    np.testing.assert_array_equal(gen.round_to_bf16(big), torch.from_numpy(big).bfloat16().float().numpy())


def test_masks_have_requested_statistics():
    m = gen.mask_bernoulli(1, 4, 20000, 0.2, seed=0, force_first=True)
    assert m[:, :, 0].all() and abs(m.mean() - 0.2) < 0.02
    mk = gen.mask_markov(1, 2, 200000, 0.2, 32, seed=1)
    assert abs(mk.mean() - 0.2) < 0.03
    x = mk[0, 0].astype(np.int8)
    starts = np.flatnonzero(np.diff(x) == 1).size
    mean_burst = x.sum() / max(starts, 1)
    assert 24 < mean_burst < 40
    per = gen.mask_markov(1, 8, 100000, (0.05, 0.3), 32, seed=2).mean(axis=2)[0]
    assert per.min() > 0.02 and per.max() < 0.36 and per.std() > 0.01
    # reproducible
    np.testing.assert_array_equal(mk, gen.mask_markov(1, 2, 200000, 0.2, 32, seed=1))
    a = gen.make_inputs(gen.workload("tiny_fp32", T=64), seed=3)
    b = gen.make_inputs(gen.workload("tiny_fp32", T=64), seed=3)
    np.testing.assert_array_equal(a.q, b.q)
    assert a.mask[0, 0, 0] == 1 and a.dO is not None


# ------------------------------------------------------------------------------------------
# router (Sec. 3.1 Eq. 3)
# ------------------------------------------------------------------------------------------
def test_router_zero_weights_route_every_token(oracle):
    """A zero-initialised router scores 0.5 everywhere, so with tau = 0.5 every token takes Global
    attention (the initial state of a converted model, Sec. 3.1)."""
    x = np.random.default_rng(0).standard_normal((2, 37, 24)).astype(np.float32)
    logit, dhat, d = oracle.router(x, np.zeros(24))
    assert np.all(logit == 0.0) and np.all(dhat == 0.5) and d.all() and d.shape == (2, 1, 37)


def test_router_against_scipy_and_threshold_monotone(oracle):
    from scipy.special import expit, logit as sp_logit
    rng = np.random.default_rng(1)
    x = rng.standard_normal((1, 500, 64)).astype(np.float32)
    w = rng.standard_normal(64) * 0.3
    lg, dhat, d = oracle.router(x, w, bias=0.25, tau=0.5)
    ref = x.astype(np.float64) @ w + 0.25
    assert np.allclose(lg, ref, rtol=0, atol=1e-12)
    assert np.allclose(dhat, expit(ref), rtol=0, atol=1e-15)
    assert np.array_equal(d[:, 0], (ref >= 0).astype(np.uint8))
    prev = None
    for tau in (0.1, 0.3, 0.5, 0.7, 0.9):       # a higher threshold routes a subset
        _, _, dt = oracle.router(x, w, bias=0.25, tau=tau)
        assert np.array_equal(dt[:, 0], (ref >= sp_logit(tau)).astype(np.uint8))
        if prev is not None:
            assert np.all(dt <= prev)
        prev = dt


def test_router_one_hot_weight_reads_one_channel(oracle):
    x = np.random.default_rng(2).standard_normal((3, 50, 16)).astype(np.float32)
    w = np.zeros(16); w[5] = 2.0
    lg, _, d = oracle.router(x, w)
    assert np.array_equal(lg, 2.0 * x[:, :, 5].astype(np.float64))
    assert np.array_equal(d[:, 0], (x[:, :, 5] >= 0).astype(np.uint8))

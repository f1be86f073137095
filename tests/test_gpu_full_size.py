"""GPU parity at the sizes and in the launch configurations the benchmark times.

The backward kernel for dK and dV picks its launch shape from the problem size: below 256 key
blocks of 128 keys over all (batch, KV head) it shares a key block's row tiles between several
workgroups (partial sums + a reduce kernel) and hands out key blocks one at a time; from 256 on --
every benchmark configuration -- one workgroup owns a key block, key blocks go to an XCD in chunks
of 2..32 neighbours, and the Local rows of all but a chunk's last key block are walked in a rotated
order.  The cases here are the ones that reach that path, element by element:

  * T = 8192 with the Qwen2.5-7B head layout, every element of every output, routed and dense;
  * the 32K forward configuration with one whole KV group compared at full length, and dK / dV at keys
    chosen at block, chunk and window edges (key 0 included);
  * the 64K training configuration at routed fractions 0.5, 0.1 and in dense mode, and both 128K
    training configurations: sampled rows, the last keys, a slab of several thousand rows of one KV
    group with dK / dV at keys inside it (interior keys, a chunk's first key block, block edges), and
    the two sum identities over all keys.

The oracle computes single rows and single keys from the definition; for dK / dV of a key it needs the
log-sum-exp and delta of every row that can see the key, which is why keys are taken inside a slab
of rows that reaches the end of the sequence.
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
# whole tensors on the unsplit dK/dV path (one workgroup per key block, chunks of two key blocks,
# rotated Local walk) and the sequential forward
# ------------------------------------------------------------------------------------------
@pytest.mark.timeout(900)
def test_bf16_qwen_layout_8k_whole_tensors(oracle):
    """B=1, T=8192, Hq=28, Hkv=4, D=128, W=1024, per-head Bernoulli(0.2): 64 key blocks x 4 KV heads = 256
    workgroups, so dK/dV takes the path of the long configurations; the backward is run twice."""
    x = make_case(T=8192, Hq=28, Hkv=4, W=1024, Hm=28, f=0.2, seed=61)
    run_and_check(oracle, x, twice=True, bands=True)


@pytest.mark.timeout(900)
def test_bf16_qwen_layout_8k_dense_mode_whole_tensors(oracle):
    """The same shape in the dense all-routed mode (identity row sets): every element of the first and the
    last KV group (14 of 28 query heads, all keys of 2 of 4 KV heads)."""
    x = make_case(T=8192, Hq=28, Hkv=4, W=1024, Hm=28, f=0.2, seed=62)
    run_and_check(oracle, x, flags=B.L2A_FLAG_DENSE, kv_heads=(0, 3), bands=True)


@pytest.mark.timeout(600)
def test_bf16_batch_of_two_on_the_unsplit_path(oracle):
    """Batch > 1 where one workgroup owns a key block: B=2, T=4096, Hq=28, Hkv=4 gives 32 key blocks x 8
    (batch, KV head) pairs = 256 workgroups (chunks of one key block), different masks per sequence; every
    element of two of the four KV groups, in both sequences."""
    x = make_case(B_=2, T=4096, Hq=28, Hkv=4, W=512, Hm=28, f=0.25, seed=63)
    run_and_check(oracle, x, kv_heads=(1, 2))


@pytest.mark.parametrize("path", ["matrix cores", "scalar"])
def test_bf16_qwen_layout_3k_whole_tensors(oracle, path):
    """The same head layout at a length that takes the split dK/dV kernel and the one-launch forward; and the
    scalar-FMA kernels (fp32 arithmetic on the same bf16 storage) on the same inputs.  Both print their largest
    gradient error per band of the row's largest reference element -- the figures behind the tolerance."""
    flags = B.L2A_FLAG_SCALAR if path == "scalar" else 0
    run_and_check(oracle, make_case(T=3000, Hq=28, Hkv=4, W=700, Hm=28, f=0.2, seed=60), flags=flags, bands=True)


# ------------------------------------------------------------------------------------------
# full-size configurations
# ------------------------------------------------------------------------------------------
def _pick(t_, rows):
    return np.stack([to_host(t_[r[0], r[2], r[1]]) for r in rows])


def full_size_checks(oracle, w, seed=0, dense=False, n_rand=40, slab_rows=8192, slab_kv_head=1, extra_keys=(),
                     whole_group=False):
    """Runs route + forward (+ backward) of workload w on the GPU and compares
      (1) sampled rows: S, A, O, both log-sum-exps, dQ;
      (2) dK, dV at every third of the last 40 keys of every KV head;
      (3) a slab -- all G heads of KV head `slab_kv_head`, every position from T - slab_rows on (the whole
          sequence with whole_group): S, A, O, log-sum-exps of every row of it, and dK, dV at keys inside it;
      (4) sum_j dV_j and sum_j dK_j over all keys (identities that hold at any size)."""
    x = gen.make_inputs(w, seed=seed, with_dO=True)
    T, G, Hq, Hkv = w.T, w.Hq // w.Hkv, w.Hq, w.Hkv
    flags = B.L2A_FLAG_DENSE if dense else 0
    lay = layer_from_numpy(x.q, x.k, x.v, x.mask, w.W, w.dtype, flags)
    dO = to_device(x.dO, w.dtype)
    lay.route(); lay.forward(); lay.backward(dO, want_delta=True)
    torch.cuda.synchronize()
    print(f"{w.name} dense={dense}: GPU pass done", flush=True)
    omask = np.ones_like(x.mask) if dense else x.mask
    pr = oracle.Problem(x.q, x.k, x.v, omask, w.W)
    d = pr.mask_per_head().transpose(0, 2, 1)  # [B,T,Hq] bool

    # ---- (1) sampled rows, routed and unrouted, early and late, tile and window edges
    rng = np.random.default_rng(1 + seed)
    ts = np.concatenate([[0, 1, 63, 64, min(w.W, T - 1), min(w.W + 1, T - 1), T - 1], rng.integers(0, T, n_rand)])
    rows = np.array([(0, int(rng.integers(0, Hq)), int(t)) for t in ts], dtype=np.int32)
    fr = oracle.fwd_rows(pr, rows)
    assert_close("S", _pick(lay.S, rows), fr["S"], "bf16")
    assert_close("A", _pick(lay.A, rows), fr["A"], "bf16")
    assert_close("O", _pick(lay.O, rows), fr["S"] + fr["A"], "bf16")
    assert_lse("lse_local", np.array([float(lay.lse_l[0, r[1], r[2]]) for r in rows]), fr["lse_l"], "bf16")
    assert_lse("lse_global", np.array([float(lay.lse_g[0, r[1], r[2]]) for r in rows]), fr["lse_g"], "bf16")
    if not dense:
        assert any(d[0, r[2], r[1]] for r in rows) and not all(d[0, r[2], r[1]] for r in rows)
    dq_l, dq_g = oracle.bwd_dq_rows(pr, x.dO, rows)
    assert_close("dq", _pick(lay.dq, rows), dq_l + dq_g, "bf16")
    print("sampled rows checked", flush=True)

    def stats_of(rows_, f_):
        st = {k: np.zeros((1, Hq, T)) for k in ("lse_l", "lse_g", "delta_l", "delta_g")}
        g_ = x.dO[0, rows_[:, 2], rows_[:, 1]].astype(np.float64)
        st["lse_l"][0, rows_[:, 1], rows_[:, 2]] = f_["lse_l"]
        st["lse_g"][0, rows_[:, 1], rows_[:, 2]] = f_["lse_g"]
        st["delta_l"][0, rows_[:, 1], rows_[:, 2]] = np.einsum("nd,nd->n", g_, f_["S"])
        st["delta_g"][0, rows_[:, 1], rows_[:, 2]] = np.einsum("nd,nd->n", g_, f_["A"])
        return st

    def check_keys(keys, st, tag):
        dk_l, dv_l, dk_g, dv_g = oracle.bwd_dkdv_keys(pr, x.dO, keys, st["lse_l"], st["delta_l"], st["lse_g"],
                                                       st["delta_g"])
        assert_close(f"dk ({tag})", np.stack([to_host(lay.dk[0, k_[2], k_[1]]) for k_ in keys]), dk_l + dk_g, "bf16")
        assert_close(f"dv ({tag})", np.stack([to_host(lay.dv[0, k_[2], k_[1]]) for k_ in keys]), dv_l + dv_g, "bf16")

    # ---- (2) the last keys: only the last rows can see them
    nlast = 40
    tail = np.array([(0, h, t) for h in range(Hq) for t in range(T - nlast, T)], dtype=np.int32)
    keys = np.array([(0, hk, j) for hk in range(Hkv) for j in range(T - nlast, T, 3)], dtype=np.int32)
    check_keys(keys, stats_of(tail, oracle.fwd_rows(pr, tail)), "last keys")
    print("last keys checked", flush=True)

    # ---- (3) a slab of rows of one KV group, and keys inside it
    t0 = 0 if whole_group else T - slab_rows
    hk = slab_kv_head
    slab = np.array([(0, hk * G + g_, t) for t in range(t0, T) for g_ in range(G)], dtype=np.int32)
    fs = oracle.fwd_rows(pr, slab)
    print(f"slab of {len(slab)} rows: oracle forward done", flush=True)
    shp = (T - t0, G, w.D)
    sl = lambda t_: to_host(t_[0, t0:, hk * G:(hk + 1) * G])
    assert_close("S (slab)", sl(lay.S), fs["S"].reshape(shp), "bf16")
    assert_close("A (slab)", sl(lay.A), fs["A"].reshape(shp), "bf16")
    assert_close("O (slab)", sl(lay.O), (fs["S"] + fs["A"]).reshape(shp), "bf16")
    st_l = lambda t_: to_host(t_[0, hk * G:(hk + 1) * G, t0:]).T     # [t, g]
    assert_lse("lse_local (slab)", st_l(lay.lse_l), fs["lse_l"].reshape(T - t0, G), "bf16")
    assert_lse("lse_global (slab)", st_l(lay.lse_g), fs["lse_g"].reshape(T - t0, G), "bf16")
    # keys: the slab's first key (with the default slab of 8192 rows the first key block of a chunk in the
    # 128K configurations), both sides of key-block (128) and half-block (64) edges, a stretch of interior
    # keys, the keys whose window ends at the last token, and whatever the caller adds
    js = {t0, t0 + 1, t0 + 63, t0 + 64, t0 + 127, t0 + 128, t0 + 129, T - w.W - 2, T - w.W - 1, T - w.W, T - 129, T - 128,
          T - 1}
    mid = t0 + (T - t0) // 4
    js |= set(range(mid, mid + 10)) | set(int(j) for j in extra_keys)
    js = sorted(j for j in js if t0 <= j < T)
    keys = np.array([(0, hk, j) for j in js], dtype=np.int32)
    check_keys(keys, stats_of(slab, fs), f"{len(js)} keys inside the slab")
    print("slab keys checked:", js[:8], "...", flush=True)

    # ---- (4) properties that hold at any size.  Every row's probabilities sum to one, so
    #   sum_j dV_j = sum over rows of that KV head of g_t  (g = dO, plus d dO for the Global branch)
    #   sum_j dK_j = 0
    # up to the bf16 rounding of the T stored values (independent, half an ulp each at most).
    dv = to_host(lay.dv)[0]   # [T,Hkv,D]
    dk = to_host(lay.dk)[0]
    weight = 1.0 + d[0].astype(np.float64)                               # [T,Hq]
    gsum = np.einsum("thd,th->hd", x.dO[0].astype(np.float64), weight)   # [Hq,D]
    gsum = gsum.reshape(Hkv, G, w.D).sum(1)
    slack = lambda a: 2e-2 * np.sqrt(T) + 2.0 ** -8 * np.sqrt((a * a).sum(0)) * 4
    assert np.all(np.abs(dv.sum(0) - gsum) <= slack(dv)), np.abs(dv.sum(0) - gsum).max()
    assert np.all(np.abs(dk.sum(0)) <= slack(dk)), np.abs(dk.sum(0)).max()
    if not dense:   # unrouted rows: zero Global output
        unr = np.argwhere(~d[0])[:: max(1, (~d[0]).sum() // 500)]
        assert all(float(lay.A[0, t_, h_].abs().max()) == 0.0 for t_, h_ in unr[:200])
    return lay


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name", ["train_128k", "qwen3_8b_128k"])
def test_full_size_128k_training_workloads(oracle, name):
    """The benchmark's workload (train_128k) and the Hq=32 / Hkv=8 bursty per-head one, at T = 131072:
    1024 key blocks per KV head, chunks of 32 key blocks (4096 keys) per XCD; the slab starts at key
    T - 8192 = 30 x 4096, the first key of a chunk."""
    w = gen.workload(name)
    full_size_checks(oracle, w, extra_keys=[w.T - 4097, w.T - 4096, w.T - 4095])


def _chunk_edges_64k(T):
    """At 64K a chunk is 16 key blocks = 2048 keys: the last two chunk boundaries, both sides."""
    return [T - 4097, T - 4096, T - 4095, T - 2049, T - 2048]


@pytest.mark.timeout(900)
@pytest.mark.parametrize("f", [0.5, 0.1])
def test_full_size_64k_training_sweep(oracle, f):
    """The 64K training configuration's sparse points (per-head Bernoulli masks): chunks of 16 key blocks."""
    w = gen.workload("train_64k", routed_fraction=f)
    full_size_checks(oracle, w, slab_rows=4608 if f > 0.3 else 6144, extra_keys=_chunk_edges_64k(w.T))


@pytest.mark.timeout(900)
def test_full_size_64k_dense_mode(oracle):
    """f = 1.0 of the same sweep: the dense all-routed mode of the kernels (identity row sets), which is the
    denominator of the sparse-versus-dense ratio."""
    w = gen.workload("train_64k")
    full_size_checks(oracle, w, dense=True, slab_rows=4608, n_rand=24, extra_keys=_chunk_edges_64k(w.T))


@pytest.mark.timeout(900)
def test_full_size_32k_shared_mask_one_whole_kv_group(oracle):
    """The 32K configuration (one Bernoulli(0.2) mask shared by all heads, so every routed position is G
    rows): forward outputs of one whole KV group at full length, and -- the configuration itself is forward
    only, the backward is run on top -- dK, dV at key 0, at key-block, chunk (8 key blocks = 1024 keys)
    and window edges, and in the middle of the sequence."""
    w = gen.workload("qwen25_7b_32k")
    T = w.T
    extra = [0, 1, 63, 64, 127, 128, 1023, 1024, 1025, 2047, 2048, w.W - 1, w.W, w.W + 1, T // 2 - 1, T // 2, T // 2 + 1,
             8 * 1024 - 1, 8 * 1024, 24 * 1024 + 127, 24 * 1024 + 128, T - 2]
    full_size_checks(oracle, w, whole_group=True, slab_kv_head=2, extra_keys=extra)


@pytest.mark.timeout(600)
def test_full_size_prefill_bursty_shared_mask_sampled(oracle):
    """Forward only, T = 131072, one bursty mask shared by all heads (every routed position is G rows)."""
    w = gen.workload("prefill_128k")
    x = gen.make_inputs(w, seed=0, with_dO=False)
    lay = layer_from_numpy(x.q, x.k, x.v, x.mask, w.W, w.dtype)
    lay.route(); lay.forward()
    torch.cuda.synchronize()
    pr = oracle.Problem(x.q, x.k, x.v, x.mask, w.W)
    d = pr.mask_per_head().transpose(0, 2, 1)
    rng = np.random.default_rng(2)
    on = np.flatnonzero(x.mask[0, 0])
    starts = on[np.flatnonzero(np.diff(on, prepend=-2) > 1)]          # first token of some bursts
    ts = np.concatenate([[0, w.T - 1], rng.choice(starts, 12), rng.choice(starts, 6) - 1, rng.integers(0, w.T, 20)])
    ts = np.clip(ts, 0, w.T - 1)
    rows = np.array([(0, int(rng.integers(0, w.Hq)), int(t)) for t in ts], dtype=np.int32)
    fr = oracle.fwd_rows(pr, rows)
    assert_close("S", _pick(lay.S, rows), fr["S"], "bf16")
    assert_close("A", _pick(lay.A, rows), fr["A"], "bf16")
    assert_close("O", _pick(lay.O, rows), fr["S"] + fr["A"], "bf16")
    assert_lse("lse_global", np.array([float(lay.lse_g[0, r[1], r[2]]) for r in rows]), fr["lse_g"], "bf16")
    assert any(d[0, r[2], r[1]] for r in rows) and not all(d[0, r[2], r[1]] for r in rows)

"""l2a_route_compact_static -- the routing compaction for callers that cannot allocate or hand over a
workspace (its chunk counters live in a fixed array in the library's device image) -- against
l2a_route_compact on the same masks, bit for bit, on two calls in a row that share the array, the
second with a smaller input; and against the oracle.  Collected last, so that a failure here hides
no other test."""
import numpy as np
import pytest
import torch

from paper_2603_17484_amd import binding as B

pytestmark = pytest.mark.gpu

# (B, T, Hq, Hkv, mask heads, routed fraction): a long input (chunks of 2048 positions, ragged last chunk),
# then a smaller one (chunks of 256), then one that uses a single counter
CALLS = [(2, 70001, 14, 2, 14, 0.3), (1, 3000, 8, 2, 1, 0.6), (1, 5, 4, 4, 4, 0.5)]


def test_static_scratch_route_compact_matches_the_workspace_entry_point(oracle):
    for i, (Bn, T, Hq, Hkv, Hm, f) in enumerate(CALLS):
        print("call", i, (Bn, T, Hq, Hkv, Hm, f), flush=True)
        mask_np = (np.random.default_rng(900 + i).random((Bn, Hm, T)) < f).astype(np.uint8) * 5
        mask = torch.from_numpy(mask_np).cuda()
        p = B.make_params(Bn, T, Hq, Hkv, 128, 64, Hm)
        want = B.alloc_route(p)            # row_idx, count, kblk_first_row, workspace
        B.l2a_route_compact(p, mask, *want)
        got = B.alloc_route(p)[:3]
        for t_ in got:
            t_.fill_(-12345)
        B.l2a_route_compact_static(p, mask, *got)
        torch.cuda.synchronize()
        for name, a, b in zip(("row_idx", "count", "kblk_first_row"), got, want[:3]):
            assert torch.equal(a, b), f"call {i}: {name} differs from l2a_route_compact"
        r, c, k = oracle.route_compact(mask_np, Hq, Hkv)
        assert np.array_equal(got[0].cpu().numpy(), r) and np.array_equal(got[1].cpu().numpy(), c)
        assert np.array_equal(got[2].cpu().numpy(), k)


def test_static_scratch_limit_is_an_error_not_a_launch():
    p = B.make_params(64, 16384, 32, 32, 128, 16)     # 131072 chunk counters > 65536
    x = torch.zeros(64, dtype=torch.int32, device="cuda")
    with pytest.raises(B.L2AError) as e:
        B.l2a_route_compact_static(p, x.view(torch.uint8), x, x, x)
    assert e.value.code == -7

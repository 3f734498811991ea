"""moe_permute_static: the permutation for callers that cannot allocate (static device tables,
no context). Checked bit for bit against moe_permute through the C ABI, and against the oracle,
on two calls in a row, the second with a smaller input; sizes beyond the static tables are
rejected. Collected last on purpose."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2605_17889_amd import binding as B

pytestmark = pytest.mark.gpu


def routed(T, E, k, seed):
    rng = np.random.default_rng(seed)
    return np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)


def call_both(T, E, k, seed):
    idx_h = routed(T, E, k, seed)
    idx = torch.from_numpy(idx_h).cuda()
    R = T * k
    new = lambda n: torch.full((n,), -5, dtype=torch.int32, device="cuda")
    got = [new(E), new(E + 1), new(R), new(R)]
    B.moe_permute_static(idx, T, k, E, *got)
    torch.cuda.synchronize()
    ctx = B.MoeContext(T, 512, 256, E, k)
    want = [new(E), new(E + 1), new(R), new(R)]
    B.moe_permute(ctx, idx, T, *want)
    torch.cuda.synchronize()
    ctx.close()
    oracle = ref.permute(idx_h, E)
    for g, w, o, name in zip(got, want, oracle, ("counts", "offsets", "perm", "inv_perm")):
        assert torch.equal(g, w), f"{name} differs from moe_permute (T={T} E={E} k={k})"
        assert np.array_equal(g.cpu().numpy(), o), f"{name} differs from the oracle"


@pytest.mark.parametrize("first,second", [
    ((30000, 8, 2, 1), (5000, 8, 2, 2)),        # both through the static tables (more than 4096 ids)
    ((9000, 128, 8, 3), (700, 64, 6, 4)),       # many experts; second call under the table limit
    ((16384, 256, 4, 5), (1000, 16, 4, 6)),     # exactly at the limit: 256 segments * 256 experts
])
def test_permute_static_matches_permute_twice(first, second):
    for T, E, k, seed in (first, second):
        print(f"permute_static T={T} E={E} k={k}", flush=True)
        call_both(T, E, k, seed)


def test_permute_static_limits_and_errors():
    one = torch.zeros(8, dtype=torch.int32, device="cuda")
    big = torch.zeros(257, dtype=torch.int32, device="cuda")
    with pytest.raises(B.MoeError, match="UNSUPPORTED_SHAPE"):       # 257 segments * 256 experts
        B.moe_permute_static(one, 16385, 4, 256, big, big, one, one)
    with pytest.raises(B.MoeError, match="INVALID_ARG"):
        B.moe_permute_static(one, 4, 3, 2, one, one, one, one)       # k > E
    with pytest.raises(B.MoeError, match="INVALID_ARG"):
        B.moe_permute_static(None, 4, 2, 8, one, big, one, one)
    counts = torch.full((8,), -1, dtype=torch.int32, device="cuda")
    offsets = torch.full((9,), -1, dtype=torch.int32, device="cuda")
    B.moe_permute_static(None, 0, 2, 8, counts, offsets, None, None)  # T = 0: empty tables
    torch.cuda.synchronize()
    assert int(counts.abs().sum()) == 0 and int(offsets.abs().sum()) == 0

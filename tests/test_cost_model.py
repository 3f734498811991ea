"""The library's expert-stage roofline estimate (host arithmetic, no GPU) against the oracle's
cost model (oracle/cost_model.py, written from Table 1 row 3 and Eq. 5 / Eq. 9) and against
properties that hold for any input."""
import math

import numpy as np
import pytest

from oracle.cost_model import expert_stage_estimate as oracle_estimate
from paper_2605_17889_amd import binding as B

FIELDS = ("flops", "operand_bytes", "intermediate_bytes", "t_stage_s", "t_per_expert_s",
          "t_kernels_s", "ridge_rows")
COUNTS = ("micro_batches", "expert_instances", "memory_bound_instances")


def close(a, b):
    return a == b or abs(a - b) <= 1e-12 * max(abs(a), abs(b))


@pytest.mark.parametrize("d,f,tf,bw,rows", [
    (6144, 16384, 2500.0, 8000.0, [[2018, 2006, 2061, 2096, 2112, 2027, 2037, 2027]]),
    (4096, 14336, 2500.0, 8000.0, [[59, 68, 64, 71, 65, 58, 54, 73]]),
    (6144, 16384, 1330.0, 5400.0, [[56, 61, 75, 58, 62, 67, 68, 65]] * 16),
    (6144, 16384, 2500.0, 8000.0, [[2125, 0, 14422, 3927, 1415, 2780, 1710, 6389]]),
    (2048, 768, 2500.0, 8000.0, [list(range(0, 128))]),
    (512, 1024, 100.0, 50.0, [[1, 0, 0, 7], [0, 0, 0, 0], [300, 312, 313, 5000]]),
])
def test_library_matches_oracle(d, f, tf, bw, rows):
    got = B.moe_estimate_expert_stage(d, f, rows, tf, bw)
    want = oracle_estimate(rows, d, f, tf, bw)
    for name in COUNTS:
        assert got[name] == want[name], name
    for name in FIELDS:
        assert close(got[name], want[name]), (name, got[name], want[name])


def test_random_inputs_match_oracle_and_invariants():
    rng = np.random.default_rng(7)
    for _ in range(50):
        E = int(rng.integers(1, 40))
        M = int(rng.integers(1, 6))
        d, f = int(rng.integers(1, 64)) * 128, int(rng.integers(1, 64)) * 128
        rows = rng.integers(0, 3000, size=(M, E)) * (rng.random((M, E)) < 0.8)
        rows = rows.astype(int).tolist()
        tf, bw = float(rng.uniform(10, 3000)), float(rng.uniform(100, 9000))
        got = B.moe_estimate_expert_stage(d, f, rows, tf, bw)
        want = oracle_estimate(rows, d, f, tf, bw)
        for name in FIELDS:
            assert close(got[name], want[name]), name
        # max of sums <= sum of maxes; both at least the pure compute and the pure memory time
        assert got["t_stage_s"] <= got["t_per_expert_s"] * (1 + 1e-12)
        assert got["t_stage_s"] * (1 + 1e-12) >= got["flops"] / (tf * 1e12)
        assert got["t_per_expert_s"] * (1 + 1e-12) >= got["operand_bytes"] / (bw * 1e9)
        assert got["flops"] == 6.0 * sum(map(sum, rows)) * d * f
        # an expert is memory-bound exactly when it has fewer rows than the ridge
        ridge = got["ridge_rows"]
        n_mem = sum(1 for mb in rows for r in mb if 0 < r < ridge)
        assert got["memory_bound_instances"] == n_mem


def test_micro_batching_multiplies_weight_traffic():
    """Section 3.1: the same tokens in M micro-batches re-read every active expert's weights M
    times; in the memory-bound regime halving the micro-batch doubles the time."""
    d, f = 6144, 16384
    whole = B.moe_estimate_expert_stage(d, f, [[1024] * 8], 2500.0, 8000.0)
    split16 = B.moe_estimate_expert_stage(d, f, [[64] * 8] * 16, 2500.0, 8000.0)
    split32 = B.moe_estimate_expert_stage(d, f, [[32] * 8] * 32, 2500.0, 8000.0)
    assert whole["flops"] == split16["flops"] == split32["flops"]
    assert whole["memory_bound_instances"] == 0 and split16["memory_bound_instances"] == 128
    w = 8 * 6.0 * d * f
    assert close(split16["operand_bytes"] - whole["operand_bytes"], 15 * w)
    assert 1.98 < split32["t_stage_s"] / split16["t_stage_s"] < 2.0
    assert split16["t_stage_s"] > 4.8 * whole["t_stage_s"]


def test_argument_errors():
    with pytest.raises(B.MoeError):
        B.moe_estimate_expert_stage(6144, 16384, [[-1, 2]], 2500.0, 8000.0)
    with pytest.raises(B.MoeError):
        B.moe_estimate_expert_stage(6144, 16384, [[1, 2]], 0.0, 8000.0)
    with pytest.raises(B.MoeError):
        B.moe_estimate_expert_stage(0, 16384, [[1, 2]], 2500.0, 8000.0)
    empty = B.moe_estimate_expert_stage(6144, 16384, [], 2500.0, 8000.0)
    assert empty["t_stage_s"] == 0.0 and empty["micro_batches"] == 0
    assert math.isfinite(empty["ridge_rows"])

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


# ------------------------------------------------------------------ experts moved over PCIe
def test_streamed_estimate_matches_oracle_and_invariants():
    """moe_estimate_streamed_stage against the oracle's Eq. 7 / Eq. 3 arithmetic, and properties:
    the load term grows by exactly one expert's matrices per moved expert, the sum is at least
    the overlap, and the two agree when nothing moves."""
    from oracle.cost_model import streamed_expert_stage_estimate as oracle_streamed
    rng = np.random.default_rng(11)
    for _ in range(40):
        E = int(rng.integers(1, 130))
        d, f = int(rng.integers(1, 64)) * 128, int(rng.integers(1, 64)) * 128
        rows = (rng.integers(0, 3000, size=E) * (rng.random(E) < 0.8)).astype(int).tolist()
        tf, bw, pcie = float(rng.uniform(10, 3000)), float(rng.uniform(100, 9000)), float(rng.uniform(5, 120))
        n = int(rng.integers(0, E + 1))
        on_dev = bool(rng.integers(0, 2))
        got = B.moe_estimate_streamed_stage(d, f, rows, n, tf, bw, pcie, on_dev)
        want = oracle_streamed(rows, d, f, n, tf, bw, pcie, on_dev)
        for name in ("moved_bytes", "t_load_s", "t_comp_s", "t_sum_s", "t_overlap_s"):
            assert close(got[name], want[name]), name
        assert got["t_sum_s"] >= got["t_overlap_s"] >= max(got["t_load_s"], got["t_comp_s"]) * (1 - 1e-12)
        if n < E:
            more = B.moe_estimate_streamed_stage(d, f, rows, n + 1, tf, bw, pcie, on_dev)
            assert close(more["moved_bytes"] - got["moved_bytes"], 6.0 * d * f)
            assert close(more["t_comp_s"], got["t_comp_s"])
    none = B.moe_estimate_streamed_stage(512, 128, [5, 0, 9], 0, 100.0, 100.0, 10.0, True)
    assert none["t_load_s"] == 0.0 and none["t_sum_s"] == none["t_overlap_s"] == none["t_comp_s"]


def test_streamed_estimate_argument_errors():
    import ctypes as C
    L = B.lib()
    shape = B.MoeShape(0, 512, 128, 4, 1)
    mach = B.MoeMachine(100.0, 100.0)
    rows = (C.c_int32 * 4)(1, 2, 3, 4)
    out = B.MoeStreamedEstimate()
    ok = lambda *a: L.moe_estimate_streamed_stage(*a)
    assert ok(C.byref(shape), rows, 2, C.byref(mach), C.c_double(10.0), 1, C.byref(out)) == 0
    assert ok(None, rows, 2, C.byref(mach), C.c_double(10.0), 1, C.byref(out)) == -1
    assert ok(C.byref(shape), None, 2, C.byref(mach), C.c_double(10.0), 1, C.byref(out)) == -1
    assert ok(C.byref(shape), rows, 5, C.byref(mach), C.c_double(10.0), 1, C.byref(out)) == -1
    assert ok(C.byref(shape), rows, -1, C.byref(mach), C.c_double(10.0), 1, C.byref(out)) == -1
    assert ok(C.byref(shape), rows, 2, C.byref(mach), C.c_double(0.0), 1, C.byref(out)) == -1
    assert ok(C.byref(shape), rows, 2, C.byref(mach), C.c_double(10.0), 1, None) == -1

"""The expert-stage roofline estimate against measurement on the GPU (the paper's motivation
curve, Section 3.1: under micro-batching the experts are memory-bound and halving the
micro-batch nearly doubles the expert latency; Eq. 5 / Eq. 9 with Table 1 row 3 give the bound).

At the Mixtral-8x22B shape with T = 4096 tokens, run as micro-batches of m tokens:
  * the measured time of the two grouped GEMMs (HIP events around the launches) is never below
    moe_estimate_expert_stage's t_stage_s at the published peaks (2.5 PFLOP/s, 8 TB/s);
  * memory_bound_instances equals the number of (micro-batch, expert) groups whose row count,
    as the library's own routing produced it, lies below ridge_rows;
  * time(m = 64) / time(m = 128) is about 2."""
import numpy as np
import pytest
import torch

from paper_2605_17889_amd import binding as B
from paper_2605_17889_amd import synth

pytestmark = pytest.mark.gpu

PEAK_TFLOPS, PEAK_GBS = 2500.0, 8000.0


def test_estimate_bounds_measured_expert_time(experts_8x22b):
    cfg = synth.PRESETS["mixtral8x22b_coalesce"]
    (W1, W3, W2), _ = experts_8x22b
    T, E, k = cfg.T, cfg.E, cfg.k
    x = synth.make_tokens(cfg, "cuda")
    wr = synth.make_router(cfg, "cuda")
    ctx = B.MoeContext(T, cfg.d_model, cfg.d_ff, E, k)
    y = torch.empty((T, cfg.d_model), dtype=torch.bfloat16, device="cuda")
    idx = torch.empty((T, k), dtype=torch.int32, device="cuda")
    w = torch.empty((T, k), dtype=torch.float32, device="cuda")
    B.moe_route(ctx, x, wr, None, T, idx, w)      # routing is per token: the same in every split
    torch.cuda.synchronize()
    idx_h = idx.cpu().numpy()
    measured = {}
    for m in (64, 128, 256, T):
        rows = [np.bincount(idx_h[t0:t0 + m].reshape(-1), minlength=E).tolist() for t0 in range(0, T, m)]

        def step():
            if m < T:
                B.moe_layer_forward_microbatched(ctx, x, wr, None, W1, W3, W2, T, m, y)
            else:
                B.moe_layer_forward(ctx, x, wr, None, W1, W3, W2, T, y)

        step()
        torch.cuda.synchronize()
        # the tables the call left behind are those of its last micro-batch
        counts = torch.empty(E, dtype=torch.int32, device="cuda")
        B.moe_last_routing(ctx, min(m, T), counts=counts)
        torch.cuda.synchronize()
        assert counts.cpu().tolist() == rows[-1]
        steps = 3
        B.moe_profile_begin(ctx, steps)
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        stage_ms, _, calls = B.moe_profile_end(ctx)
        assert calls == steps
        ms = (stage_ms["gateup"] + stage_ms["down"]) / steps
        est = B.moe_estimate_expert_stage(cfg.d_model, cfg.d_ff, rows, PEAK_TFLOPS, PEAK_GBS)
        below_ridge = sum(1 for mb in rows for r in mb if 0 < r < est["ridge_rows"])
        print(f"m={m}: measured {ms:.3f} ms, bound {est['t_stage_s'] * 1e3:.3f} ms, memory-bound "
              f"{est['memory_bound_instances']} of {est['expert_instances']} groups, ridge "
              f"{est['ridge_rows']:.0f} rows", flush=True)
        assert est["memory_bound_instances"] == below_ridge
        assert est["expert_instances"] == sum(1 for mb in rows for r in mb if r > 0)
        assert ms * 1e-3 >= est["t_stage_s"], (m, ms, est["t_stage_s"])
        measured[m] = ms
    ratio = measured[64] / measured[128]
    print(f"time(m=64) / time(m=128) = {ratio:.3f}", flush=True)
    assert 1.8 <= ratio <= 2.2
    # coalesced execution is compute-bound at this shape: no group below the ridge
    est = B.moe_estimate_expert_stage(cfg.d_model, cfg.d_ff,
                                      [np.bincount(idx_h.reshape(-1), minlength=E).tolist()],
                                      PEAK_TFLOPS, PEAK_GBS)
    assert est["memory_bound_instances"] == 0
    assert measured[256] / measured[T] > 2.0      # the intensity collapse of micro-batching
    ctx.close()

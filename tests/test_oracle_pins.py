"""Pins for the CPU oracle: it is checked against hand-derived values, closed forms,
library routines on special cases, brute force of a different code shape, and invariants —
never against itself and never against the HIP path. CPU only."""
import json
import math
import os

import numpy as np
import pytest
import torch

from oracle import ref
from paper_2605_17889_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _load(name):
    with open(os.path.join(GOLD, name)) as fh:
        return json.load(fh)


def _bf16_bits_from_float(a):
    """float array whose values are bf16-exact -> uint16 raw bits (asserts exactness)."""
    a32 = np.asarray(a, np.float32)
    bits = (a32.view(np.uint32) >> 16).astype(np.uint16)
    back = (bits.astype(np.uint32) << 16).view(np.float32)
    assert np.array_equal(back, a32), "fixture value is not bf16-exact"
    return bits


def _bf16_to_f64(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def _hx(s):
    return float.fromhex(s) if isinstance(s, str) and "x" in s else float(s)


# --------------------------------------------------------------------------- router logits
@pytest.mark.parametrize("case", _load("route_tree_cases.json")["cases"], ids=lambda c: c["name"])
def test_logit_tree_hand_cases(case):
    d, E = case["d"], case["E"]
    x = np.zeros((1, d), np.float32)
    for i, v in case["x"].items():
        x[0, int(i)] = _hx(v)
    w = np.full((d, E), _hx(case["w_default"]), np.float32)
    for key, v in case["w"].items():
        if "," in key:
            i, e = (int(s) for s in key.split(","))
        else:
            i, e = int(key), 0
        w[i, e] = _hx(v)
    bias = None if case["bias"] is None else np.array([_hx(b) for b in case["bias"]], np.float32)
    got = ref.logits(_bf16_bits_from_float(x), w, bias)
    want = np.array([_hx(v) for v in case["expected"]], np.float32)
    assert np.array_equal(got[0].view(np.uint32), want.view(np.uint32)), (got, want)


def test_logits_exact_on_small_integers():
    """When every product and partial sum is an exactly representable integer, any correct
    summation returns the exact dot product; compare with an int64 matmul."""
    rng = np.random.default_rng(11)
    T, d, E = 5, 1024, 7
    xi = rng.integers(-8, 9, size=(T, d))
    wi = rng.integers(-16, 17, size=(d, E))
    got = ref.logits(_bf16_bits_from_float(xi.astype(np.float32)), wi.astype(np.float32))
    assert np.array_equal(got.astype(np.int64), xi @ wi)


def test_logits_within_fp32_bound_of_double():
    """The canonical fp32 logit stays within the standard forward error bound
    (d * 2^-24 * sum|x_i w_i|) of the double-precision dot product from numpy."""
    cfg = synth.PRESETS["tiny"]
    x = synth.bf16_bits(synth.make_tokens(cfg))
    w = synth.make_router(cfg).numpy()
    got = ref.logits(x, w)
    xd = _bf16_to_f64(x)
    exact = xd @ w.astype(np.float64)
    bound = cfg.d_model * 2.0 ** -24 * (np.abs(xd) @ np.abs(w.astype(np.float64)))
    assert np.all(np.abs(got - exact) <= bound)
    assert np.max(np.abs(got - exact)) > 0          # it really is an fp32 sum, not the double one
    assert np.allclose(ref.logits_f64(x, w), exact, rtol=1e-13, atol=1e-13)


# --------------------------------------------------------------------------------- top-k
@pytest.mark.parametrize("case", _load("topk_cases.json")["cases"], ids=lambda c: c["name"])
def test_topk_hand_cases(case):
    lg = np.array([[float(v) for v in case["logits"]]], np.float32)
    idx, g = ref.topk(lg, case["k"])
    assert idx[0].tolist() == case["idx"]
    assert abs(float(g[0].sum()) - 1.0) <= 1e-6
    if "gates" in case:
        assert np.allclose(g[0], case["gates"], atol=2e-7)


def test_topk_equals_full_sort_and_gate_identities():
    """Brute force: a full stable sort of (-logit, index) gives the same order; for k = 2 the
    gates have the closed form sigmoid(l0 - l1); softmax over all experts followed by
    renormalisation over the selected ones equals the softmax over the selected logits."""
    rng = np.random.default_rng(5)
    T, E = 400, 8
    lg = rng.normal(0, 1.5, size=(T, E)).astype(np.float32)
    lg[::7, 3] = lg[::7, 5]                      # plant exact ties
    lg[::11] = np.round(lg[::11])                # and many more
    for k in (1, 2, 3, 8):
        idx, g = ref.topk(lg, k)
        order = np.argsort(-lg.astype(np.float64), axis=1, kind="stable")[:, :k]
        assert np.array_equal(idx, order)
        assert np.all(np.abs(g.sum(1) - 1) <= 1e-6)
        full = np.exp(lg.astype(np.float64) - lg.max(1, keepdims=True))
        full /= full.sum(1, keepdims=True)
        sel = np.take_along_axis(full, idx.astype(np.int64), 1)
        sel /= sel.sum(1, keepdims=True)
        assert np.allclose(g, sel, atol=1e-7)
        if k == E:
            assert np.array_equal(np.sort(idx, 1), np.tile(np.arange(E), (T, 1)))
        if k == 2:
            l0 = np.take_along_axis(lg, idx[:, :1].astype(np.int64), 1)[:, 0].astype(np.float64)
            l1 = np.take_along_axis(lg, idx[:, 1:].astype(np.int64), 1)[:, 0].astype(np.float64)
            assert np.allclose(g[:, 0], 1 / (1 + np.exp(l1 - l0)), atol=1e-7)


@pytest.mark.parametrize("E,ks", [(128, (1, 8, 64)), (200, (6, 33)), (256, (64,))])
def test_topk_many_experts_equals_full_sort(E, ks):
    """The same brute force with more than 64 experts (several experts per lane on the GPU),
    planted ties across the 64-expert boundaries and a row of all-equal logits."""
    rng = np.random.default_rng(E)
    T = 120
    lg = rng.normal(0, 1.5, size=(T, E)).astype(np.float32)
    lg[::5, 3] = lg[::5, 67]
    lg[::5, E - 1] = lg[::5, 3]
    lg[1::9] = np.round(lg[1::9])
    lg[7] = 0.25
    for k in ks:
        idx, g = ref.topk(lg, k)
        order = np.argsort(-lg.astype(np.float64), axis=1, kind="stable")[:, :k]
        assert np.array_equal(idx, order)
        assert np.all(np.abs(g.sum(1) - 1) <= 1e-5)
        assert np.allclose(g[7], 1.0 / k, atol=1e-7) and idx[7].tolist() == list(range(k))
        sel = np.take_along_axis(lg.astype(np.float64), idx.astype(np.int64), 1)
        w = np.exp(sel - sel[:, :1])
        assert np.allclose(g, w / w.sum(1, keepdims=True), atol=1e-7)


# ----------------------------------------------------------------------------- permutation
def test_permute_worked_example():
    c = _load("permute_worked_example.json")
    counts, offsets, perm, inv = ref.permute(np.array(c["topk_idx"], np.int32), c["E"])
    assert counts.tolist() == c["counts"] and offsets.tolist() == c["offsets"]
    assert perm.tolist() == c["perm"] and inv.tolist() == c["inv_perm"]


@pytest.mark.parametrize("T,E,k,seed", [(1, 4, 1, 0), (37, 8, 2, 1), (1000, 64, 6, 2), (513, 3, 3, 3),
                                        (700, 128, 8, 4), (300, 256, 64, 5), (90, 200, 5, 6)])
def test_permute_matches_stable_sort_and_invariants(T, E, k, seed):
    rng = np.random.default_rng(seed)
    idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    if E > 2:
        idx[idx == 2] = 1 if k == 1 else idx[idx == 2]      # k=1: leave expert 2 empty
    counts, offsets, perm, inv = ref.permute(idx, E)
    flat = idx.reshape(-1)
    R = T * k
    assert counts.sum() == R                                  # sum of counts = T*k
    assert np.array_equal(counts, np.bincount(flat, minlength=E))
    assert offsets[0] == 0 and offsets[-1] == R and np.array_equal(np.diff(offsets), counts)
    assert np.array_equal(perm, np.argsort(flat, kind="stable"))   # library routine
    assert np.array_equal(perm[inv], np.arange(R)) and np.array_equal(inv[perm], np.arange(R))
    e_sorted = flat[perm]
    assert np.all(np.diff(e_sorted) >= 0)
    same = np.diff(e_sorted) == 0
    assert np.all(np.diff(perm)[same] > 0)                    # stability inside a group


def test_gather_is_row_copy():
    rng = np.random.default_rng(9)
    x = rng.integers(0, 65536, size=(6, 16)).astype(np.uint16)
    perm = np.array([3, 0, 5, 11, 7, 1, 2, 4, 6, 8, 9, 10], np.int32)
    got = ref.gather(x, perm, 2)
    assert np.array_equal(got, x[perm // 2])


# ------------------------------------------------------------------------------ expert FFN
def test_ffn_worked_example_by_hand():
    c = _load("ffn_worked_example.json")
    assert abs(c["silu_1"] - 1 / (1 + math.exp(-1))) < 1e-16
    xb = _bf16_bits_from_float(np.array([c["x"]], np.float32))
    W1 = _bf16_bits_from_float(np.array([c["W1"]], np.float32))
    W3 = _bf16_bits_from_float(np.array([c["W3"]], np.float32))
    W2 = _bf16_bits_from_float(np.array([c["W2"]], np.float32))
    y, h = ref.expert_ffn(xb, np.array([0, 1], np.int32), W1, W3, W2, want_h=True)
    assert np.allclose(h[0], [2 * c["silu_1"], 0.0], rtol=1e-15, atol=0)
    assert np.allclose(y[0], c["o"], rtol=1e-15)


def test_ffn_scalar_closed_form():
    for xv, w1, w3, w2 in [(1.5, -2.0, 0.5, 3.0), (-0.75, 1.25, -4.0, 0.125), (0.0, 1.0, 1.0, 1.0)]:
        b = lambda v: _bf16_bits_from_float(np.array(v, np.float32).reshape(1, 1, 1))
        y = ref.expert_ffn(b(xv).reshape(1, 1), np.array([0, 1], np.int32), b(w1), b(w3), b(w2))
        a = w1 * xv
        want = w2 * (a / (1 + math.exp(-a))) * (w3 * xv)
        assert y.shape == (1, 1) and abs(y[0, 0] - want) <= 1e-15 * max(1.0, abs(want))


def test_ffn_identity_weights_closed_form():
    """f = d and W1 = W3 = W2 = I  =>  y = SiLU(x) * x elementwise."""
    d = 24
    rng = np.random.default_rng(2)
    xb = _bf16_bits_from_float(torch.tensor(rng.normal(size=(5, d))).bfloat16().float().numpy())
    eye = _bf16_bits_from_float(np.eye(d, dtype=np.float32)[None])
    y = ref.expert_ffn(xb, np.array([0, 5], np.int32), eye, eye, eye)
    xv = _bf16_to_f64(xb)
    assert np.allclose(y, xv / (1 + np.exp(-xv)) * xv, rtol=1e-14, atol=1e-300)


def _rand_bits(rng, shape, std):
    return synth.bf16_bits(torch.tensor(rng.normal(0, std, size=shape), dtype=torch.float32).bfloat16())


def test_single_expert_is_three_library_matmuls():
    """E = 1, k = 1 is a plain SwiGLU MLP: three numpy matmuls with non-square, asymmetric
    weights (catches a transposed operand or swapped W1/W3/W2)."""
    rng = np.random.default_rng(3)
    T, d, f = 9, 512, 96
    x = _rand_bits(rng, (T, d), 1.0)
    W1, W3, W2 = _rand_bits(rng, (1, f, d), 0.05), _rand_bits(rng, (1, f, d), 0.05), _rand_bits(rng, (1, d, f), 0.05)
    wr = rng.normal(0, 0.02, size=(d, 1)).astype(np.float32)
    y, idx, g = ref.layer_tokens(x, wr, None, W1, W3, W2, 1)
    assert np.all(idx == 0) and np.all(g == 1.0)
    xd = _bf16_to_f64(x)
    a = xd @ _bf16_to_f64(W1[0]).T
    b = xd @ _bf16_to_f64(W3[0]).T
    want = (a / (1 + np.exp(-a)) * b) @ _bf16_to_f64(W2[0]).T
    assert np.allclose(y, want, rtol=1e-12, atol=1e-14)


def _dense_bruteforce(x, lg, W1, W3, W2, k):
    """Per-token dense evaluation: run ALL experts, weight them with a dense gate vector that
    is the softmax over all E logits, zeroed off the top-k and renormalised."""
    T, d = x.shape
    E = W1.shape[0]
    xd = _bf16_to_f64(x)
    y = np.zeros((T, d))
    for t in range(T):
        l = lg[t].astype(np.float64)
        order = sorted(range(E), key=lambda e: (-l[e], e))[:k]
        p = np.exp(l - l.max())
        p /= p.sum()
        dense = np.zeros(E)
        dense[order] = p[order]
        dense /= dense.sum()
        for e in range(E):
            a = _bf16_to_f64(W1[e]) @ xd[t]
            b = _bf16_to_f64(W3[e]) @ xd[t]
            y[t] += dense[e] * (_bf16_to_f64(W2[e]) @ (a / (1 + np.exp(-a)) * b))
    return y


@pytest.mark.parametrize("E,k", [(8, 2), (5, 3), (4, 4), (128, 8), (64, 6)])
def test_layer_equals_dense_bruteforce(E, k):
    rng = np.random.default_rng(100 + E)
    T, d, f = 24, 512, 40
    x = _rand_bits(rng, (T, d), 1.0)
    W1, W3, W2 = _rand_bits(rng, (E, f, d), 0.05), _rand_bits(rng, (E, f, d), 0.05), _rand_bits(rng, (E, d, f), 0.05)
    wr = rng.normal(0, 0.05, size=(d, E)).astype(np.float32)
    bias = rng.normal(0, 0.5, size=E).astype(np.float32)
    y, idx, g = ref.layer_tokens(x, wr, bias, W1, W3, W2, k)
    lg = ref.logits(x, wr, bias)
    want = _dense_bruteforce(x, lg, W1, W3, W2, k)
    scale = np.abs(want).max()
    assert np.max(np.abs(y - want)) <= 1e-7 * scale      # gates are rounded to fp32 (2^-24)
    assert np.all(np.abs(g.sum(1) - 1) <= 1e-6)          # gates sum to one


def test_tiny_config_dense_bruteforce_and_invariants():
    cfg = synth.PRESETS["tiny"]
    L = synth.make_layer(cfg)
    x, wr = synth.bf16_bits(L["x"]), L["w_router"].numpy()
    W1, W3, W2 = (synth.bf16_bits(L[n]) for n in ("W1", "W3", "W2"))
    tokens = np.arange(0, cfg.T, 8, dtype=np.int32)
    y, idx, g = ref.layer_tokens(x, wr, None, W1, W3, W2, cfg.k, tokens)
    lg = ref.logits(x, wr)
    want = _dense_bruteforce(x[tokens], lg[tokens], W1, W3, W2, cfg.k)
    assert np.max(np.abs(y - want)) <= 1e-7 * np.abs(want).max()
    idx_all, g_all = ref.topk(lg, cfg.k)
    counts, offsets, perm, inv = ref.permute(idx_all, cfg.E)
    assert counts.sum() == cfg.T * cfg.k
    assert np.all(np.abs(g_all.sum(1) - 1) <= 1e-6)
    assert np.array_equal(idx_all[tokens], idx)


def test_linearity_equivariance_zero_row():
    rng = np.random.default_rng(42)
    T, d, f, E, k = 12, 512, 32, 4, 2
    x = _rand_bits(rng, (T, d), 1.0)
    x[5] = 0                                             # a zero token
    W1, W3, W2 = _rand_bits(rng, (E, f, d), 0.05), _rand_bits(rng, (E, f, d), 0.05), _rand_bits(rng, (E, d, f), 0.05)
    wr = rng.normal(0, 0.05, size=(d, E)).astype(np.float32)
    y, idx, g = ref.layer_tokens(x, wr, None, W1, W3, W2, k)
    assert np.all(y[5] == 0)
    # doubling W2 of one expert doubles exactly that expert's contribution
    e = 1
    W2b = W2.copy()
    W2b[e] = _bf16_bits_from_float(2 * (W2[e].astype(np.uint32) << 16).view(np.float32))
    y2, _, _ = ref.layer_tokens(x, wr, None, W1, W3, W2b, k)
    xp_rows = np.arange(T)
    contrib = np.zeros_like(y)
    for t in xp_rows:
        for s in range(k):
            if idx[t, s] == e:
                o = ref.expert_ffn(x[t:t + 1], np.array([0] * (e + 1) + [1] * (E - e), np.int32), W1, W3, W2)
                contrib[t] = g[t, s] * o[0]
    assert np.allclose(y2 - y, contrib, rtol=1e-9, atol=1e-12)
    assert np.any(contrib != 0)
    # permuting tokens permutes outputs
    p = rng.permutation(T)
    yp, _, _ = ref.layer_tokens(np.ascontiguousarray(x[p]), wr, None, W1, W3, W2, k)
    assert np.array_equal(yp, y[p])


@pytest.mark.parametrize("m", [1, 7, 64, 100, 10 ** 6])
def test_coalesced_equals_microbatched(m):
    """Running the stages over micro-batches of any size m reproduces the per-token definition
    bit for bit (the oracle's statement of Opportunity 1: coalescing changes cost, not results)."""
    rng = np.random.default_rng(7)
    T, d, f, E, k = 100, 512, 24, 8, 2
    x = _rand_bits(rng, (T, d), 1.0)
    W1, W3, W2 = _rand_bits(rng, (E, f, d), 0.05), _rand_bits(rng, (E, f, d), 0.05), _rand_bits(rng, (E, d, f), 0.05)
    wr = rng.normal(0, 0.05, size=(d, E)).astype(np.float32)
    y_def, _, _ = ref.layer_tokens(x, wr, None, W1, W3, W2, k)
    y_m = ref.layer_staged(x, wr, None, W1, W3, W2, k, m)
    assert np.array_equal(y_def, y_m)


def test_combine_stage_matches_numpy():
    rng = np.random.default_rng(8)
    T, d, k = 10, 8, 3
    yp = rng.normal(size=(T * k, d))
    inv = rng.permutation(T * k).astype(np.int32)
    g = rng.random(size=(T, k)).astype(np.float32)
    want = np.einsum("tk,tkd->td", g.astype(np.float64), yp[inv.reshape(T, k)])
    assert np.allclose(ref.combine(yp, inv, g), want, rtol=1e-14)
    bits = _rand_bits(rng, (T * k, d), 1.0)
    want = np.einsum("tk,tkd->td", g.astype(np.float64), _bf16_to_f64(bits)[inv.reshape(T, k)])
    assert np.allclose(ref.combine(bits, inv, g), want, rtol=1e-14)


def test_argument_errors():
    with pytest.raises(ValueError):
        ref.logits(np.zeros((1, 100), np.uint16), np.zeros((100, 2), np.float32))   # d % 512
    with pytest.raises(ValueError):
        ref.topk(np.zeros((1, 4), np.float32), 5)                                     # k > E
    with pytest.raises(ValueError):
        ref.permute(np.array([[0, 9]], np.int32), 4)                                  # index range


# ------------------------------------------------------------------------- cost accounting
def test_table1_row3_accounting():
    """Table 1 row 3: per expert D_Y = 6*d_h*d_e bytes, C = 6*rows*d_h*d_e FLOPs."""
    c = synth.PRESETS["mixtral8x22b_prefill"]
    assert synth.expert_ffn_flops(c.R, c.d_model, c.d_ff) == 6 * 16384 * 6144 * 16384
    assert synth.expert_weight_bytes(c.E, c.d_model, c.d_ff) == 8 * 6 * 6144 * 16384
    assert abs(synth.expert_ffn_flops(c.R, c.d_model, c.d_ff) / 1e12 - 9.896) < 1e-3


def test_zipf_calibration_with_oracle_router():
    cfg = synth.LayerConfig("zipf_small", 4096, 512, 64, 8, 2, seed=77, zipf_s=1.2, empty_expert=True)
    x = synth.bf16_bits(synth.make_tokens(cfg))
    wr = synth.make_router(cfg).numpy()
    base = ref.logits(x, wr)

    def count_fn(bias):
        idx, _ = ref.topk(base + bias.numpy()[None, :], cfg.k)
        return np.bincount(idx.reshape(-1), minlength=cfg.E)

    bias = synth.calibrate_expert_bias(cfg, count_fn)
    counts = count_fn(bias)
    target = synth.zipf_target_counts(cfg).numpy()
    live = target > 0
    assert counts[~live].sum() == 0 and (~live).sum() == 1
    assert np.all(np.abs(counts[live] - target[live]) <= 0.02 * target[live] + 2)
    srt = np.sort(target[live])[::-1]
    assert np.allclose(srt / srt[0], np.arange(1, 8) ** -1.2, rtol=1e-12)


# ------------------------------------------------------------------------- roofline cost model
def test_cost_model_hand_values():
    """Eq. 5 / Eq. 9 with Table 1 row 3, against values worked out by hand."""
    from oracle.cost_model import expert_stage_estimate as est
    # one expert, 1000 rows, d_h = 1000, d_e = 2000, device 1 TFLOP/s and 1 GB/s:
    # D_X = 2e6 B, D_Y = 12e6 B, C = 12e9 FLOP -> memory 14e6/1e9 = 0.014 s, compute 0.012 s
    o = est([[1000]], 1000, 2000, 1.0, 1.0)
    assert o["flops"] == 12e9 and o["operand_bytes"] == 14e6
    assert abs(o["t_stage_s"] - 0.014) < 1e-15 and abs(o["t_per_expert_s"] - 0.014) < 1e-15
    assert o["memory_bound_instances"] == 1 and o["expert_instances"] == 1
    # same expert on a 0.5 TFLOP/s device: compute 0.024 s wins
    o = est([[1000]], 1000, 2000, 0.5, 1.0)
    assert abs(o["t_stage_s"] - 0.024) < 1e-15 and o["memory_bound_instances"] == 0
    # ridge: (2 r d + 6 d f)/BW = 6 r d f/TF  ->  r = 12e6/1e9 / (12e6/1e12 - 2e3/1e9) = 1200
    assert abs(est([[1]], 1000, 2000, 1.0, 1.0)["ridge_rows"] - 1200.0) < 1e-9
    # two experts (300 and 0 rows) in each of 2 micro-batches: empty experts cost nothing, M = 2 doubles
    a = est([[300, 0]], 1000, 2000, 1.0, 1.0)
    b = est([[300, 0], [300, 0]], 1000, 2000, 1.0, 1.0)
    assert a["expert_instances"] == 1 and b["expert_instances"] == 2
    assert abs(b["t_stage_s"] - 2 * a["t_stage_s"]) < 1e-18 and b["micro_batches"] == 2
    # stage form never exceeds the per-expert form (max of sums <= sum of maxes)
    c = est([[5000, 10]], 1000, 2000, 1.0, 1.0)
    assert c["t_stage_s"] <= c["t_per_expert_s"] + 1e-18
    # 5000 rows: compute 0.06 s vs memory 0.022 s; 10 rows: memory 0.01202 s vs compute 0.00012 s
    assert abs(c["t_per_expert_s"] - (0.06 + 0.01202)) < 1e-12
    assert abs(c["t_stage_s"] - max((10e6 + 12e6 + 2e4 + 12e6) / 1e9, 0.06012)) < 1e-12


def test_cost_model_per_kernel_split_hand_values():
    """t_kernels_s and intermediate_bytes by hand. The split of the stage into its two grouped
    contractions, with the intermediate H counted, is this repository's extension of Table 1
    row 3 / Eq. 5 (the table prices the stage as one operation and leaves H out).
    One expert, 1000 rows, d_h = 1000, d_e = 2000, 1 TFLOP/s, 1 GB/s:
      gate/up: bytes = x rows 2e6 + W1,W3 8e6 + H written 4e6 = 14e6 -> 0.014 s; 8e9 FLOP -> 0.008 s
      down   : bytes = H read 4e6 + W2 4e6 + outputs 2e6     = 10e6 -> 0.010 s; 4e9 FLOP -> 0.004 s
      t_kernels = max(0.014, 0.008) + max(0.010, 0.004) = 0.024 s
      intermediate_bytes = H written 4e6 + H read 4e6 + outputs 2e6 = 10e6"""
    from oracle.cost_model import expert_stage_estimate as est
    o = est([[1000]], 1000, 2000, 1.0, 1.0)
    assert o["intermediate_bytes"] == 10e6
    assert abs(o["t_kernels_s"] - 0.024) < 1e-15
    # 0.5 TFLOP/s: gate/up compute 0.016 > 0.014, down memory 0.010 > 0.008 -> 0.026
    assert abs(est([[1000]], 1000, 2000, 0.5, 1.0)["t_kernels_s"] - 0.026) < 1e-15
    # 0.25 TFLOP/s: both compute-bound, 0.032 + 0.016
    assert abs(est([[1000]], 1000, 2000, 0.25, 1.0)["t_kernels_s"] - 0.048) < 1e-15
    # a second expert with 10 rows joins the same two launches (sums inside each max):
    #   gate/up bytes 14e6 + (2e4 + 8e6 + 4e4) = 22.06e6, FLOP 8.08e9; down bytes 10e6 + (4e4 + 4e6 + 2e4)
    #   = 14.06e6, FLOP 4.04e9 -> 0.02206 + 0.01406; intermediates 10e6 + 2*4e4 + 2e4
    o = est([[1000, 10]], 1000, 2000, 1.0, 1.0)
    assert abs(o["t_kernels_s"] - 0.03612) < 1e-15 and o["intermediate_bytes"] == 10.1e6
    # micro-batches add up; an empty expert adds nothing
    o2 = est([[1000, 10], [0, 1000]], 1000, 2000, 1.0, 1.0)
    assert abs(o2["t_kernels_s"] - (0.03612 + 0.024)) < 1e-15 and o2["intermediate_bytes"] == 20.1e6


def test_cost_model_benchmark_floors():
    """The floors quoted for the benchmark shapes: 8x22B prefill 9.896 TFLOP -> 3.958 ms at
    2.5 PFLOP/s; 8x7B decode 2.819 GB of weights -> 352 us at 8 TB/s; 16 micro-batches of 256
    tokens re-read 16 x 4.832 GB -> 9.66 ms."""
    from oracle.cost_model import expert_stage_estimate as est
    o = est([[2048] * 8], 6144, 16384, 2500.0, 8000.0)
    assert abs(o["flops"] / 1e12 - 9.896) < 1e-3 and abs(o["t_stage_s"] * 1e3 - 3.958) < 1e-3
    assert o["memory_bound_instances"] == 0 and 300 < o["ridge_rows"] < 330
    o = est([[64] * 8], 4096, 14336, 2500.0, 8000.0)
    assert abs(o["operand_bytes"] / 1e9 - (2.819 + 8 * 64 * 4096 * 2 / 1e9)) < 1e-3
    assert abs(o["t_stage_s"] * 1e6 - 352.9) < 0.5 and o["memory_bound_instances"] == 8
    o = est([[64] * 8] * 16, 6144, 16384, 2500.0, 8000.0)
    assert abs(o["t_stage_s"] * 1e3 - 16 * (4.832e9 + 8 * 64 * 6144 * 2) / 8e12 * 1e3) < 1e-3
    assert 9.66 < o["t_stage_s"] * 1e3 < 9.69 and o["memory_bound_instances"] == 128


def test_streamed_cost_model_hand_values():
    """Eq. 7 / Eq. 3 by hand. d_h = 512, d_e = 128: one expert's matrices are 6*512*128 =
    393 216 B. Two of four experts moved at 1 GB/s: 786 432 B -> 786.432 us. Rows (100, 0, 50,
    10): inputs 2*160*512 = 163 840 B; with the inputs moved too: 950 272 B -> 950.272 us.
    Computation at 1 TFLOP/s, 1 GB/s device memory: bytes = 3 experts * 393 216 + 163 840 =
    1 343 488 B -> 1343.488 us; FLOPs 6*160*512*128 = 62 914 560 -> 62.9 us: memory side."""
    from oracle import cost_model as cm
    r = cm.streamed_expert_stage_estimate([100, 0, 50, 10], 512, 128, 2, 1.0, 1.0, 1.0)
    assert r["moved_bytes"] == 786432.0
    assert abs(r["t_load_s"] - 786.432e-6) < 1e-12
    assert abs(r["t_comp_s"] - 1343.488e-6) < 1e-12
    assert abs(r["t_sum_s"] - (786.432e-6 + 1343.488e-6)) < 1e-12
    assert abs(r["t_overlap_s"] - 1343.488e-6) < 1e-12
    r = cm.streamed_expert_stage_estimate([100, 0, 50, 10], 512, 128, 2, 1.0, 1.0, 1.0,
                                          inputs_on_device=False)
    assert r["moved_bytes"] == 950272.0 and abs(r["t_load_s"] - 950.272e-6) < 1e-12
    # nothing moved: the load term vanishes and sum == overlap == computation
    r = cm.streamed_expert_stage_estimate([100, 0, 50, 10], 512, 128, 0, 1.0, 1.0, 1.0)
    assert r["t_load_s"] == 0.0 and r["t_sum_s"] == r["t_overlap_s"] == r["t_comp_s"]
    # fast device, slow link: the transfer is the larger term
    r = cm.streamed_expert_stage_estimate([2048] * 8, 6144, 16384, 2, 2500.0, 8000.0, 57.0)
    assert abs(r["t_load_s"] - 2 * 6 * 6144 * 16384 / 57e9) < 1e-9 and r["t_overlap_s"] == r["t_load_s"]

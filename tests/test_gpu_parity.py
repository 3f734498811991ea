"""GPU parity: the HIP library (through its C ABI) against the CPU oracle on the same seeded
inputs. Integer outputs must match bit for bit; floating-point outputs within
rel-L2 <= 1e-2 and max-abs <= 2e-2 * max|y_ref| (bf16 operands, fp32 accumulation)."""
import dataclasses
import json
import os
import sys

import numpy as np
import pytest
import torch

from oracle import ref
from paper_2605_17889_amd import binding as B
from paper_2605_17889_amd import synth

pytestmark = pytest.mark.gpu

GOLD = os.path.join(os.path.dirname(__file__), "golden")
REL_L2_TOL = 1e-2
MAX_ABS_TOL = 2e-2
GATE_TOL = 1e-6


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def dev(a, dtype=None):
    t = torch.as_tensor(a)
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda().contiguous()


def bits(t):
    return synth.bf16_bits(t)


def bf16_to_f64(bits_):
    return (bits_.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def bf16_tensor_from_bits(b):
    return torch.from_numpy(b.view(np.int16)).view(torch.bfloat16)


def assert_close_ffn(got_bf16_bits, want_f64, what):
    got = bf16_to_f64(got_bf16_bits)
    scale = np.abs(want_f64).max()
    if scale == 0:
        assert np.all(got == 0), what
        return 0.0, 0.0
    rel = np.linalg.norm(got - want_f64) / np.linalg.norm(want_f64)
    mx = np.abs(got - want_f64).max() / scale
    say(f"    {what}: rel-L2 {rel:.3e}  max-abs/max|ref| {mx:.3e}")
    assert rel <= REL_L2_TOL, (what, rel)
    assert mx <= MAX_ABS_TOL, (what, mx)
    return rel, mx


def rand_bits(rng, shape, std):
    return bits(torch.tensor(rng.normal(0, std, size=shape), dtype=torch.float32).bfloat16())


# ------------------------------------------------------------------------------- routing
@pytest.mark.parametrize("T,d,E,k,use_bias", [
    (1, 512, 8, 2, False), (3, 512, 8, 2, True), (257, 1024, 8, 2, False), (130, 512, 5, 3, True),
    (64, 512, 16, 4, False), (33, 512, 33, 6, True), (70, 512, 64, 8, True), (19, 1536, 8, 8, False),
    (5, 512, 1, 1, False),
    # more than 64 experts: logits in passes of 64 experts, selection by one wavefront per token
    (70, 2048, 128, 8, True), (33, 512, 65, 3, False), (21, 1024, 200, 10, True),
    (9, 512, 256, 64, False), (130, 512, 129, 1, True),
    # enough 64-token blocks x expert groups of 16 for the matrix-core logits kernel, ragged T
    (2085, 1024, 128, 8, True), (1040, 512, 256, 6, False), (4100, 512, 64, 6, True),
    (8195, 1536, 32, 4, False), (2048, 512, 128, 2, False), (1000, 512, 128, 8, True),
])
def test_route_bit_exact(T, d, E, k, use_bias):
    say(f"route T={T} d={d} E={E} k={k} bias={use_bias}")
    rng = np.random.default_rng(T * 1000 + E)
    x = rand_bits(rng, (T, d), 1.0)
    wr = rng.normal(0, 0.02, size=(d, E)).astype(np.float32)
    bias = rng.normal(0, 0.3, size=E).astype(np.float32) if use_bias else None
    lg_ref = ref.logits(x, wr, bias)
    idx_ref, g_ref = ref.topk(lg_ref, k)

    ctx = B.MoeContext(max(T, 1), d, 256, E, k)
    idx = torch.empty((T, k), dtype=torch.int32, device="cuda")
    g = torch.empty((T, k), dtype=torch.float32, device="cuda")
    lg = torch.empty((T, E), dtype=torch.float32, device="cuda")
    B.moe_route(ctx, dev(bf16_tensor_from_bits(x)), dev(wr), None if bias is None else dev(bias), T,
                idx, g, lg)
    torch.cuda.synchronize()
    assert np.array_equal(lg.cpu().numpy().view(np.uint32), lg_ref.view(np.uint32))   # logits bit-exact
    assert np.array_equal(idx.cpu().numpy(), idx_ref)
    assert np.max(np.abs(g.cpu().numpy() - g_ref)) <= GATE_TOL
    assert np.max(np.abs(g.cpu().numpy().sum(1) - 1)) <= GATE_TOL
    # the same selection from supplied logits
    idx2 = torch.empty_like(idx)
    g2 = torch.empty_like(g)
    B.moe_route_from_logits(ctx, lg, T, idx2, g2)
    torch.cuda.synchronize()
    assert torch.equal(idx2, idx) and torch.equal(g2, g)
    ctx.close()


def test_route_matrix_core_logits_extreme_values():
    """The matrix-core logits kernel (E a multiple of 16, many tokens) must round every
    multiply-add like fmaf, denormal products and sums, signed zeros and wide exponent ranges
    included: the logits are compared bit for bit with the oracle."""
    T, d, E, k = 2085, 512, 128, 4
    rng = np.random.default_rng(77)
    x = rng.normal(0, 1.0, size=(T, d)).astype(np.float32)
    wr = rng.normal(0, 1.0, size=(d, E)).astype(np.float32)
    # rows 0..699: products and sums in the denormal range; 700..1399: exponents spread over
    # 2^-40..2^40 per element (heavy cancellation); the rest ordinary with planted zeros
    x[:700] *= 2.0 ** -70
    x[700:1400] *= np.exp2(rng.integers(-40, 41, size=(700, d))).astype(np.float32)
    x[1400:][rng.random((T - 1400, d)) < 0.2] = 0.0
    x[1400:][rng.random((T - 1400, d)) < 0.05] = -0.0
    wr[:, :64] *= 2.0 ** -70                      # with rows 0..699: products near 2^-140
    wr[rng.random((d, E)) < 0.1] = 0.0
    xb = bits(torch.tensor(x).bfloat16())
    lg_ref = ref.logits(xb, wr, None)
    assert np.any((lg_ref != 0) & (np.abs(lg_ref) < 1.1754944e-38))       # denormal logits present
    ctx = B.MoeContext(T, d, 256, E, k)
    idx = torch.empty((T, k), dtype=torch.int32, device="cuda")
    g = torch.empty((T, k), dtype=torch.float32, device="cuda")
    lg = torch.empty((T, E), dtype=torch.float32, device="cuda")
    B.moe_route(ctx, dev(bf16_tensor_from_bits(xb)), dev(wr), None, T, idx, g, lg)
    torch.cuda.synchronize()
    got = lg.cpu().numpy()
    assert np.array_equal(got.view(np.uint32), lg_ref.view(np.uint32))
    idx_ref, _ = ref.topk(lg_ref, k)
    assert np.array_equal(idx.cpu().numpy(), idx_ref)
    ctx.close()


@pytest.mark.parametrize("T,d,E,k", [
    (2000, 512, 80, 23), (1025, 1536, 160, 56), (3001, 1024, 144, 9), (500, 1536, 256, 3),
    (2000, 1024, 96, 48), (1023, 1024, 65, 48), (500, 1536, 200, 29), (7, 512, 128, 42),
])
def test_route_many_experts_with_duplicate_columns(T, d, E, k):
    """Expert counts that are multiples of 16 but not powers of two (matrix-core logits where the
    batch is large enough), odd counts (vector-unit logits), large k, and router columns that are
    copies of each other, so that every token has exact ties that the selection must break by
    the lower expert index in every lane arrangement."""
    say(f"route with tied experts T={T} d={d} E={E} k={k}")
    rng = np.random.default_rng(T + 7 * E + k)
    x = rand_bits(rng, (T, d), 1.0)
    wr = rng.normal(0, 0.02, size=(d, E)).astype(np.float32)
    src = rng.integers(0, E, size=6)
    dst = rng.integers(0, E, size=6)
    wr[:, dst] = wr[:, src]
    bias = rng.normal(0, 0.3, size=E).astype(np.float32)
    bias[dst] = bias[src]
    lg_ref = ref.logits(x, wr, bias)
    idx_ref, g_ref = ref.topk(lg_ref, k)
    ctx = B.MoeContext(T, d, 256, E, k)
    idx = torch.empty((T, k), dtype=torch.int32, device="cuda")
    g = torch.empty((T, k), dtype=torch.float32, device="cuda")
    lg = torch.empty((T, E), dtype=torch.float32, device="cuda")
    B.moe_route(ctx, dev(bf16_tensor_from_bits(x)), dev(wr), dev(bias), T, idx, g, lg)
    torch.cuda.synchronize()
    assert np.array_equal(lg.cpu().numpy().view(np.uint32), lg_ref.view(np.uint32))
    assert np.array_equal(idx.cpu().numpy(), idx_ref)
    assert np.max(np.abs(g.cpu().numpy() - g_ref)) <= GATE_TOL
    ctx.close()


def test_route_golden_tree_cases_on_gpu():
    cases = json.load(open(os.path.join(GOLD, "route_tree_cases.json")))["cases"]
    hx = lambda s: float.fromhex(s)
    for case in cases:
        say(f"route golden {case['name']}")
        d, E = case["d"], case["E"]
        x = np.zeros((1, d), np.float32)
        for i, v in case["x"].items():
            x[0, int(i)] = hx(v)
        w = np.full((d, E), hx(case["w_default"]), np.float32)
        for key, v in case["w"].items():
            i, e = (int(s) for s in key.split(",")) if "," in key else (int(key), 0)
            w[i, e] = hx(v)
        bias = None if case["bias"] is None else np.array([hx(b) for b in case["bias"]], np.float32)
        ctx = B.MoeContext(1, d, 256, E, 1)
        idx = torch.empty((1, 1), dtype=torch.int32, device="cuda")
        g = torch.empty((1, 1), dtype=torch.float32, device="cuda")
        lg = torch.empty((1, E), dtype=torch.float32, device="cuda")
        B.moe_route(ctx, dev(x, torch.bfloat16), dev(w), None if bias is None else dev(bias), 1, idx, g, lg)
        torch.cuda.synchronize()
        want = np.array([hx(v) for v in case["expected"]], np.float32)
        assert np.array_equal(lg.cpu().numpy()[0].view(np.uint32), want.view(np.uint32)), case["name"]
        ctx.close()


def test_route_from_logits_golden_ties():
    cases = json.load(open(os.path.join(GOLD, "topk_cases.json")))["cases"]
    for case in cases:
        lg = np.array([[float(v) for v in case["logits"]]], np.float32)
        E, k = lg.shape[1], case["k"]
        ctx = B.MoeContext(1, 512, 256, E, k)
        idx = torch.empty((1, k), dtype=torch.int32, device="cuda")
        g = torch.empty((1, k), dtype=torch.float32, device="cuda")
        B.moe_route_from_logits(ctx, dev(lg), 1, idx, g)
        torch.cuda.synchronize()
        assert idx.cpu().numpy()[0].tolist() == case["idx"], case["name"]
        if "gates" in case:
            assert np.allclose(g.cpu().numpy()[0], case["gates"], atol=GATE_TOL)
        ctx.close()


def test_route_from_logits_many_experts_ties_and_order():
    """More than 64 experts (wavefront selection): ties go to the lower index across lanes and
    across the 64-expert words, -0.0 == +0.0, NaN ranks last, slots are in descending order."""
    E, k = 200, 6
    lg = np.full((4, E), -1.0, np.float32)
    lg[0, [199, 70, 6, 134]] = 2.0                       # four equal maxima: 6, 70, 134, 199
    lg[0, 65] = 1.5
    lg[0, 1] = 1.0
    lg[1, :] = 0.0                                       # all equal: experts 0..5
    lg[1, 3] = -0.0
    lg[2, :] = np.nan                                    # NaN everywhere except three
    lg[2, [190, 64, 63]] = [-5.0, -7.0, -6.0]
    lg[3, :] = np.linspace(-3, 3, E).astype(np.float32)  # strictly increasing: 199, 198, ...
    want = [[6, 70, 134, 199, 65, 1], [0, 1, 2, 3, 4, 5], [190, 63, 64, 0, 1, 2],
            [199, 198, 197, 196, 195, 194]]
    ctx = B.MoeContext(4, 512, 256, E, k)
    idx = torch.empty((4, k), dtype=torch.int32, device="cuda")
    g = torch.empty((4, k), dtype=torch.float32, device="cuda")
    B.moe_route_from_logits(ctx, dev(lg), 4, idx, g)
    torch.cuda.synchronize()
    assert idx.cpu().numpy().tolist() == want
    gh = g.cpu().numpy()
    assert np.allclose(gh[1], 1.0 / k, atol=GATE_TOL)
    e = np.exp(np.array([0, 0, 0, 0, -0.5, -1.0]))
    assert np.allclose(gh[0], e / e.sum(), atol=GATE_TOL)
    idx_ref, g_ref = ref.topk(lg[[0, 1, 3]], k)
    assert np.array_equal(idx.cpu().numpy()[[0, 1, 3]], idx_ref)
    assert np.max(np.abs(gh[[0, 1, 3]] - g_ref)) <= GATE_TOL
    ctx.close()


# --------------------------------------------------------------------------- permutation
@pytest.mark.parametrize("T,E,k,seed,empty", [
    (1, 8, 2, 0, False), (37, 8, 2, 1, True), (256, 8, 2, 2, False), (1000, 64, 6, 3, False),
    (4096, 8, 2, 4, True), (777, 3, 3, 5, False), (16384, 8, 2, 6, False), (129, 40, 1, 7, True),
    (5000, 128, 8, 8, True), (333, 65, 2, 9, False), (2000, 256, 6, 10, True), (64, 200, 64, 11, False),
    # around the single-launch limit of 4096 ids, and the multi-launch path at other expert counts
    (4096, 5, 1, 12, False), (4097, 8, 1, 13, False), (1025, 8, 4, 14, True), (3000, 16, 4, 15, False),
    (2100, 33, 2, 16, True), (70000, 17, 1, 17, False),
])
def test_permute_bit_exact(T, E, k, seed, empty):
    say(f"permute T={T} E={E} k={k} empty={empty}")
    rng = np.random.default_rng(seed)
    pool = np.arange(E) if not (empty and E > k) else np.delete(np.arange(E), E // 2)
    idx = np.stack([rng.permutation(pool)[:k] for _ in range(T)]).astype(np.int32)
    d = 512
    x = rand_bits(rng, (T, d), 1.0)
    c_ref, o_ref, p_ref, i_ref = ref.permute(idx, E)
    xp_ref = ref.gather(x, p_ref, k)

    ctx = B.MoeContext(T, d, 256, E, k)
    R = T * k
    counts = torch.empty(E, dtype=torch.int32, device="cuda")
    offsets = torch.empty(E + 1, dtype=torch.int32, device="cuda")
    perm = torch.empty(R, dtype=torch.int32, device="cuda")
    inv = torch.empty(R, dtype=torch.int32, device="cuda")
    xp = torch.empty((R, d), dtype=torch.bfloat16, device="cuda")
    B.moe_permute(ctx, dev(idx), T, counts, offsets, perm, inv, dev(bf16_tensor_from_bits(x)), xp)
    torch.cuda.synchronize()
    assert np.array_equal(counts.cpu().numpy(), c_ref)
    assert np.array_equal(offsets.cpu().numpy(), o_ref)
    assert np.array_equal(perm.cpu().numpy(), p_ref)
    assert np.array_equal(inv.cpu().numpy(), i_ref)
    assert np.array_equal(bits(xp), xp_ref)
    assert int(counts.sum()) == R
    ctx.close()


# ---------------------------------------------------------------- expert FFN and combine
@pytest.mark.parametrize("config", [0, 0 + 128, 0 + 256, 0 + 512, 1, 2, 3, 4, 2 + 16, 3 + 32, 4 + 16, 4 + 32])   # +16 / +32: cached / non-temporal weights
@pytest.mark.parametrize("d,f,rows", [
    (512, 256, [300, 0, 1, 77]),          # empty expert, single row, ragged tails
    (512, 512, [256, 257, 64, 31, 0, 5, 128, 129]),
    (1024, 768, [513, 40]),
])
def test_expert_ffn_parity(config, d, f, rows):
    say(f"expert_ffn config={config} d={d} f={f} rows={rows}")
    rng = np.random.default_rng(d + f + len(rows))
    E = len(rows)
    R = int(sum(rows))
    offsets = np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)
    xp = rand_bits(rng, (R, d), 1.0)
    W1, W3, W2 = rand_bits(rng, (E, f, d), 0.05), rand_bits(rng, (E, f, d), 0.05), rand_bits(rng, (E, d, f), 0.05)
    want = ref.expert_ffn(xp, offsets, W1, W3, W2)

    ctx = B.MoeContext(R, d, f, E, 1)
    B.moe_set_gemm_config(ctx, config)
    try:
        yp = torch.full((R, d), float("nan"), dtype=torch.bfloat16, device="cuda")
        B.moe_expert_ffn(ctx, dev(bf16_tensor_from_bits(xp)), dev(offsets), R,
                         dev(bf16_tensor_from_bits(W1)), dev(bf16_tensor_from_bits(W3)),
                         dev(bf16_tensor_from_bits(W2)), yp)
        torch.cuda.synchronize()
    finally:
        B.moe_set_gemm_config(ctx, -1)
    got = bits(yp)
    assert not np.isnan(bf16_to_f64(got)).any()
    assert_close_ffn(got, want, f"expert_ffn cfg{config}")
    ctx.close()


ALL_TILE_CONFIGS = [0 + 256, 0 + 512, 1, 2, 3, 4]


@pytest.mark.parametrize("config", ALL_TILE_CONFIGS)
def test_expert_ffn_silu_range_and_zero_rows(config):
    """The fused SiLU epilogue far outside the benchmark's value range: tokens scaled by 8 and
    weights of std 0.2 put the gate pre-activation at |a| of 40 to 150, where exp(-a) overflows
    fp32 on the negative side (SiLU -> -0, the true value is below bf16's smallest subnormal)
    and vanishes on the positive side (SiLU -> a). Some rows are exactly zero (zero output
    required) and some are tiny (SiLU(a)*b underflows fp32). All rows, every tile height."""
    d, f, rows = 512, 512, [300, 70, 1, 129]
    say(f"expert_ffn silu range config={config}")
    rng = np.random.default_rng(4242)
    E, R = len(rows), sum(rows)
    offsets = np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)
    xf = rng.normal(0, 8.0, size=(R, d))
    zero_rows = np.array([0, 5, 299, 300, 369, 370, 371, R - 1])
    tiny_rows = np.array([1, 301, 372])
    xf[zero_rows] = 0.0
    xf[tiny_rows] *= 1e-30
    xp = bits(torch.tensor(xf, dtype=torch.float32).bfloat16())
    W1, W3, W2 = rand_bits(rng, (E, f, d), 0.2), rand_bits(rng, (E, f, d), 0.2), rand_bits(rng, (E, d, f), 0.2)
    want, h = ref.expert_ffn(xp, offsets, W1, W3, W2, want_h=True)
    # the case really reaches the range it is meant for
    a = bf16_to_f64(xp[2:3]) @ bf16_to_f64(W1[0]).T
    assert np.abs(a).max() > 89.0 and a.min() < -89.0

    ctx = B.MoeContext(R, d, f, E, 1)
    B.moe_set_gemm_config(ctx, config)
    try:
        yp = torch.full((R, d), float("nan"), dtype=torch.bfloat16, device="cuda")
        B.moe_expert_ffn(ctx, dev(bf16_tensor_from_bits(xp)), dev(offsets), R,
                         dev(bf16_tensor_from_bits(W1)), dev(bf16_tensor_from_bits(W3)),
                         dev(bf16_tensor_from_bits(W2)), yp)
        torch.cuda.synchronize()
    finally:
        B.moe_set_gemm_config(ctx, -1)
    got = bits(yp)
    gf = bf16_to_f64(got)
    assert np.isfinite(gf).all()
    assert np.all(gf[zero_rows] == 0.0), "a zero token must give a zero row"
    big = np.setdiff1d(np.arange(R), np.concatenate([zero_rows, tiny_rows]))
    assert_close_ffn(got[big], want[big], f"silu range cfg{config}")
    # tiny rows: the result is below bf16's normal range; it must stay tiny and finite
    assert np.abs(gf[tiny_rows]).max() <= max(np.abs(want[tiny_rows]).max() * 1.05, 1e-37)
    ctx.close()


def test_expert_ffn_configs_agree_bitwise():
    """Every tile configuration runs the same accumulation chain per output element."""
    rng = np.random.default_rng(123)
    d, f, rows = 512, 512, [200, 3, 0, 130]
    E, R = len(rows), sum(rows)
    offsets = np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)
    xp = dev(bf16_tensor_from_bits(rand_bits(rng, (R, d), 1.0)))
    W1, W3, W2 = (dev(bf16_tensor_from_bits(rand_bits(rng, s, 0.05))) for s in ((E, f, d), (E, f, d), (E, d, f)))
    ctx = B.MoeContext(R, d, f, E, 1)
    outs = []
    try:
        for config in (0, 0 + 128, 0 + 256, 0 + 512, 0 + 512 + 128, 1, 2, 3, 1 + 32, 3 + 16):
            B.moe_set_gemm_config(ctx, config)
            yp = torch.empty((R, d), dtype=torch.bfloat16, device="cuda")
            B.moe_expert_ffn(ctx, xp, dev(offsets), R, W1, W3, W2, yp)
            torch.cuda.synchronize()
            outs.append(bits(yp))
    finally:
        B.moe_set_gemm_config(ctx, -1)
    assert all(np.array_equal(outs[0], o) for o in outs[1:])
    ctx.close()


@pytest.mark.parametrize("T,d,k", [(1, 512, 1), (50, 512, 2), (33, 1024, 3), (256, 4096, 2),
                                   (100, 1024, 17), (7, 512, 64)])   # up to the largest k supported
def test_combine_parity(T, d, k):
    say(f"combine T={T} d={d} k={k}")
    rng = np.random.default_rng(T + d + k)
    yp = rand_bits(rng, (T * k, d), 1.0)
    inv = rng.permutation(T * k).astype(np.int32)
    g = rng.random(size=(T, k)).astype(np.float32)
    want = ref.combine(yp, inv, g)
    ctx = B.MoeContext(T, d, 256, max(k, 2), k)
    y = torch.empty((T, d), dtype=torch.bfloat16, device="cuda")
    B.moe_combine(ctx, dev(bf16_tensor_from_bits(yp)), dev(inv), dev(g), T, y)
    torch.cuda.synchronize()
    got = bf16_to_f64(bits(y))
    # one rounding to bf16 of an fp32 sum of k products: relative error <= 2^-8, plus the fp32
    # sum's own error (k roundings of 2^-24 relative to partial sums no larger than a few times
    # the largest result; allowed here as k * 2^-23 of the largest result)
    fp32_noise = max(1e-6, k * 2.0 ** -23) * np.abs(want).max()
    assert np.all(np.abs(got - want) <= 2.0 ** -8 * np.abs(want) + fp32_noise)
    ctx.close()


# ----------------------------------------------------------------------------- whole layer
def run_layer(cfg, L, T=None, micro=None, ctx=None):
    T = cfg.T if T is None else T
    own = ctx is None
    if own:
        ctx = B.MoeContext(cfg.T, cfg.d_model, cfg.d_ff, cfg.E, cfg.k)
    y = torch.empty((T, cfg.d_model), dtype=torch.bfloat16, device="cuda")
    args = (ctx, L["x"][:T].contiguous(), L["w_router"], L["bias"], L["W1"], L["W3"], L["W2"], T)
    if micro is None:
        B.moe_layer_forward(*args, y)
    else:
        B.moe_layer_forward_microbatched(*args, micro, y)
    torch.cuda.synchronize()
    return y, ctx


def fetch_routing(ctx, T):
    R = T * ctx.k
    out = {"topk_idx": torch.empty((T, ctx.k), dtype=torch.int32, device="cuda"),
           "topk_w": torch.empty((T, ctx.k), dtype=torch.float32, device="cuda"),
           "counts": torch.empty(ctx.E, dtype=torch.int32, device="cuda"),
           "offsets": torch.empty(ctx.E + 1, dtype=torch.int32, device="cuda"),
           "perm": torch.empty(R, dtype=torch.int32, device="cuda"),
           "inv_perm": torch.empty(R, dtype=torch.int32, device="cuda")}
    B.moe_last_routing(ctx, T, **out)
    torch.cuda.synchronize()
    return {n: t.cpu().numpy() for n, t in out.items()}


def host_layer(L):
    return {"x": bits(L["x"]), "w_router": L["w_router"].cpu().numpy(),
            "bias": None if L["bias"] is None else L["bias"].cpu().numpy(),
            "W1": bits(L["W1"]), "W3": bits(L["W3"]), "W2": bits(L["W2"])}


def check_routing_exact(cfg, Hh, routing, T):
    lg = ref.logits(Hh["x"][:T], Hh["w_router"], Hh["bias"])
    idx_ref, g_ref = ref.topk(lg, cfg.k)
    c_ref, o_ref, p_ref, i_ref = ref.permute(idx_ref, cfg.E)
    assert np.array_equal(routing["topk_idx"], idx_ref)
    assert np.max(np.abs(routing["topk_w"] - g_ref)) <= GATE_TOL
    assert np.array_equal(routing["counts"], c_ref) and np.array_equal(routing["offsets"], o_ref)
    assert np.array_equal(routing["perm"], p_ref) and np.array_equal(routing["inv_perm"], i_ref)
    assert int(c_ref.sum()) == T * cfg.k
    return idx_ref, o_ref, p_ref


def sample_tokens(cfg, offsets, perm, per_expert, seed, tile=256, whole_tiles=True):
    """Tokens for the FFN check at full size. One expert (the first with more than one row tile,
    else the largest) contributes EVERY row of its first row tile and EVERY row of its last,
    partial one, so that each wavefront and fragment-row position of a full tile and of a tail
    tile is compared at the real reduction depth; every other non-empty expert contributes the
    first and last row of its group and `per_expert` seeded rows in between."""
    rng = np.random.default_rng(seed)
    sizes = [int(offsets[e + 1] - offsets[e]) for e in range(cfg.E)]
    multi = [e for e in range(cfg.E) if sizes[e] > tile]
    whole = (multi[0] if multi else int(np.argmax(sizes))) if whole_tiles else -1
    rows = []
    for e in range(cfg.E):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi == lo:
            continue
        if e == whole:
            last0 = lo + (hi - lo - 1) // tile * tile
            pick = set(range(lo, min(hi, lo + tile))) | set(range(last0, hi))
        else:
            pick = {lo, hi - 1}
            pick.update(int(v) for v in rng.integers(lo, hi, size=per_expert))
        rows.extend(sorted(pick))
    return np.unique(perm[np.array(rows)] // cfg.k).astype(np.int32)


def test_layer_tiny_all_tokens():
    cfg = synth.PRESETS["tiny"]
    say("layer tiny: all tokens, coalesced + micro-batched")
    L = synth.make_layer(cfg, "cuda")
    Hh = host_layer(L)
    y, ctx = run_layer(cfg, L)
    routing = fetch_routing(ctx, cfg.T)
    check_routing_exact(cfg, Hh, routing, cfg.T)
    want, _, _ = ref.layer_tokens(Hh["x"], Hh["w_router"], None, Hh["W1"], Hh["W3"], Hh["W2"], cfg.k)
    assert_close_ffn(bits(y), want, "tiny layer")
    for m in (64, 100, 1, 256, 1000):
        ym, _ = run_layer(cfg, L, micro=m, ctx=ctx)
        assert torch.equal(ym.view(torch.int16), y.view(torch.int16)), f"micro m={m} differs"
    # determinism: the same call twice gives the same bits
    y2, _ = run_layer(cfg, L, ctx=ctx)
    assert torch.equal(y2.view(torch.int16), y.view(torch.int16))
    ctx.close()


@pytest.mark.parametrize("T", [1, 2, 63, 65, 255])
def test_layer_tiny_ragged_T(T):
    cfg = synth.PRESETS["tiny"]
    say(f"layer tiny T={T}")
    L = synth.make_layer(cfg, "cuda")
    Hh = host_layer(L)
    y, ctx = run_layer(cfg, L, T=T)
    check_routing_exact(cfg, Hh, fetch_routing(ctx, T), T)
    want, _, _ = ref.layer_tokens(Hh["x"], Hh["w_router"], None, Hh["W1"], Hh["W3"], Hh["W2"], cfg.k,
                                  tokens=np.arange(T, dtype=np.int32))
    assert_close_ffn(bits(y), want, f"tiny T={T}")
    ctx.close()


def test_gemm_config_values():
    """The tuning knob belongs to one context and validates its argument."""
    ctx = B.MoeContext(16, 512, 256, 8, 2)
    for bad in (9, 5, 5 + 32, 5 + 64, 5 + 128, 5 + 256, 5 + 512, -2):
        with pytest.raises(B.MoeError):
            B.moe_set_gemm_config(ctx, bad)
    for ok in (0, 3, 4, 4 + 32, 1 + 16, -1 + 32, -1 + 64, 2 + 32 + 64, -1 + 128, 0 + 128 + 64, -1 + 256, -1 + 512, 0 + 512 + 128 + 64, -1):
        B.moe_set_gemm_config(ctx, ok)
    ctx.close()


def test_layer_T0_and_errors():
    cfg = synth.PRESETS["tiny"]
    L = synth.make_layer(cfg, "cuda")
    ctx = B.MoeContext(cfg.T, cfg.d_model, cfg.d_ff, cfg.E, cfg.k)
    y = torch.zeros((1, cfg.d_model), dtype=torch.bfloat16, device="cuda")
    B.moe_layer_forward(ctx, L["x"], L["w_router"], None, L["W1"], L["W3"], L["W2"], 0, y)   # no-op
    with pytest.raises(B.MoeError):
        B.moe_layer_forward(ctx, L["x"], L["w_router"], None, L["W1"], L["W3"], L["W2"], cfg.T + 1, y)
    with pytest.raises(B.MoeError):
        B.moe_layer_forward(ctx, None, L["w_router"], None, L["W1"], L["W3"], L["W2"], 4, y)
    with pytest.raises(B.MoeError):
        B.moe_layer_forward_microbatched(ctx, L["x"], L["w_router"], None, L["W1"], L["W3"], L["W2"], 4, 0, y)
    with pytest.raises(B.MoeError):
        B.MoeContext(16, 500, 1024, 8, 2)
    torch.cuda.synchronize()
    ctx.close()


@pytest.mark.parametrize("T", [16, 64, 256])    # 32-row, 32-row and 128-row tile configurations
def test_layer_mixtral8x7b_decode(T):
    import dataclasses
    cfg = dataclasses.replace(synth.PRESETS["mixtral8x7b_decode"], T=T)
    say(f"layer 8x7B decode T={T}: routing and FFN on all tokens")
    L = synth.make_layer(cfg, "cuda")
    Hh = host_layer(L)
    y, ctx = run_layer(cfg, L)
    routing = fetch_routing(ctx, cfg.T)
    _, o_ref, p_ref = check_routing_exact(cfg, Hh, routing, cfg.T)
    say(f"    rows per expert {routing['counts'].tolist()}")
    want, _, _ = ref.layer_tokens(Hh["x"], Hh["w_router"], None, Hh["W1"], Hh["W3"], Hh["W2"], cfg.k)
    assert_close_ffn(bits(y), want, f"8x7B decode T={T} (all tokens)")
    ctx.close()


@pytest.mark.parametrize("preset", ["qwen3_30b_a3b_prefill", "deepseek_v2_lite_prefill"])
def test_layer_many_small_experts_full_size(preset):
    """The many-expert presets at the size and launch configuration that bench.py times."""
    cfg = synth.PRESETS[preset]
    say(f"layer {preset}: T={cfg.T} E={cfg.E} k={cfg.k}; routing all tokens, FFN on sampled tokens")
    L = synth.make_layer(cfg, "cuda")
    Hh = host_layer(L)
    y, ctx = run_layer(cfg, L)
    routing = fetch_routing(ctx, cfg.T)
    _, o_ref, p_ref = check_routing_exact(cfg, Hh, routing, cfg.T)
    c = routing["counts"]
    say(f"    rows per expert min {int(c.min())} max {int(c.max())}")
    tokens = sample_tokens(cfg, o_ref, p_ref, 1024 // cfg.E, 5)
    want, _, _ = ref.layer_tokens(Hh["x"], Hh["w_router"], None, Hh["W1"], Hh["W3"], Hh["W2"], cfg.k, tokens)
    assert_close_ffn(bits(y)[tokens], want, f"{preset} ({tokens.size} tokens)")
    ctx.close()


def layer_8x22b(cfg, experts):
    (W1, W3, W2), (h1, h3, h2) = experts
    L = {"x": synth.make_tokens(cfg, "cuda"), "w_router": synth.make_router(cfg, "cuda"), "bias": None,
         "W1": W1, "W3": W3, "W2": W2}
    Hh = {"x": bits(L["x"]), "w_router": L["w_router"].cpu().numpy(), "bias": None,
          "W1": h1, "W3": h3, "W2": h2}
    return L, Hh


def test_layer_mixtral8x22b_prefill(experts_8x22b):
    cfg = synth.PRESETS["mixtral8x22b_prefill"]
    say("layer 8x22B prefill T=8192")
    L, Hh = layer_8x22b(cfg, experts_8x22b)
    y, ctx = run_layer(cfg, L)
    routing = fetch_routing(ctx, cfg.T)
    _, o_ref, p_ref = check_routing_exact(cfg, Hh, routing, cfg.T)
    say(f"    rows per expert {routing['counts'].tolist()}")
    tokens = sample_tokens(cfg, o_ref, p_ref, 64, 2)
    want, _, _ = ref.layer_tokens(Hh["x"], Hh["w_router"], None, Hh["W1"], Hh["W3"], Hh["W2"], cfg.k, tokens)
    rel16, _ = assert_close_ffn(bits(y)[tokens], want, f"8x22B prefill ({tokens.size} tokens)")
    B.moe_set_expert_output_fp32(ctx, True)
    y32, _ = run_layer(cfg, L, ctx=ctx)
    rel32, _ = assert_close_ffn(bits(y32)[tokens], want, "8x22B prefill, fp32 expert outputs")
    assert rel32 < rel16, (rel32, rel16)
    ctx.close()


def test_layer_mixtral8x22b_large_batch(experts_8x22b):
    """T = 65536: the intermediate H is 4.3 GB, past 32-bit byte offsets."""
    import dataclasses
    cfg = dataclasses.replace(synth.PRESETS["mixtral8x22b_prefill"], T=65536, seed=12)
    say("layer 8x22B, T=65536 (H beyond 4 GiB)")
    L, Hh = layer_8x22b(cfg, experts_8x22b)
    y, ctx = run_layer(cfg, L)
    routing = fetch_routing(ctx, cfg.T)
    _, o_ref, p_ref = check_routing_exact(cfg, Hh, routing, cfg.T)
    say(f"    rows per expert {routing['counts'].tolist()}")
    tokens = sample_tokens(cfg, o_ref, p_ref, 64, 3)
    want, _, _ = ref.layer_tokens(Hh["x"], Hh["w_router"], None, Hh["W1"], Hh["W3"], Hh["W2"], cfg.k, tokens)
    assert_close_ffn(bits(y)[tokens], want, f"8x22B T=65536 ({tokens.size} tokens)")
    ctx.close()
    del L, y
    torch.cuda.empty_cache()


def test_layer_mixtral8x22b_coalesced_vs_microbatched(experts_8x22b):
    cfg = synth.PRESETS["mixtral8x22b_coalesce"]
    say(f"layer 8x22B T={cfg.T}: coalesced vs {cfg.T // cfg.micro_tokens} micro-batches of {cfg.micro_tokens}")
    L, Hh = layer_8x22b(cfg, experts_8x22b)
    y, ctx = run_layer(cfg, L)
    routing = fetch_routing(ctx, cfg.T)
    _, o_ref, p_ref = check_routing_exact(cfg, Hh, routing, cfg.T)
    ym, _ = run_layer(cfg, L, micro=cfg.micro_tokens, ctx=ctx)
    assert torch.equal(ym.view(torch.int16), y.view(torch.int16)), "micro-batched output differs"
    tokens = sample_tokens(cfg, o_ref, p_ref, 64, 3)
    want, _, _ = ref.layer_tokens(Hh["x"], Hh["w_router"], None, Hh["W1"], Hh["W3"], Hh["W2"], cfg.k, tokens)
    assert_close_ffn(bits(y)[tokens], want, f"8x22B coalesced ({tokens.size} tokens)")
    ctx.close()


@pytest.mark.parametrize("preset", ["tiny", "mixtral8x7b_decode"])
def test_layer_with_materialised_gather_bitwise(preset):
    """The unfused path (gathered rows written to the workspace, taken by itself for batches
    beyond 32-bit row offsets) gives the bits of the fused one."""
    cfg = synth.PRESETS[preset]
    say(f"layer {preset}: gather materialised vs fused into the gate/up loads")
    L = synth.make_layer(cfg, "cuda")
    y_fused, ctx = run_layer(cfg, L)
    B.moe_set_gemm_config(ctx, -1 + 64)
    try:
        y_plain, _ = run_layer(cfg, L, ctx=ctx)
        y_micro, _ = run_layer(cfg, L, micro=100, ctx=ctx)
    finally:
        B.moe_set_gemm_config(ctx, -1)
    assert np.array_equal(bits(y_plain), bits(y_fused))
    assert np.array_equal(bits(y_micro), bits(y_fused))
    ctx.close()


@pytest.mark.parametrize("shape", ["tiny", "many_experts"])
def test_layer_replays_from_a_hip_graph(shape):
    """The layer call only enqueues kernels (no allocation, no memset, no host synchronisation),
    so it can be captured once and replayed: every replay must give the eager result for the
    input that is in the captured buffer at that time. The second shape (64 experts, 2048
    tokens) runs the matrix-core router, the 16-lane selection and the many-expert permutation."""
    cfg = synth.PRESETS["tiny"]
    if shape == "many_experts":
        cfg = dataclasses.replace(cfg, T=2048, d_model=512, d_ff=256, E=64, k=4)
    say(f"layer {shape} captured into a HIP graph, three replays with eager work in between")
    L = synth.make_layer(cfg, "cuda")
    T = cfg.T
    ctx = B.MoeContext(T, cfg.d_model, cfg.d_ff, cfg.E, cfg.k)
    x = L["x"].clone()
    y = torch.empty((T, cfg.d_model), dtype=torch.bfloat16, device="cuda")
    args = (L["w_router"], L["bias"], L["W1"], L["W3"], L["W2"], T)
    B.moe_layer_forward(ctx, x, *args, y)                 # first launches happen outside the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            B.moe_layer_forward(ctx, x, *args, y)
    gen = torch.Generator(device="cuda").manual_seed(77)
    for _ in range(3):
        x.copy_(torch.randn(x.shape, generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16))
        y.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        got = bits(y).copy()
        y_eager = torch.empty_like(y)
        B.moe_layer_forward(ctx, x, *args, y_eager)
        torch.cuda.synchronize()
        assert np.array_equal(got, bits(y_eager))
    del graph
    ctx.close()


def pinned_tail(W, n):
    return W[W.shape[0] - n:].cpu().contiguous().pin_memory()


@pytest.mark.parametrize("n_streamed", [0, 1, 3, 8])
def test_layer_streamed_experts_tiny_bitwise(n_streamed):
    """Experts whose weights arrive from pinned host memory give the bits of the resident call;
    repeated calls reuse the two staging slots."""
    cfg = synth.PRESETS["tiny"]
    say(f"layer tiny, last {n_streamed} experts streamed from host memory")
    L = synth.make_layer(cfg, "cuda")
    Hh = host_layer(L)
    oracle_y, _, _ = ref.layer_tokens(Hh["x"], Hh["w_router"], None, Hh["W1"], Hh["W3"], Hh["W2"], cfg.k)
    y_res, ctx = run_layer(cfg, L)
    E = cfg.E
    host = [pinned_tail(L[n], n_streamed) if n_streamed else None for n in ("W1", "W3", "W2")]
    dev_w = [L[n][:E - n_streamed].contiguous() if n_streamed < E else None for n in ("W1", "W3", "W2")]
    for T in (cfg.T, 100, cfg.T):
        want = y_res if T == cfg.T else run_layer(cfg, L, T=T, ctx=ctx)[0]
        y = torch.full((T, cfg.d_model), float("nan"), dtype=torch.bfloat16, device="cuda")
        B.moe_layer_forward_streamed(ctx, L["x"][:T].contiguous(), L["w_router"], L["bias"], *dev_w, *host,
                                     n_streamed, T, y)
        torch.cuda.synchronize()
        assert np.array_equal(bits(y), bits(want)), f"T={T}"
        assert_close_ffn(bits(y), oracle_y[:T], f"tiny streamed n={n_streamed} T={T} vs oracle")
    ctx.close()


@pytest.mark.parametrize("n_streamed", [1, 3])
def test_layer_streamed_back_to_back_without_host_sync(n_streamed):
    """Three streamed calls enqueued one behind the other with no host synchronisation in
    between, each with its own pinned weight set. The stream is kept busy beforehand so that all
    three calls are enqueued while the first has not started: the copy stream could then run
    ahead of the kernels, and only the wait for a slot's `freed` event (recorded by the previous
    call's last use of that slot) keeps a later call's weights from overwriting the ones an
    earlier call has yet to use. Each output must equal the resident call with that call's weights."""
    import dataclasses
    cfg = synth.PRESETS["tiny"]
    say(f"layer tiny, three streamed calls back to back, last {n_streamed} experts from host memory")
    E, T = cfg.E, cfg.T
    ctx = B.MoeContext(T, cfg.d_model, cfg.d_ff, E, cfg.k)
    base = synth.make_layer(cfg, "cuda")
    sets, want = [], []
    for seed in (0, 21, 22):
        W = synth.make_experts(dataclasses.replace(cfg, seed=seed), "cuda")
        L = dict(base, W1=W[0], W3=W[1], W2=W[2])
        sets.append(L)
        want.append(bits(run_layer(cfg, L, ctx=ctx)[0]).copy())
    assert not np.array_equal(want[0], want[1])
    host = [[pinned_tail(L[n], n_streamed) for n in ("W1", "W3", "W2")] for L in sets]
    devw = [[L[n][:E - n_streamed].contiguous() for n in ("W1", "W3", "W2")] for L in sets]
    ys = [torch.full((T, cfg.d_model), float("nan"), dtype=torch.bfloat16, device="cuda") for _ in sets]
    busy = torch.randn((8192, 8192), device="cuda", dtype=torch.bfloat16)
    torch.cuda.synchronize()
    for _ in range(40):                       # tens of milliseconds of queued work
        busy = (busy @ busy).clamp_(-1, 1)
    for L, h, dw, y in zip(sets, host, devw, ys):
        B.moe_layer_forward_streamed(ctx, L["x"], L["w_router"], None, *dw, *h, n_streamed, T, y)
    torch.cuda.synchronize()
    for i, y in enumerate(ys):
        assert np.array_equal(bits(y), want[i]), f"call {i} used another call's weights"
    ctx.close()


def test_layer_streamed_experts_8x22b_bitwise(experts_8x22b):
    cfg = synth.PRESETS["mixtral8x22b_prefill"]
    say("layer 8x22B prefill, last 2 experts streamed from host memory")
    L, Hh = layer_8x22b(cfg, experts_8x22b)
    y_res, ctx = run_layer(cfg, L)
    routing = fetch_routing(ctx, cfg.T)
    # oracle on rows of every expert, the streamed ones (the last two) included
    tokens = sample_tokens(cfg, routing["offsets"], routing["perm"], 8, 9, whole_tiles=False)
    want, _, _ = ref.layer_tokens(Hh["x"], Hh["w_router"], None, Hh["W1"], Hh["W3"], Hh["W2"], cfg.k, tokens)
    n = 2
    host = [pinned_tail(L[m], n) for m in ("W1", "W3", "W2")]
    dev_w = [L[m][:cfg.E - n] for m in ("W1", "W3", "W2")]
    for _ in range(2):
        y = torch.full((cfg.T, cfg.d_model), float("nan"), dtype=torch.bfloat16, device="cuda")
        B.moe_layer_forward_streamed(ctx, L["x"], L["w_router"], None, *dev_w, *host, n, cfg.T, y)
        torch.cuda.synchronize()
        assert np.array_equal(bits(y), bits(y_res))
        assert_close_ffn(bits(y)[tokens], want, f"8x22B streamed vs oracle ({tokens.size} tokens)")
    ctx.close()


@pytest.mark.parametrize("preset", ["mixtral8x22b_zipf", "mixtral8x22b_zipf_empty"])
def test_layer_mixtral8x22b_zipf(experts_8x22b, preset):
    cfg = synth.PRESETS[preset]
    say(f"layer {preset} T={cfg.T}")
    L, Hh = layer_8x22b(cfg, experts_8x22b)
    base = ref.logits(Hh["x"], Hh["w_router"])

    def count_fn(bias):                       # calibration runs on the oracle's router
        idx, _ = ref.topk(base + bias.numpy()[None, :], cfg.k)
        return np.bincount(idx.reshape(-1), minlength=cfg.E)

    bias = synth.calibrate_expert_bias(cfg, count_fn)
    L["bias"], Hh["bias"] = bias.cuda(), bias.numpy()
    y, ctx = run_layer(cfg, L)
    routing = fetch_routing(ctx, cfg.T)
    _, o_ref, p_ref = check_routing_exact(cfg, Hh, routing, cfg.T)
    counts = routing["counts"]
    say(f"    rows per expert {counts.tolist()}")
    target = synth.zipf_target_counts(cfg).numpy()
    live = target > 0
    assert np.all(np.abs(counts[live] - target[live]) <= 0.02 * target[live])
    assert (counts[~live] == 0).all() and (~live).sum() == (1 if cfg.empty_expert else 0)
    tokens = sample_tokens(cfg, o_ref, p_ref, 64, 4)
    want, _, _ = ref.layer_tokens(Hh["x"], Hh["w_router"], Hh["bias"], Hh["W1"], Hh["W3"], Hh["W2"], cfg.k, tokens)
    assert_close_ffn(bits(y)[tokens], want, f"{preset} ({tokens.size} tokens)")
    ctx.close()


# ------------------------------------------------------- other expert counts and top-k values
@pytest.mark.parametrize("T,d,f,E,k,use_bias", [
    (300, 512, 256, 64, 8, True),      # many small experts, some of them empty
    (257, 1024, 512, 16, 4, False),
    (40, 512, 256, 3, 3, True),        # k = E: every token visits every expert
    (129, 512, 768, 5, 1, False),      # top-1
    (700, 2048, 768, 128, 8, True),    # Qwen3-30B-A3B-shaped: 128 small experts, top-8
    (300, 2048, 1408, 64, 6, False),   # DeepSeek-V2-Lite-shaped: expert dim not a multiple of 256
    (500, 512, 128, 256, 5, True),     # the most experts and the smallest expert dim supported
    (60, 512, 128, 96, 33, True),      # large k: more than two selection slots per lane
    (25, 512, 256, 256, 64, False),    # the largest k and E supported together
])
def test_layer_other_expert_shapes(T, d, f, E, k, use_bias):
    say(f"layer T={T} d={d} f={f} E={E} k={k}")
    cfg = synth.LayerConfig("custom", T, d, f, E, k, seed=900 + E)
    L = synth.make_layer(cfg, "cuda")
    if use_bias:
        g = torch.Generator(device="cpu").manual_seed(E)
        L["bias"] = (torch.randn(E, generator=g) * 1.5).cuda()
    Hh = host_layer(L)
    y, ctx = run_layer(cfg, L)
    routing = fetch_routing(ctx, T)
    check_routing_exact(cfg, Hh, routing, T)
    want, _, _ = ref.layer_tokens(Hh["x"], Hh["w_router"], Hh["bias"], Hh["W1"], Hh["W3"], Hh["W2"], k)
    assert_close_ffn(bits(y), want, f"E={E} k={k}")
    ym, _ = run_layer(cfg, L, micro=37, ctx=ctx)
    assert torch.equal(ym.view(torch.int16), y.view(torch.int16)), "micro-batched output differs"
    ctx.close()


# ---------------------------------------------- expert outputs kept in fp32 until the combine
@pytest.mark.parametrize("T,d,f,E,k", [
    (256, 512, 1024, 8, 2),        # the tiny preset's shape: one short row tile per expert
    (1500, 1024, 2048, 4, 2),      # ~750 rows per expert: full, partial and half-height 256-row tiles
    (300, 2048, 768, 128, 8),      # many small experts
])
def test_layer_fp32_expert_outputs(T, d, f, E, k):
    """moe_set_expert_output_fp32: the down projection stores fp32 and the combine reads it, so
    an output element sees one bf16 rounding fewer. Checked against the oracle on every token
    (closer than the default path), and for the invariances the default path has: micro-batched
    == coalesced, every tile configuration gives the same bits, streamed experts give the same
    bits, and switching the option off restores the default bits."""
    say(f"layer T={T} d={d} f={f} E={E} k={k}: fp32 expert outputs")
    cfg = synth.LayerConfig("custom", T, d, f, E, k, seed=4100 + E)
    L = synth.make_layer(cfg, "cuda")
    Hh = host_layer(L)
    want, _, _ = ref.layer_tokens(Hh["x"], Hh["w_router"], None, Hh["W1"], Hh["W3"], Hh["W2"], k)
    y16, ctx = run_layer(cfg, L)
    rel16, _ = assert_close_ffn(bits(y16), want, "bf16 expert outputs")
    B.moe_set_expert_output_fp32(ctx, True)
    B.moe_set_expert_output_fp32(ctx, True)          # idempotent
    y32, _ = run_layer(cfg, L, ctx=ctx)
    rel32, _ = assert_close_ffn(bits(y32), want, "fp32 expert outputs")
    assert rel32 < rel16, (rel32, rel16)
    for m in (37, 256):
        ym, _ = run_layer(cfg, L, micro=m, ctx=ctx)
        assert torch.equal(ym.view(torch.int16), y32.view(torch.int16)), f"micro m={m} differs"
    if E <= 16:
        # a 37-token micro-batch runs the small tiles, the coalesced call of the middle shape the
        # large ones; force each configuration as well
        for config in ALL_TILE_CONFIGS + [0 + 512 + 128]:
            B.moe_set_gemm_config(ctx, config)
            yc, _ = run_layer(cfg, L, ctx=ctx)
            assert torch.equal(yc.view(torch.int16), y32.view(torch.int16)), f"config {config} differs"
        B.moe_set_gemm_config(ctx, -1)
    n = min(3, E)
    host = [pinned_tail(L[name], n) for name in ("W1", "W3", "W2")]
    dev_w = [L[name][:E - n].contiguous() for name in ("W1", "W3", "W2")]
    ys = torch.full((T, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    B.moe_layer_forward_streamed(ctx, L["x"], L["w_router"], L["bias"], *dev_w, *host, n, T, ys)
    torch.cuda.synchronize()
    assert torch.equal(ys.view(torch.int16), y32.view(torch.int16)), "streamed differs"
    B.moe_set_expert_output_fp32(ctx, False)
    yb, _ = run_layer(cfg, L, ctx=ctx)
    assert torch.equal(yb.view(torch.int16), y16.view(torch.int16)), "default bits not restored"
    ctx.close()


def test_profile_stage_times_of_layer_and_expert_ffn():
    """moe_profile_begin / moe_profile_end: a layer call records all of its stages, a standalone
    moe_expert_ffn call its two GEMM stages; launches and calls are counted; the outputs are the
    bits of an unprofiled call."""
    cfg = synth.PRESETS["tiny"]
    say("stage profiling: layer call and moe_expert_ffn")
    L = synth.make_layer(cfg, "cuda")
    y_plain, ctx = run_layer(cfg, L)
    B.moe_profile_begin(ctx, 3)
    for _ in range(3):
        y_prof, _ = run_layer(cfg, L, ctx=ctx)
    stage_ms, launches, calls = B.moe_profile_end(ctx)
    assert calls == 3
    assert torch.equal(y_prof.view(torch.int16), y_plain.view(torch.int16))
    for name in ("route", "permute", "gateup", "down", "combine"):
        assert stage_ms[name] > 0 and launches[name] >= 3, (name, stage_ms, launches)
    assert stage_ms["gather"] == 0 and launches["gather"] == 0     # fused into the gate/up loads
    routing = fetch_routing(ctx, cfg.T)
    R = cfg.T * cfg.k
    xp = torch.empty((R, cfg.d_model), dtype=torch.bfloat16, device="cuda")
    scratch = {n: torch.empty_like(torch.as_tensor(routing[n]).cuda()) for n in ("counts", "offsets", "perm", "inv_perm")}
    B.moe_permute(ctx, torch.as_tensor(routing["topk_idx"]).cuda(), cfg.T, scratch["counts"], scratch["offsets"],
                  scratch["perm"], scratch["inv_perm"], L["x"], xp)
    yp = torch.empty((R, cfg.d_model), dtype=torch.bfloat16, device="cuda")
    B.moe_profile_begin(ctx, 2)
    for _ in range(2):
        B.moe_expert_ffn(ctx, xp, scratch["offsets"], R, L["W1"], L["W3"], L["W2"], yp)
    torch.cuda.synchronize()
    stage_ms, launches, calls = B.moe_profile_end(ctx)
    assert calls == 2 and launches["gateup"] == 2 and launches["down"] == 2
    assert stage_ms["gateup"] > 0 and stage_ms["down"] > 0
    assert all(stage_ms[n] == 0 for n in ("route", "permute", "gather", "combine"))
    # the same per call: every call has every stage, and the cells add up to the totals' scale
    B.moe_profile_begin(ctx, 4)
    for _ in range(4):
        run_layer(cfg, L, ctx=ctx, micro=100)
    per_call, launches4, calls4 = B.moe_profile_end_per_call(ctx, 3)      # room for 3 of the 4 calls
    assert calls4 == 4 and len(per_call) == 3
    for c in per_call:
        assert all(c[n] > 0 for n in ("route", "permute", "gateup", "down", "combine")) and c["gather"] == 0
    assert launches4["gateup"] == 4 * 3                              # 3 micro-batches of <= 100 tokens per call
    ctx.close()


def test_permute_drops_out_of_range_experts():
    """An expert index outside [0, E) is dropped from every group: inv_perm = -1, counts and
    offsets only cover the valid ids, and the remaining ids keep their stable order."""
    T, E, k, d = 50, 4, 2, 512
    rng = np.random.default_rng(77)
    idx = rng.integers(0, E, size=(T, k)).astype(np.int32)
    bad = [(3, 0), (17, 1), (49, 0)]
    for t, s in bad:
        idx[t, s] = E + 5 if (t + s) % 2 else -1
    flat = idx.reshape(-1)
    valid = (flat >= 0) & (flat < E)
    ids = np.nonzero(valid)[0]
    order = ids[np.argsort(flat[ids], kind="stable")]
    ctx = B.MoeContext(T, d, 256, E, k)
    R = T * k
    counts = torch.empty(E, dtype=torch.int32, device="cuda")
    offsets = torch.empty(E + 1, dtype=torch.int32, device="cuda")
    perm = torch.full((R,), -7, dtype=torch.int32, device="cuda")
    inv = torch.empty(R, dtype=torch.int32, device="cuda")
    x = torch.ones((T, d), dtype=torch.bfloat16, device="cuda")
    xp = torch.full((R, d), 3.0, dtype=torch.bfloat16, device="cuda")
    B.moe_permute(ctx, dev(idx), T, counts, offsets, perm, inv, x, xp)
    torch.cuda.synchronize()
    assert np.array_equal(counts.cpu().numpy(), np.bincount(flat[valid], minlength=E))
    assert int(offsets.cpu().numpy()[-1]) == len(ids)
    assert np.array_equal(perm.cpu().numpy()[:len(ids)], order)
    inv_h = inv.cpu().numpy()
    assert np.all(inv_h[~valid] == -1)
    assert np.array_equal(inv_h[order], np.arange(len(ids)))
    xp_h = xp.float().cpu().numpy()
    assert np.all(xp_h[:len(ids)] == 1.0) and np.all(xp_h[len(ids):] == 0.0)
    ctx.close()

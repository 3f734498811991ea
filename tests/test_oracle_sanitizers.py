"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): a small
driver (tests/oracle_sanitize_driver.c) is compiled together with oracle/moe_oracle.c with
-fsanitize=address,undefined and no recovery, fed the hand-derived pins and small random layers
through exactly-sized heap buffers, and its printed results are compared with the pins (and, for
the random layers, with the ordinary build of the oracle). Any out-of-bounds access, signed
overflow or invalid shift inside the oracle ends the driver with a non-zero status."""
import json
import os
import subprocess

import numpy as np
import pytest
import torch

from oracle import ref
from paper_2605_17889_amd import synth

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
GOLD = os.path.join(HERE, "golden")


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    out = tmp_path_factory.mktemp("asan") / "oracle_sanitized"
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-ffp-contract=off", "-fopenmp", "-march=x86-64-v3",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
           os.path.join(HERE, "oracle_sanitize_driver.c"), os.path.join(ROOT, "oracle", "moe_oracle.c"),
           "-o", str(out), "-lm"]
    subprocess.run(cmd, check=True)
    return str(out)


def run(driver, tmp_path, text):
    path = tmp_path / "case.txt"
    path.write_text(text)
    env = dict(os.environ, OMP_NUM_THREADS="2",
               ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    proc = subprocess.run([driver, str(path)], capture_output=True, text=True, env=env, timeout=300)
    assert proc.returncode == 0, proc.stderr[-4000:]
    out = {}
    for line in proc.stdout.splitlines():
        name, *vals = line.split()
        out[name] = vals
    assert out["rc"] == ["0"]
    return out


def floats(vals):
    return np.array([float.fromhex(v) if "0x" in v else float(v) for v in vals])


def fmt(a):
    return " ".join(str(v) for v in np.asarray(a).reshape(-1).tolist())


def test_topk_pins_under_sanitizers(driver, tmp_path):
    for case in json.load(open(os.path.join(GOLD, "topk_cases.json")))["cases"]:
        lg = [str(v) for v in case["logits"]]
        out = run(driver, tmp_path, f"topk 1 {len(lg)} {case['k']} " + " ".join(lg))
        assert [int(v) for v in out["idx"]] == case["idx"], case["name"]
        if "gates" in case:
            assert np.allclose(floats(out["gates"]), case["gates"], atol=1e-6)


def test_permute_pin_and_edges_under_sanitizers(driver, tmp_path):
    ex = json.load(open(os.path.join(GOLD, "permute_worked_example.json")))
    flat = np.array(ex["topk_idx"]).reshape(-1)
    out = run(driver, tmp_path, f"permute {flat.size} {ex['E']} {fmt(flat)}")
    for name in ("counts", "offsets", "perm", "inv_perm"):
        assert [int(v) for v in out[name]] == ex[name], name
    # no ids at all; one expert; the last expert only
    out = run(driver, tmp_path, "permute 0 4")
    assert [int(v) for v in out["offsets"]] == [0] * 5 and out["perm"] == []
    out = run(driver, tmp_path, "permute 5 1 0 0 0 0 0")
    assert [int(v) for v in out["perm"]] == [0, 1, 2, 3, 4]
    out = run(driver, tmp_path, "permute 3 7 6 6 6")
    assert [int(v) for v in out["offsets"]] == [0, 0, 0, 0, 0, 0, 0, 3]
    # a larger seeded case against numpy's stable sort
    rng = np.random.default_rng(3)
    idx = rng.integers(0, 13, size=1000)
    out = run(driver, tmp_path, f"permute {idx.size} 13 {fmt(idx)}")
    assert [int(v) for v in out["perm"]] == np.argsort(idx, kind="stable").tolist()


def test_ffn_worked_example_under_sanitizers(driver, tmp_path):
    ex = json.load(open(os.path.join(GOLD, "ffn_worked_example.json")))
    b = lambda a: synth.bf16_bits(torch.tensor(a, dtype=torch.float32).bfloat16())
    text = f"ffn 1 2 2 1 0 1 {fmt(b(ex['x']))} {fmt(b(ex['W1']))} {fmt(b(ex['W3']))} {fmt(b(ex['W2']))}"
    out = run(driver, tmp_path, text)
    assert np.allclose(floats(out["y_perm"]), ex["o"], rtol=1e-15)


def test_logits_tree_pins_under_sanitizers(driver, tmp_path):
    hx = float.fromhex
    for case in json.load(open(os.path.join(GOLD, "route_tree_cases.json")))["cases"]:
        d, E = case["d"], case["E"]
        x = np.zeros((1, d), np.float32)
        for i, v in case["x"].items():
            x[0, int(i)] = hx(v)
        w = np.full((d, E), hx(case["w_default"]), np.float32)
        for key, v in case["w"].items():
            i, e = (int(s) for s in key.split(",")) if "," in key else (int(key), 0)
            w[i, e] = hx(v)
        xb = synth.bf16_bits(torch.from_numpy(x).bfloat16())
        ws = " ".join(float(v).hex() for v in w.reshape(-1))
        bias = case["bias"]
        text = f"logits 1 {d} {E} {0 if bias is None else 1} {fmt(xb)} {ws}"
        if bias is not None:
            text += " " + " ".join(bias)
        out = run(driver, tmp_path, text)
        want = np.array([hx(v) for v in case["expected"]], np.float32)
        got = floats(out["logits"]).astype(np.float32)
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), case["name"]


@pytest.mark.parametrize("T,f,E,k,m", [(37, 96, 5, 2, 7), (16, 64, 3, 3, 100), (9, 32, 8, 1, 1)])
def test_layer_under_sanitizers(driver, tmp_path, T, f, E, k, m):
    """The whole layer (definition on a token subset; stage form on micro-batches of m, the
    last one short) through the sanitized build: equal to the ordinary build, and coalesced
    equal to micro-batched."""
    d = 512
    rng = np.random.default_rng(T + E)
    b = lambda a: synth.bf16_bits(torch.tensor(a, dtype=torch.float32).bfloat16())
    x = b(rng.normal(0, 1, (T, d)))
    w = rng.normal(0, 0.02, (d, E)).astype(np.float32)
    W1, W3, W2 = b(rng.normal(0, 0.05, (E, f, d))), b(rng.normal(0, 0.05, (E, f, d))), b(rng.normal(0, 0.05, (E, d, f)))
    tokens = np.array(sorted(rng.choice(T, size=min(T, 5), replace=False)), np.int32)
    ws = " ".join(float(v).hex() for v in w.reshape(-1))
    text = (f"layer {T} {d} {f} {E} {k} {m} {tokens.size} {fmt(tokens)} {fmt(x)} {ws} "
            f"{fmt(W1)} {fmt(W3)} {fmt(W2)}")
    out = run(driver, tmp_path, text)
    want, idx, _ = ref.layer_tokens(x, w, None, W1, W3, W2, k)
    assert [int(v) for v in out["idx"]] == idx[tokens].reshape(-1).tolist()
    y_tok = floats(out["y_tokens"]).reshape(tokens.size, d)
    y_stg = floats(out["y_staged"]).reshape(T, d)
    scale = np.abs(want).max()
    assert np.abs(y_tok - want[tokens]).max() <= 1e-12 * scale
    assert np.abs(y_stg - want).max() <= 1e-12 * scale

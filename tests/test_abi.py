"""CPU-only checks of the C-ABI library: it loads, exports every symbol that include/moe.h
declares, and its host-only entry points behave. No kernel is launched here."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "moe.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2605_17889_amd import build
    if not os.path.exists(build.LIB):
        build.build()
    L = C.CDLL(build.LIB)
    L.moe_status_string.restype = C.c_char_p
    L.moe_workspace_bytes.restype = C.c_size_t
    return L


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_required_entry_points():
    names = declared_symbols()
    for need in ("moe_route", "moe_permute", "moe_expert_ffn", "moe_combine", "moe_layer_forward",
                 "moe_layer_forward_microbatched"):
        assert need in names


def test_every_declared_symbol_is_exported(lib):
    for name in declared_symbols():
        assert hasattr(lib, name), f"{name} declared in moe.h but not exported by libmoe.so"


def test_binding_covers_every_declared_symbol():
    from paper_2605_17889_amd import binding
    assert sorted(binding.EXPORTS) == declared_symbols()


def test_status_strings(lib):
    assert lib.moe_status_string(0) == b"MOE_OK"
    assert lib.moe_status_string(-1) == b"MOE_ERR_INVALID_ARG"
    assert lib.moe_status_string(-2) == b"MOE_ERR_UNSUPPORTED_SHAPE"
    assert lib.moe_status_string(-3) == b"MOE_ERR_WORKSPACE"
    assert lib.moe_status_string(-4) == b"MOE_ERR_HIP"
    assert lib.moe_status_string(77) == b"MOE_ERR_UNKNOWN"


def test_workspace_bytes_and_shape_rules(lib):
    from paper_2605_17889_amd.binding import MoeShape
    ok = MoeShape(8192, 6144, 16384, 8, 2)
    n = lib.moe_workspace_bytes(C.byref(ok))
    R = 8192 * 2
    assert n >= R * (6144 * 2 * 2 + 16384 * 2)            # x_perm + y_perm + H
    assert n < R * (6144 * 2 * 2 + 16384 * 2) + (8 << 20)
    for bad in (MoeShape(16, 500, 1024, 8, 2),             # d_model % 512
                MoeShape(16, 512, 1000, 8, 2),             # d_ff % 128
                MoeShape(16, 512, 1024, 257, 2),           # E > 256
                MoeShape(16, 512, 1024, 128, 65),          # k > 64
                MoeShape(16, 512, 1024, 4, 5),             # k > E
                MoeShape(16, 512, 1024, 8, 0),             # k < 1
                MoeShape(-1, 512, 1024, 8, 2),
                MoeShape(1 << 30, 512, 1024, 8, 2)):       # T_max*k >= 2^31
        assert lib.moe_workspace_bytes(C.byref(bad)) == 0
    assert lib.moe_workspace_bytes(None) == 0
    for good in (MoeShape(16, 2048, 768, 128, 8), MoeShape(16, 2048, 1408, 64, 6),
                 MoeShape(16, 512, 128, 256, 64)):
        assert lib.moe_workspace_bytes(C.byref(good)) > 0


def test_null_arguments_are_rejected_before_any_gpu_work(lib):
    assert lib.moe_create(None, None, 0) == -1
    assert lib.moe_destroy(None) == -1
    assert lib.moe_layer_forward(None, None, None, None, None, None, None, 4, None, None) == -1
    assert lib.moe_layer_forward_streamed(None, None, None, None, None, None, None, None, None, None,
                                          1, 4, None, None) == -1
    assert lib.moe_set_gemm_config(None, 0) == -1
    assert lib.moe_permute_static(None, -1, 2, 8, None, None, None, None, None) == -1
    assert lib.moe_permute_static(None, 4, 3, 2, None, None, None, None, None) == -1


def test_binding_fails_loudly_without_gpu():
    import torch
    from paper_2605_17889_amd import binding
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(binding.MoeError):
        binding.MoeContext(16, 512, 1024, 8, 2)

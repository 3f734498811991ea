"""ctypes binding of libmoe.so: argument marshalling only.

Functions carry the C-ABI names of include/moe.h and take torch tensors that already live on
the GPU (torch is used for device memory and streams, nothing else). Every step of the layer
runs in the library's HIP kernels; there is no CPU or torch fallback: a missing library or
GPU raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch  # imported before the library so that both share one HIP runtime

from . import build as _build

MOE_OK = 0
STAGES = ("route", "permute", "gather", "gateup", "down", "combine")

EXPORTS = (
    "moe_create", "moe_destroy", "moe_workspace_bytes", "moe_status_string", "moe_route",
    "moe_route_from_logits", "moe_permute", "moe_expert_ffn", "moe_combine", "moe_layer_forward",
    "moe_layer_forward_microbatched", "moe_last_routing", "moe_profile_begin", "moe_profile_end",
    "moe_set_gemm_config", "moe_estimate_expert_stage", "moe_layer_forward_streamed",
    "moe_estimate_streamed_stage", "moe_permute_static", "moe_set_expert_output_fp32",
    "moe_profile_end_per_call",
)


class MoeShape(C.Structure):
    _fields_ = [("T_max", C.c_int32), ("d_model", C.c_int32), ("d_ff", C.c_int32),
                ("E", C.c_int32), ("k", C.c_int32)]


class MoeMachine(C.Structure):
    _fields_ = [("tflops", C.c_double), ("gbytes_per_s", C.c_double)]


class MoeExpertEstimate(C.Structure):
    _fields_ = [("micro_batches", C.c_int32), ("expert_instances", C.c_int32),
                ("memory_bound_instances", C.c_int32), ("flops", C.c_double),
                ("operand_bytes", C.c_double), ("intermediate_bytes", C.c_double),
                ("t_stage_s", C.c_double), ("t_per_expert_s", C.c_double),
                ("t_kernels_s", C.c_double), ("ridge_rows", C.c_double)]


class MoeStreamedEstimate(C.Structure):
    _fields_ = [("moved_bytes", C.c_double), ("t_load_s", C.c_double), ("t_comp_s", C.c_double),
                ("t_sum_s", C.c_double), ("t_overlap_s", C.c_double)]


class MoeError(RuntimeError):
    pass


_lib = None


def library_path() -> str:
    return _build.LIB


def lib():
    """Load libmoe.so (built in-tree by build.py); fail loudly if it is not there."""
    global _lib
    if _lib is None:
        path = library_path()
        if not os.path.exists(path):
            raise MoeError(f"{path} is missing: run `python -m paper_2605_17889_amd.build` "
                           "(there is no fallback implementation)")
        L = C.CDLL(path)
        for name in EXPORTS:
            getattr(L, name).restype = C.c_int
        L.moe_workspace_bytes.restype = C.c_size_t
        L.moe_status_string.restype = C.c_char_p
        _lib = L
    return _lib


def status_string(rc: int) -> str:
    return lib().moe_status_string(C.c_int(rc)).decode()


def _check(rc: int, what: str) -> None:
    if rc != MOE_OK:
        raise MoeError(f"{what}: {status_string(rc)} ({rc})")


def _ptr(t: Optional[torch.Tensor], dtype: torch.dtype, what: str):
    if t is None:
        return C.c_void_p(0)
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise MoeError(f"{what}: expected a contiguous cuda tensor of {dtype}, got "
                       f"{t.dtype} on {t.device}, contiguous={t.is_contiguous()}")
    return C.c_void_p(t.data_ptr())


def _stream(stream) -> C.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


class MoeContext:
    """Owns a moe_ctx*. Shapes: see include/moe.h."""

    def __init__(self, T_max: int, d_model: int, d_ff: int, E: int, k: int, device: int = 0):
        if not torch.cuda.is_available():
            raise MoeError("no GPU: libmoe has no CPU path")
        self.shape = MoeShape(T_max, d_model, d_ff, E, k)
        self.device = device
        self._h = C.c_void_p(0)
        _check(lib().moe_create(C.byref(self._h), C.byref(self.shape), C.c_int(device)), "moe_create")

    def close(self) -> None:
        if self._h:
            torch.cuda.synchronize(self.device)
            lib().moe_destroy(self._h)
            self._h = C.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- shorthand
    @property
    def T_max(self): return self.shape.T_max
    @property
    def d_model(self): return self.shape.d_model
    @property
    def d_ff(self): return self.shape.d_ff
    @property
    def E(self): return self.shape.E
    @property
    def k(self): return self.shape.k


def workspace_bytes(T_max, d_model, d_ff, E, k) -> int:
    return lib().moe_workspace_bytes(C.byref(MoeShape(T_max, d_model, d_ff, E, k)))


def moe_route(ctx: MoeContext, x, w_router, bias, T, topk_idx, topk_w, logits_out=None, stream=None):
    _check(lib().moe_route(ctx._h, _ptr(x, torch.bfloat16, "x"), _ptr(w_router, torch.float32, "w_router"),
                           _ptr(bias, torch.float32, "bias"), C.c_int32(T),
                           _ptr(topk_idx, torch.int32, "topk_idx"), _ptr(topk_w, torch.float32, "topk_w"),
                           _ptr(logits_out, torch.float32, "logits_out"), _stream(stream)), "moe_route")


def moe_route_from_logits(ctx: MoeContext, logits, T, topk_idx, topk_w, stream=None):
    _check(lib().moe_route_from_logits(ctx._h, _ptr(logits, torch.float32, "logits"), C.c_int32(T),
                                       _ptr(topk_idx, torch.int32, "topk_idx"),
                                       _ptr(topk_w, torch.float32, "topk_w"), _stream(stream)),
           "moe_route_from_logits")


def moe_permute(ctx: MoeContext, topk_idx, T, counts, offsets, perm, inv_perm, x=None, x_perm=None,
                stream=None):
    _check(lib().moe_permute(ctx._h, _ptr(topk_idx, torch.int32, "topk_idx"), C.c_int32(T),
                             _ptr(counts, torch.int32, "counts"), _ptr(offsets, torch.int32, "offsets"),
                             _ptr(perm, torch.int32, "perm"), _ptr(inv_perm, torch.int32, "inv_perm"),
                             _ptr(x, torch.bfloat16, "x"), _ptr(x_perm, torch.bfloat16, "x_perm"),
                             _stream(stream)), "moe_permute")


def moe_permute_static(topk_idx, T, k, E, counts, offsets, perm, inv_perm, stream=None):
    """The grouping of moe_permute without a context and without any allocation."""
    _check(lib().moe_permute_static(_ptr(topk_idx, torch.int32, "topk_idx"), C.c_int32(T), C.c_int32(k),
                                    C.c_int32(E), _ptr(counts, torch.int32, "counts"),
                                    _ptr(offsets, torch.int32, "offsets"), _ptr(perm, torch.int32, "perm"),
                                    _ptr(inv_perm, torch.int32, "inv_perm"), _stream(stream)),
           "moe_permute_static")


def moe_expert_ffn(ctx: MoeContext, x_perm, offsets, R, W1, W3, W2, y_perm, stream=None):
    _check(lib().moe_expert_ffn(ctx._h, _ptr(x_perm, torch.bfloat16, "x_perm"),
                                _ptr(offsets, torch.int32, "offsets"), C.c_int32(R),
                                _ptr(W1, torch.bfloat16, "W1"), _ptr(W3, torch.bfloat16, "W3"),
                                _ptr(W2, torch.bfloat16, "W2"), _ptr(y_perm, torch.bfloat16, "y_perm"),
                                _stream(stream)), "moe_expert_ffn")


def moe_combine(ctx: MoeContext, y_perm, inv_perm, topk_w, T, y, stream=None):
    _check(lib().moe_combine(ctx._h, _ptr(y_perm, torch.bfloat16, "y_perm"),
                             _ptr(inv_perm, torch.int32, "inv_perm"), _ptr(topk_w, torch.float32, "topk_w"),
                             C.c_int32(T), _ptr(y, torch.bfloat16, "y"), _stream(stream)), "moe_combine")


def moe_layer_forward(ctx: MoeContext, x, w_router, bias, W1, W3, W2, T, y, stream=None):
    _check(lib().moe_layer_forward(ctx._h, _ptr(x, torch.bfloat16, "x"),
                                   _ptr(w_router, torch.float32, "w_router"),
                                   _ptr(bias, torch.float32, "bias"), _ptr(W1, torch.bfloat16, "W1"),
                                   _ptr(W3, torch.bfloat16, "W3"), _ptr(W2, torch.bfloat16, "W2"),
                                   C.c_int32(T), _ptr(y, torch.bfloat16, "y"), _stream(stream)),
           "moe_layer_forward")


def moe_layer_forward_microbatched(ctx: MoeContext, x, w_router, bias, W1, W3, W2, T, micro_tokens, y,
                                   stream=None):
    _check(lib().moe_layer_forward_microbatched(
        ctx._h, _ptr(x, torch.bfloat16, "x"), _ptr(w_router, torch.float32, "w_router"),
        _ptr(bias, torch.float32, "bias"), _ptr(W1, torch.bfloat16, "W1"), _ptr(W3, torch.bfloat16, "W3"),
        _ptr(W2, torch.bfloat16, "W2"), C.c_int32(T), C.c_int32(micro_tokens),
        _ptr(y, torch.bfloat16, "y"), _stream(stream)), "moe_layer_forward_microbatched")


def _host_ptr(t: torch.Tensor, dtype: torch.dtype, what: str):
    if t.is_cuda or t.dtype != dtype or not t.is_contiguous() or not t.is_pinned():
        raise MoeError(f"{what}: expected a contiguous pinned host tensor of {dtype}")
    return C.c_void_p(t.data_ptr())


def moe_layer_forward_streamed(ctx: MoeContext, x, w_router, bias, W1, W3, W2, W1_host, W3_host,
                               W2_host, n_streamed, T, y, stream=None):
    """Last n_streamed experts' weights in pinned host tensors; the others (device) may be None
    when every expert is streamed."""
    hp = (lambda t, n: C.c_void_p(0)) if n_streamed == 0 else (lambda t, n: _host_ptr(t, torch.bfloat16, n))
    _check(lib().moe_layer_forward_streamed(
        ctx._h, _ptr(x, torch.bfloat16, "x"), _ptr(w_router, torch.float32, "w_router"),
        _ptr(bias, torch.float32, "bias"), _ptr(W1, torch.bfloat16, "W1"), _ptr(W3, torch.bfloat16, "W3"),
        _ptr(W2, torch.bfloat16, "W2"), hp(W1_host, "W1_host"), hp(W3_host, "W3_host"),
        hp(W2_host, "W2_host"), C.c_int32(n_streamed), C.c_int32(T), _ptr(y, torch.bfloat16, "y"),
        _stream(stream)), "moe_layer_forward_streamed")


def moe_last_routing(ctx: MoeContext, T, topk_idx=None, topk_w=None, counts=None, offsets=None,
                     perm=None, inv_perm=None, stream=None):
    _check(lib().moe_last_routing(ctx._h, C.c_int32(T), _ptr(topk_idx, torch.int32, "topk_idx"),
                                  _ptr(topk_w, torch.float32, "topk_w"), _ptr(counts, torch.int32, "counts"),
                                  _ptr(offsets, torch.int32, "offsets"), _ptr(perm, torch.int32, "perm"),
                                  _ptr(inv_perm, torch.int32, "inv_perm"), _stream(stream)),
           "moe_last_routing")


def moe_profile_begin(ctx: MoeContext, max_calls: int):
    _check(lib().moe_profile_begin(ctx._h, C.c_int32(max_calls)), "moe_profile_begin")


def moe_profile_end(ctx: MoeContext):
    """-> (dict stage -> total ms, dict stage -> launches, calls)."""
    ms = (C.c_double * len(STAGES))()
    launches = (C.c_int64 * len(STAGES))()
    calls = C.c_int32(0)
    _check(lib().moe_profile_end(ctx._h, ms, launches, C.byref(calls)), "moe_profile_end")
    return ({s: ms[i] for i, s in enumerate(STAGES)},
            {s: launches[i] for i, s in enumerate(STAGES)}, calls.value)


def moe_profile_end_per_call(ctx: MoeContext, capacity_calls: int):
    """-> (list over calls of dict stage -> ms, dict stage -> launches, calls)."""
    n = len(STAGES)
    ms = (C.c_double * (n * capacity_calls))()
    launches = (C.c_int64 * n)()
    calls = C.c_int32(0)
    _check(lib().moe_profile_end_per_call(ctx._h, ms, C.c_int32(capacity_calls), launches,
                                          C.byref(calls)), "moe_profile_end_per_call")
    got = min(calls.value, capacity_calls)
    return ([{s: ms[c * n + i] for i, s in enumerate(STAGES)} for c in range(got)],
            {s: launches[i] for i, s in enumerate(STAGES)}, calls.value)


def moe_estimate_expert_stage(d_model: int, d_ff: int, rows, tflops: float, gbytes_per_s: float) -> dict:
    """rows: host sequence [micro_batches][E] of routed row counts. Host arithmetic only."""
    micro_batches = len(rows)
    E = len(rows[0]) if micro_batches else 1
    flat = (C.c_int32 * max(1, micro_batches * E))(*[int(v) for mb in rows for v in mb])
    shape = MoeShape(0, d_model, d_ff, E, 1)
    machine = MoeMachine(tflops, gbytes_per_s)
    out = MoeExpertEstimate()
    _check(lib().moe_estimate_expert_stage(C.byref(shape), flat, C.c_int32(micro_batches),
                                           C.byref(machine), C.byref(out)),
           "moe_estimate_expert_stage")
    return {name: getattr(out, name) for name, _ in MoeExpertEstimate._fields_}


def moe_estimate_streamed_stage(d_model: int, d_ff: int, rows, n_moved: int, tflops: float,
                                gbytes_per_s: float, pcie_gbytes_per_s: float,
                                inputs_on_device: bool = True) -> dict:
    """rows: host sequence [E] of routed row counts of one coalesced batch. Host arithmetic only."""
    E = len(rows)
    flat = (C.c_int32 * max(1, E))(*[int(v) for v in rows])
    shape = MoeShape(0, d_model, d_ff, max(E, 1), 1)
    mach = MoeMachine(tflops, gbytes_per_s)
    out = MoeStreamedEstimate()
    _check(lib().moe_estimate_streamed_stage(C.byref(shape), flat, C.c_int32(n_moved), C.byref(mach),
                                             C.c_double(pcie_gbytes_per_s),
                                             C.c_int32(1 if inputs_on_device else 0), C.byref(out)),
           "moe_estimate_streamed_stage")
    return {n: getattr(out, n) for n, _ in MoeStreamedEstimate._fields_}


def moe_set_gemm_config(ctx: MoeContext, config: int):
    _check(lib().moe_set_gemm_config(ctx._h, C.c_int(config)), "moe_set_gemm_config")


def moe_set_expert_output_fp32(ctx: MoeContext, enable: bool):
    _check(lib().moe_set_expert_output_fp32(ctx._h, C.c_int(1 if enable else 0)),
           "moe_set_expert_output_fp32")

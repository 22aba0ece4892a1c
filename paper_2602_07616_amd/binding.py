"""Thin ctypes binding of libsere.so (include/sere.h): same names, argument
marshalling only.  Every step of the layer runs in the library's HIP kernels;
PyTorch supplies device memory and the stream.  There is no fallback: if the
library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

SERE_F32 = 0
SERE_BF16 = 1

SERE_FLAG_RESIDUAL = 1
SERE_FLAG_SIM_COSINE = 2
SERE_FLAG_SIM_CKA_LINEAR = 4

SERE_OK = 0
SERE_ERR_NULL_PTR = -1
SERE_ERR_BAD_SHAPE = -2
SERE_ERR_BAD_TOPK = -3
SERE_ERR_BAD_DTYPE = -4
SERE_ERR_MISALIGNED = -5
SERE_ERR_WORKSPACE_TOO_SMALL = -6
SERE_ERR_BAD_FLAGS = -7
SERE_ERR_NONFINITE_THRESHOLD = -8
SERE_ERR_HIP = -9
SERE_ERR_BAD_KERNEL = -10
SERE_ERR_SCRATCH_TOO_SMALL = -11
SERE_STATIC_SCRATCH_BYTES = 32 << 20
SERE_CKA_LINEAR, SERE_CKA_RBF, SERE_CKA_POLY = 0, 1, 2

STAGES = ("router", "route", "gate_up", "down", "combine", "sim_pairs")

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsere.so")


class SereError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"libsere status {status}: {text}")
        self.status = status


class sere_config(ctypes.Structure):
    _fields_ = [("num_tokens", ctypes.c_int32), ("hidden", ctypes.c_int32),
                ("num_experts", ctypes.c_int32), ("top_k", ctypes.c_int32),
                ("inter", ctypes.c_int32), ("num_shared", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("select_top_k", ctypes.c_int32),
                ("threshold", ctypes.c_float), ("flags", ctypes.c_int32)]


class sere_route_out(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in (
        "topk_ids", "topk_weights", "rerouted_ids", "count_before", "count_after",
        "primary_mask", "num_active", "expert_offsets", "sorted_token", "sorted_slot")]


_lib: Optional[ctypes.CDLL] = None


def load() -> ctypes.CDLL:
    """Load libsere.so built in-tree (building it first if it was never built)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from . import build as _build
        _build.build(force=True)
    # PyTorch ships its own copy of the HIP runtime; it must be in the process before this
    # library is, so that both bind to the same one (two runtimes in one process do not
    # share devices, streams or memory)
    import torch  # noqa: F401
    lib = ctypes.CDLL(LIB_PATH)
    vp, sz, ci = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
    cfgp, outp = ctypes.POINTER(sere_config), ctypes.POINTER(sere_route_out)
    lib.sere_workspace_bytes.restype = sz
    lib.sere_workspace_bytes.argtypes = [cfgp]
    lib.sere_route.restype = ci
    lib.sere_route.argtypes = [cfgp, vp, vp, vp, outp, vp, sz, vp]
    lib.sere_reroute.restype = ci
    lib.sere_reroute.argtypes = [cfgp, vp, vp, outp, vp, sz, vp]
    lib.sere_moe_decode.restype = ci
    lib.sere_moe_decode.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, vp, vp, outp, vp, sz, vp]
    lib.sere_moe_decode_static.restype = ci
    lib.sere_moe_decode_static.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, vp, vp, outp, vp]
    lib.sere_moe_decode_baseline.restype = ci
    lib.sere_moe_decode_baseline.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, vp, outp, vp, sz, vp]
    lib.sere_similarity_workspace_bytes.restype = sz
    lib.sere_similarity_workspace_bytes.argtypes = [cfgp, ctypes.c_int32]
    lib.sere_similarity.restype = ci
    lib.sere_similarity.argtypes = [cfgp, vp, ctypes.c_int32, ctypes.c_int32, vp, vp, vp, vp, sz, vp]
    lib.sere_similarity_cka_workspace_bytes.restype = sz
    lib.sere_similarity_cka_workspace_bytes.argtypes = [cfgp, ctypes.c_int32]
    lib.sere_similarity_cka.restype = ci
    lib.sere_similarity_cka.argtypes = [cfgp, vp, ctypes.c_int32, ctypes.c_int32, vp, vp, ctypes.c_int32,
                                        ctypes.c_double, ctypes.c_double, vp, vp, sz, vp]
    lib.sere_stream_read.restype = ci
    lib.sere_stream_read.argtypes = [vp, sz, vp, vp]
    lib.sere_stage_timing.restype = ci
    lib.sere_stage_timing.argtypes = [ci]
    lib.sere_stage_timing_read.restype = ci
    lib.sere_stage_timing_read.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int32)]
    lib.sere_status_string.restype = ctypes.c_char_p
    lib.sere_status_string.argtypes = [ci]
    _lib = lib
    return lib


def sere_status_string(status: int) -> str:
    return load().sere_status_string(status).decode()


def _check(status: int) -> None:
    if status != SERE_OK:
        raise SereError(status, sere_status_string(status))


def make_config(num_tokens, hidden, num_experts, top_k, inter, num_shared, dtype,
                select_top_k, threshold, flags=0) -> sere_config:
    return sere_config(num_tokens, hidden, num_experts, top_k, inter, num_shared, dtype,
                       select_top_k, threshold, flags)


def sere_workspace_bytes(cfg: sere_config) -> int:
    return int(load().sere_workspace_bytes(ctypes.byref(cfg)))


def _ptr(t) -> ctypes.c_void_p:
    """Device address of a torch tensor (or a raw int address, or None)."""
    if t is None:
        return ctypes.c_void_p(0)
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


@dataclass
class RouteBuffers:
    """Device tensors for every optional routing output."""
    topk_ids: object
    topk_weights: object
    rerouted_ids: object
    count_before: object
    count_after: object
    primary_mask: object
    num_active: object
    expert_offsets: object
    sorted_token: object
    sorted_slot: object

    @staticmethod
    def allocate(cfg: sere_config, device="cuda") -> "RouteBuffers":
        import torch
        T, K, M = cfg.num_tokens, cfg.top_k, cfg.num_experts
        i32 = dict(dtype=torch.int32, device=device)
        return RouteBuffers(
            torch.full((T, K), -1, **i32), torch.zeros((T, K), dtype=torch.float32, device=device),
            torch.full((T, K), -1, **i32), torch.full((M,), -1, **i32), torch.full((M,), -1, **i32),
            torch.full((M,), -1, **i32), torch.full((2,), -1, **i32), torch.full((M + 1,), -1, **i32),
            torch.full((T * K,), -1, **i32), torch.full((T * K,), -1, **i32))

    def as_struct(self) -> sere_route_out:
        return sere_route_out(*[_ptr(getattr(self, n)).value for n, _ in sere_route_out._fields_])


def _route_out(out) -> Optional[ctypes.Structure]:
    if out is None:
        return None
    return out.as_struct() if isinstance(out, RouteBuffers) else out


def _byref_or_null(s):
    return ctypes.byref(s) if s is not None else None


def sere_route(cfg, hidden, router_w, sim, out, workspace, stream=None) -> None:
    o = _route_out(out)
    _check(load().sere_route(ctypes.byref(cfg), _ptr(hidden), _ptr(router_w), _ptr(sim),
                             _byref_or_null(o), _ptr(workspace),
                             workspace.numel() * workspace.element_size(), _stream(stream)))


def sere_reroute(cfg, topk_ids, sim, out, workspace, stream=None) -> None:
    o = _route_out(out)
    _check(load().sere_reroute(ctypes.byref(cfg), _ptr(topk_ids), _ptr(sim), _byref_or_null(o),
                               _ptr(workspace), workspace.numel() * workspace.element_size(),
                               _stream(stream)))


def sere_moe_decode(cfg, hidden, router_w, w_gate_up, w_down, shared_gate_up, shared_down, sim,
                    out, dbg, workspace, stream=None) -> None:
    o = _route_out(dbg)
    _check(load().sere_moe_decode(ctypes.byref(cfg), _ptr(hidden), _ptr(router_w), _ptr(w_gate_up),
                                  _ptr(w_down), _ptr(shared_gate_up), _ptr(shared_down), _ptr(sim),
                                  _ptr(out), _byref_or_null(o), _ptr(workspace),
                                  workspace.numel() * workspace.element_size(), _stream(stream)))


def sere_moe_decode_static(cfg, hidden, router_w, w_gate_up, w_down, shared_gate_up, shared_down, sim,
                           out, dbg, stream=None) -> None:
    o = _route_out(dbg)
    _check(load().sere_moe_decode_static(ctypes.byref(cfg), _ptr(hidden), _ptr(router_w), _ptr(w_gate_up),
                                         _ptr(w_down), _ptr(shared_gate_up), _ptr(shared_down), _ptr(sim),
                                         _ptr(out), _byref_or_null(o), _stream(stream)))


def sere_moe_decode_baseline(cfg, hidden, router_w, w_gate_up, w_down, shared_gate_up,
                             shared_down, out, dbg, workspace, stream=None) -> None:
    o = _route_out(dbg)
    _check(load().sere_moe_decode_baseline(
        ctypes.byref(cfg), _ptr(hidden), _ptr(router_w), _ptr(w_gate_up), _ptr(w_down),
        _ptr(shared_gate_up), _ptr(shared_down), _ptr(out), _byref_or_null(o), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream(stream)))


def sere_similarity_workspace_bytes(cfg: sere_config, batch_tokens: int) -> int:
    return int(load().sere_similarity_workspace_bytes(ctypes.byref(cfg), batch_tokens))


def sere_similarity(cfg, calib, num_batches, batch_tokens, w_gate_up, w_down, sim, workspace,
                    stream=None) -> None:
    _check(load().sere_similarity(ctypes.byref(cfg), _ptr(calib), num_batches, batch_tokens,
                                  _ptr(w_gate_up), _ptr(w_down), _ptr(sim), _ptr(workspace),
                                  workspace.numel() * workspace.element_size(), _stream(stream)))


def sere_similarity_cka_workspace_bytes(cfg: sere_config, batch_tokens: int) -> int:
    return int(load().sere_similarity_cka_workspace_bytes(ctypes.byref(cfg), batch_tokens))


def sere_similarity_cka(cfg, calib, num_batches, batch_tokens, w_gate_up, w_down, kernel, param0, param1, sim,
                        workspace, stream=None) -> None:
    _check(load().sere_similarity_cka(ctypes.byref(cfg), _ptr(calib), num_batches, batch_tokens,
                                      _ptr(w_gate_up), _ptr(w_down), kernel, float(param0), float(param1),
                                      _ptr(sim), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                      _stream(stream)))


def sere_stream_read(src, nbytes: int, sink, stream=None) -> None:
    """Plain streaming read of the first nbytes bytes of the tensor src (benchmark helper)."""
    _check(load().sere_stream_read(_ptr(src), nbytes, _ptr(sink), _stream(stream)))


def sere_stage_timing(enable: bool) -> None:
    _check(load().sere_stage_timing(1 if enable else 0))


def sere_stage_timing_read():
    """-> ({stage: total ms}, {stage: launches}) since the last read."""
    ms = (ctypes.c_double * len(STAGES))()
    n = (ctypes.c_int32 * len(STAGES))()
    _check(load().sere_stage_timing_read(ms, n))
    return ({s: ms[i] for i, s in enumerate(STAGES)}, {s: n[i] for i, s in enumerate(STAGES)})


def alloc_workspace(cfg: sere_config, device="cuda"):
    """A torch uint8 tensor of sere_workspace_bytes(cfg) (256-byte aligned by the allocator)."""
    import torch
    n = sere_workspace_bytes(cfg)
    if n == 0:
        raise SereError(SERE_ERR_BAD_SHAPE, "invalid configuration")
    return torch.empty(n, dtype=torch.uint8, device=device)

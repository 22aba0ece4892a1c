"""Python face of the CPU oracle (oracle/sere_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  The HIP library and its Python binding never
import this package.

All tensors are numpy arrays in storage format: ``float32`` for dtype 0,
``uint16`` bf16 bit patterns for dtype 1.  Every function here only marshals
arguments into the C routines; the arithmetic lives in the C file, which
cites the passages of the paper it follows.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np

from .build import LIB, build

F32 = 0
BF16 = 1


def _p(a: Optional[np.ndarray]):
    if a is None:
        return ctypes.c_void_p(0)
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.c_void_p)


def _check(a: np.ndarray, dtype: int) -> np.ndarray:
    want = np.float32 if dtype == F32 else np.uint16
    assert a.dtype == want, (a.dtype, dtype)
    return np.ascontiguousarray(a)


@dataclass
class LayerResult:
    logits: np.ndarray          # [T,M] f64
    topk_ids: np.ndarray        # [T,K] i32  (I)
    topk_weights: np.ndarray    # [T,K] f64  (W)
    min_gap: float
    primary_mask: np.ndarray    # [M] (H)
    rerouted_ids: np.ndarray    # [T,K] (I')
    final_set: np.ndarray       # [M] 0/1
    count_before: np.ndarray    # [M]
    count_after: np.ndarray     # [M]
    offsets: np.ndarray         # [M+1] from count_after
    sorted_token: np.ndarray    # [T*K]
    sorted_slot: np.ndarray     # [T*K]
    n_active_before: int
    n_active_after: int
    out_base: Optional[np.ndarray]   # [T,dh] f64, standard top-k MoE
    out_sere: Optional[np.ndarray]   # [T,dh] f64, with the re-routed map


class OracleLib:
    """The oracle's routines bound to one compiled library file."""

    def __init__(self, path: Optional[str] = None):
        if path is None:
            build(force=False)
            path = LIB
        self.c = ctypes.CDLL(path)
        self.c.oracle_max_threads.restype = ctypes.c_int

    def set_threads(self, n: int) -> None:
        self.c.oracle_set_threads(ctypes.c_int(n))

    def max_threads(self) -> int:
        return int(self.c.oracle_max_threads())

    def router_logits(self, hidden, router_w, dtype: int) -> np.ndarray:
        hidden, router_w = _check(hidden, dtype), _check(router_w, dtype)
        T, dh = hidden.shape
        M = router_w.shape[0]
        assert router_w.shape[1] == dh
        out = np.empty((T, M), dtype=np.float64)
        self.c.oracle_router_logits(_p(hidden), _p(router_w), dtype, T, M, dh, _p(out))
        return out

    def topk_gate(self, logits, K: int):
        """-> ids [T,K] int32, weights [T,K] float64, min_gap float."""
        logits = np.ascontiguousarray(logits, dtype=np.float64)
        T, M = logits.shape
        assert 1 <= K <= M
        ids = np.empty((T, K), dtype=np.int32)
        w = np.empty((T, K), dtype=np.float64)
        gap = ctypes.c_double(0.0)
        self.c.oracle_topk_gate(_p(logits), T, M, K, _p(ids), _p(w), ctypes.byref(gap))
        return ids, w, float(gap.value)

    def primary_mask(self, ids, S: int, M: int) -> np.ndarray:
        ids = np.ascontiguousarray(ids, dtype=np.int32)
        T, K = ids.shape
        assert 1 <= S <= K
        H = np.empty(M, dtype=np.int32)
        self.c.oracle_primary_mask(_p(ids), T, K, S, M, _p(H))
        return H

    def reroute_per_slot(self, ids, sim, S: int, rho: float) -> np.ndarray:
        ids = np.ascontiguousarray(ids, dtype=np.int32)
        sim = np.ascontiguousarray(sim, dtype=np.float32)
        T, K = ids.shape
        M = sim.shape[0]
        assert sim.shape == (M, M) and 1 <= S <= K
        out = np.empty_like(ids)
        self.c.oracle_reroute_per_slot(_p(ids), _p(sim), T, K, M, S, ctypes.c_float(rho),
                                       _p(out))
        return out

    def reroute_sets(self, ids, sim, S: int, rho: float):
        """-> ids' [T,K], final_set [M] 0/1, target [M] (v* or -1), sim_star [M]."""
        ids = np.ascontiguousarray(ids, dtype=np.int32)
        sim = np.ascontiguousarray(sim, dtype=np.float32)
        T, K = ids.shape
        M = sim.shape[0]
        assert sim.shape == (M, M) and 1 <= S <= K
        out = np.empty_like(ids)
        final_set = np.empty(M, dtype=np.int32)
        target = np.empty(M, dtype=np.int32)
        sim_star = np.empty(M, dtype=np.float32)
        self.c.oracle_reroute_sets(_p(ids), _p(sim), T, K, M, S, ctypes.c_float(rho), _p(out),
                                   _p(final_set), _p(target), _p(sim_star))
        return out, final_set, target, sim_star

    def compact(self, ids, M: int):
        """-> count [M], offsets [M+1], sorted_token [T*K], sorted_slot [T*K], n_active."""
        ids = np.ascontiguousarray(ids, dtype=np.int32)
        T, K = ids.shape
        count = np.empty(M, dtype=np.int32)
        offsets = np.empty(M + 1, dtype=np.int32)
        tok = np.empty(T * K, dtype=np.int32)
        slot = np.empty(T * K, dtype=np.int32)
        n = ctypes.c_int32(0)
        self.c.oracle_compact(_p(ids), T, K, M, _p(count), _p(offsets), _p(tok), _p(slot),
                              ctypes.byref(n))
        return count, offsets, tok, slot, int(n.value)

    def expert_ffn(self, x, w_gate_up_e, w_down_e, dtype: int) -> np.ndarray:
        x = _check(x, dtype)
        w_gate_up_e, w_down_e = _check(w_gate_up_e, dtype), _check(w_down_e, dtype)
        dh = x.shape[0]
        dm = w_down_e.shape[1]
        assert w_gate_up_e.shape == (2 * dm, dh) and w_down_e.shape == (dh, dm)
        y = np.empty(dh, dtype=np.float64)
        self.c.oracle_expert_ffn(_p(x), _p(w_gate_up_e), _p(w_down_e), dtype, dh, dm, _p(y))
        return y

    def moe_layer(self, hidden, w_gate_up, w_down, shared_gate_up, shared_down, dtype: int,
                  ids, weights) -> np.ndarray:
        hidden = _check(hidden, dtype)
        w_gate_up, w_down = _check(w_gate_up, dtype), _check(w_down, dtype)
        T, dh = hidden.shape
        M, dm2, _ = w_gate_up.shape
        dm = dm2 // 2
        assert w_gate_up.shape == (M, 2 * dm, dh) and w_down.shape == (M, dh, dm)
        n_sh = 0
        if shared_gate_up is not None:
            shared_gate_up = _check(shared_gate_up, dtype)
            shared_down = _check(shared_down, dtype)
            n_sh = shared_gate_up.shape[0]
            assert shared_gate_up.shape == (n_sh, 2 * dm, dh)
            assert shared_down.shape == (n_sh, dh, dm)
        ids = np.ascontiguousarray(ids, dtype=np.int32)
        weights = np.ascontiguousarray(weights, dtype=np.float64)
        K = ids.shape[1]
        assert ids.shape == (T, K) and weights.shape == (T, K)
        assert ids.min() >= 0 and ids.max() < M
        out = np.empty((T, dh), dtype=np.float64)
        self.c.oracle_moe_layer(_p(hidden), _p(w_gate_up), _p(w_down), _p(shared_gate_up),
                                _p(shared_down), dtype, T, dh, M, K, dm, n_sh, _p(ids),
                                _p(weights), _p(out))
        return out

    def similarity_frobenius(self, calib, w_gate_up, w_down, dtype: int) -> np.ndarray:
        """-> S [M,M] float64 (cast to float32 to feed the layer)."""
        calib = _check(calib, dtype)
        w_gate_up, w_down = _check(w_gate_up, dtype), _check(w_down, dtype)
        N, n, dh = calib.shape
        M, dm2, _ = w_gate_up.shape
        dm = dm2 // 2
        assert w_gate_up.shape == (M, 2 * dm, dh) and w_down.shape == (M, dh, dm)
        act = np.empty((M, n, dh), dtype=np.float64)
        sim = np.empty((M, M), dtype=np.float64)
        self.c.oracle_similarity_frobenius(_p(calib), _p(w_gate_up), _p(w_down), dtype, N, n,
                                           dh, M, dm, _p(act), _p(sim))
        return sim

    def similarity_cosine(self, calib, w_gate_up, w_down, dtype: int) -> np.ndarray:
        """-> S [M,M] float64, the cosine metric of the appendix on similarity metrics."""
        calib = _check(calib, dtype)
        w_gate_up, w_down = _check(w_gate_up, dtype), _check(w_down, dtype)
        N, n, dh = calib.shape
        M, dm2, _ = w_gate_up.shape
        dm = dm2 // 2
        assert w_gate_up.shape == (M, 2 * dm, dh) and w_down.shape == (M, dh, dm)
        act = np.empty((M, n, dh), dtype=np.float64)
        sim = np.empty((M, M), dtype=np.float64)
        self.c.oracle_similarity_cosine(_p(calib), _p(w_gate_up), _p(w_down), dtype, N, n,
                                        dh, M, dm, _p(act), _p(sim))
        return sim

    def similarity_cka_linear(self, calib, w_gate_up, w_down, dtype: int) -> np.ndarray:
        """-> S [M,M] float64, linear-kernel CKA with the unbiased HSIC estimator (appendix on
        similarity metrics); needs at least 4 tokens per calibration batch."""
        calib = _check(calib, dtype)
        w_gate_up, w_down = _check(w_gate_up, dtype), _check(w_down, dtype)
        N, n, dh = calib.shape
        M, dm2, _ = w_gate_up.shape
        dm = dm2 // 2
        assert n >= 4
        assert w_gate_up.shape == (M, 2 * dm, dh) and w_down.shape == (M, dh, dm)
        act = np.empty((M, n, dh), dtype=np.float64)
        gram = np.empty((M, n, n), dtype=np.float64)
        sim = np.empty((M, M), dtype=np.float64)
        self.c.oracle_similarity_cka_linear(_p(calib), _p(w_gate_up), _p(w_down), dtype, N, n,
                                            dh, M, dm, _p(act), _p(gram), _p(sim))
        return sim

    def similarity_cka(self, calib, w_gate_up, w_down, dtype: int, kernel: str, p0: float = 0.0,
                       p1: float = 0.0) -> np.ndarray:
        """-> S [M,M] float64, CKA with the kernel "linear", "rbf" (p0 = sigma) or "poly"
        (p0 = c, p1 = degree) of the appendix on similarity metrics."""
        calib = _check(calib, dtype)
        w_gate_up, w_down = _check(w_gate_up, dtype), _check(w_down, dtype)
        N, n, dh = calib.shape
        M, dm2, _ = w_gate_up.shape
        dm = dm2 // 2
        assert n >= 4
        kid = {"linear": 0, "rbf": 1, "poly": 2}[kernel]
        assert kid != 1 or p0 > 0.0
        assert kid != 2 or (p1 >= 1 and float(p1).is_integer())
        act = np.empty((M, n, dh), dtype=np.float64)
        gram = np.empty((M, n, n), dtype=np.float64)
        sim = np.empty((M, M), dtype=np.float64)
        self.c.oracle_similarity_cka(_p(calib), _p(w_gate_up), _p(w_down), dtype, N, n, dh, M, dm, kid,
                                     ctypes.c_double(p0), ctypes.c_double(p1), _p(act), _p(gram), _p(sim))
        return sim

    def route(self, hidden, router_w, dtype: int, K: int, sim, S: int,
              rho: float) -> LayerResult:
        """Routing half of the layer (no expert is executed)."""
        logits = self.router_logits(hidden, router_w, dtype)
        M = logits.shape[1]
        ids, w, gap = self.topk_gate(logits, K)
        H = self.primary_mask(ids, S, M)
        new_ids, final_set, _, _ = self.reroute_sets(ids, sim, S, rho)
        cnt_b, _, _, _, n_b = self.compact(ids, M)
        cnt_a, offs, tok, slot, n_a = self.compact(new_ids, M)
        return LayerResult(logits, ids, w, gap, H, new_ids, final_set, cnt_b, cnt_a, offs, tok,
                           slot, n_b, n_a, None, None)

    def layer(self, hidden, router_w, w_gate_up, w_down, shared_gate_up, shared_down,
              dtype: int, K: int, sim, S: int, rho: float, want_base: bool = True,
              want_sere: bool = True) -> LayerResult:
        """The whole layer, without (out_base) and with (out_sere) re-routing."""
        r = self.route(hidden, router_w, dtype, K, sim, S, rho)
        if want_base:
            r.out_base = self.moe_layer(hidden, w_gate_up, w_down, shared_gate_up, shared_down,
                                        dtype, r.topk_ids, r.topk_weights)
        if want_sere:
            r.out_sere = self.moe_layer(hidden, w_gate_up, w_down, shared_gate_up, shared_down,
                                        dtype, r.rerouted_ids, r.topk_weights)
        return r


_default: Optional[OracleLib] = None


def default() -> OracleLib:
    global _default
    if _default is None:
        _default = OracleLib()
    return _default


def __getattr__(name: str):
    # oracle.layer(...), oracle.route(...), ... use the default library
    if not name.startswith("_") and hasattr(OracleLib, name):
        return getattr(default(), name)
    raise AttributeError(name)

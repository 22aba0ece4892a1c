"""Moving a generated workload into HBM and calling the library on it.

Only plumbing: numpy storage arrays become torch device tensors (bf16 bit
patterns are reinterpreted, never converted), buffers are allocated, and the
C-ABI entry points are called through the binding.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np

from . import binding as B
from .workloads import BF16, F32, Workload


def to_device(a: Optional[np.ndarray], dtype: int, device="cuda"):
    """numpy storage array -> torch tensor on `device` (bf16 for uint16 bit patterns)."""
    import torch
    if a is None:
        return None
    if dtype == F32:
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint16).view(np.int16)).to(device)
    return t.view(torch.bfloat16)


def to_host(t, dtype: int) -> np.ndarray:
    """torch tensor -> numpy storage array (uint16 bit patterns for bf16)."""
    import torch
    if dtype == F32:
        return t.detach().cpu().numpy()
    return t.detach().view(torch.int16).cpu().numpy().view(np.uint16)


def similarity_on_device(wl: Workload, weights=None, device="cuda", metric="frobenius", cka=None):
    """Expert-similarity matrix of the workload's layer from its calibration
    tokens, computed by the library (sere_similarity); returns a device fp32 [M, M]
    tensor.  `weights` = (router_w, w_gate_up, w_down, ...) already on the device.
    metric: "frobenius" | "cosine" | "cka_linear"; or cka = (kernel, param0, param1) with kernel
    "linear" | "rbf" | "poly" for sere_similarity_cka."""
    import torch
    sp = wl.spec
    n_batches, n_tokens = wl.calib.shape[0], wl.calib.shape[1]
    cfg = B.make_config(n_tokens, sp.hidden, sp.experts, min(sp.top_k, sp.experts), sp.inter, 0,
                        sp.dtype, 1, 0.0, {"frobenius": 0, "cosine": B.SERE_FLAG_SIM_COSINE,
                                          "cka_linear": B.SERE_FLAG_SIM_CKA_LINEAR}[metric])
    gu = to_device(wl.w_gate_up, sp.dtype, device) if weights is None else weights[1]
    dn = to_device(wl.w_down, sp.dtype, device) if weights is None else weights[2]
    calib = to_device(wl.calib, sp.dtype, device)
    sim = torch.empty((sp.experts, sp.experts), dtype=torch.float32, device=device)
    if cka is not None:
        kernel, p0, p1 = cka
        ws = torch.empty(B.sere_similarity_cka_workspace_bytes(cfg, n_tokens), dtype=torch.uint8, device=device)
        B.sere_similarity_cka(cfg, calib, n_batches, n_tokens, gu, dn,
                              {"linear": B.SERE_CKA_LINEAR, "rbf": B.SERE_CKA_RBF, "poly": B.SERE_CKA_POLY}[kernel],
                              p0, p1, sim, ws)
    else:
        ws = torch.empty(B.sere_similarity_workspace_bytes(cfg, n_tokens), dtype=torch.uint8, device=device)
        B.sere_similarity(cfg, calib, n_batches, n_tokens, gu, dn, sim, ws)
    torch.cuda.synchronize()
    return sim


@dataclass
class DeviceLayer:
    """One MoE layer's tensors resident in HBM plus the call-time buffers."""
    spec: object
    hidden: object
    router_w: object
    w_gate_up: object
    w_down: object
    shared_gate_up: object
    shared_down: object
    sim: object
    out: object
    workspace: object
    route: B.RouteBuffers
    cfg: B.sere_config

    @staticmethod
    def from_workload(wl: Workload, sim: np.ndarray, S: int, rho: float, device="cuda",
                      weights=None) -> "DeviceLayer":
        """`weights` lets several DeviceLayers (other batches / settings) share one
        resident copy of the expert tensors: (router_w, w_gate_up, w_down, sgu, sdn)."""
        import torch
        sp = wl.spec
        cfg = B.make_config(wl.hidden.shape[0], sp.hidden, sp.experts, sp.top_k, sp.inter,
                            sp.shared, sp.dtype, S, rho)
        if weights is None:
            weights = (to_device(wl.router_w, sp.dtype, device), to_device(wl.w_gate_up, sp.dtype, device),
                       to_device(wl.w_down, sp.dtype, device),
                       to_device(wl.shared_gate_up, sp.dtype, device),
                       to_device(wl.shared_down, sp.dtype, device))
        tdt = torch.float32 if sp.dtype == F32 else torch.bfloat16
        if isinstance(sim, np.ndarray):
            sim = torch.from_numpy(np.ascontiguousarray(sim, dtype=np.float32)).to(device)
        return DeviceLayer(
            sp, to_device(wl.hidden, sp.dtype, device), *weights, sim,
            torch.zeros((wl.hidden.shape[0], sp.hidden), dtype=tdt, device=device),
            B.alloc_workspace(cfg, device), B.RouteBuffers.allocate(cfg, device), cfg)

    def weights(self):
        return (self.router_w, self.w_gate_up, self.w_down, self.shared_gate_up, self.shared_down)

    def set_knobs(self, S: int, rho: float) -> None:
        self.cfg.select_top_k = S
        self.cfg.threshold = rho

    def run_route(self, stream=None, with_outputs=True) -> None:
        B.sere_route(self.cfg, self.hidden, self.router_w, self.sim,
                     self.route if with_outputs else None, self.workspace, stream)

    def run_reroute(self, stream=None, with_outputs=True) -> None:
        """Re-routing alone on the top-K ids of the last run with outputs (indices in, indices out)."""
        B.sere_reroute(self.cfg, self.route.topk_ids, self.sim, self.route if with_outputs else None,
                       self.workspace, stream)

    def run_decode(self, stream=None, with_outputs=True) -> None:
        B.sere_moe_decode(self.cfg, self.hidden, self.router_w, self.w_gate_up, self.w_down,
                          self.shared_gate_up, self.shared_down, self.sim, self.out,
                          self.route if with_outputs else None, self.workspace, stream)

    def run_baseline(self, stream=None, with_outputs=True) -> None:
        B.sere_moe_decode_baseline(self.cfg, self.hidden, self.router_w, self.w_gate_up,
                                   self.w_down, self.shared_gate_up, self.shared_down, self.out,
                                   self.route if with_outputs else None, self.workspace, stream)

    def routing_to_host(self) -> dict:
        import torch
        torch.cuda.synchronize()
        return {n: getattr(self.route, n).cpu().numpy() for n, _ in B.sere_route_out._fields_}

    def out_to_host_f64(self) -> np.ndarray:
        import torch
        torch.cuda.synchronize()
        return self.out.detach().to(torch.float64).cpu().numpy()


class DecodeStack:
    """L consecutive MoE layers of a decoder chained on the device:
    x_{l+1} = x_l + MoE_l(x_l) (the residual connection is added by the library's
    combine step, SERE_FLAG_RESIDUAL), each layer with its own weights and its own
    similarity matrix (Sec. 3.1.1: one matrix per layer).  Attention and
    normalisation, which sit between MoE blocks in a real decoder, are not part of
    this path.  Layer l reads the tensor layer l-1 wrote: no copy, no kernel in between.
    """

    def __init__(self, workloads, sims, S: int, rho: float, device="cuda", share_weights=False):
        """workloads: one per layer (same shape); sims: one [M, M] matrix per layer.
        share_weights: every layer uses layer 0's resident tensors (timing only)."""
        self.layers = []
        weights = None
        for wl, sim in zip(workloads, sims):
            layer = DeviceLayer.from_workload(wl, sim, S, rho, device, weights=weights if share_weights else None)
            if share_weights and weights is None:
                weights = layer.weights()
            layer.cfg.flags = B.SERE_FLAG_RESIDUAL
            if self.layers:
                layer.hidden = self.layers[-1].out
            self.layers.append(layer)

    def set_knobs(self, S: int, rho: float) -> None:
        for l in self.layers:
            l.set_knobs(S, rho)

    def run(self, stream=None, reroute=True, with_outputs=True) -> None:
        for l in self.layers:
            if reroute:
                l.run_decode(stream, with_outputs)
            else:
                l.run_baseline(stream, with_outputs)

    def active_counts(self):
        """[(before, after)] per layer of the last run with outputs."""
        import torch
        torch.cuda.synchronize()
        return [tuple(l.route.num_active.cpu().tolist()) for l in self.layers]

    def out_to_host_f64(self) -> np.ndarray:
        return self.layers[-1].out_to_host_f64()

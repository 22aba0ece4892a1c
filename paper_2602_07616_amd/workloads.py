"""Seeded synthetic inputs for the batch-decode MoE layer.

This module only draws numbers and lays them out; it holds none of the
method's arithmetic (no routing, no expert FFN, no similarity).  Both the CPU
oracle's tests and the HIP path's tests/bench obtain their inputs here, so the
two sides always see the same bits.

Every tensor is a numpy array.  bf16 tensors are carried as ``uint16`` bit
patterns (the upper half of the IEEE fp32 word, rounded to nearest-even once
from an fp32 draw); fp32 tensors as ``float32``.

The random source is a counter-based generator: the value at index ``i`` of a
named stream depends only on ``(seed, stream name, i)``, so a prefix of a
stream is the same no matter how many values are drawn, and nothing depends on
a library's generator staying stable between versions.

The layer shapes stand in for the models the paper serves (its model table in
the appendix on experiment settings: Qwen3-30B-A3B with 128 experts / top-8,
DeepSeek-V2-Lite with 64 experts / top-6 plus 2 shared, Qwen1.5-MoE-A2.7B with
60 experts / top-4 plus 4 shared); real weights and calibration corpora are
not used anywhere.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field, replace
from typing import Dict, Optional, Tuple

import numpy as np

F32 = 0
BF16 = 1

_MASK = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_CHUNK = 1 << 17  # pairs per chunk when filling large tensors


# --------------------------------------------------------------------------
# counter-based random numbers
# --------------------------------------------------------------------------
def _mix64_int(z: int) -> int:
    z &= _MASK
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK
    return z ^ (z >> 31)


def _mix64(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
    z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
    return z ^ (z >> np.uint64(31))


def stream_key(seed: int, name: str) -> int:
    """64-bit key of a named substream of ``seed``."""
    h = 0xCBF29CE484222325
    for byte in name.encode():
        h = ((h ^ byte) * 0x100000001B3) & _MASK
    return _mix64_int(_mix64_int(seed & _MASK) ^ h)


def raw_bits(seed: int, name: str, start: int, count: int) -> np.ndarray:
    """``count`` 64-bit words of stream ``name`` beginning at counter ``start``."""
    key = stream_key(seed, name)
    with np.errstate(over="ignore"):
        ctr = np.arange(start + 1, start + count + 1, dtype=np.uint64)
        return _mix64(np.uint64(key) + ctr * np.uint64(_GOLDEN))


def _normal_pairs(seed: int, name: str, pair_start: int, pairs: int) -> np.ndarray:
    """2*pairs standard normals (Box-Muller; both branches of a pair are used)."""
    bits = raw_bits(seed, name, pair_start, pairs)
    hi = (bits >> np.uint64(32)).astype(np.float64)
    lo = (bits & np.uint64(0xFFFFFFFF)).astype(np.float64)
    u1 = (hi + 0.5) * (1.0 / 4294967296.0)
    u2 = (lo + 0.5) * (1.0 / 4294967296.0)
    r = np.sqrt(-2.0 * np.log(u1))
    ang = (2.0 * np.pi) * u2
    out = np.empty(2 * pairs, dtype=np.float32)
    out[0::2] = r * np.cos(ang)
    out[1::2] = r * np.sin(ang)
    return out


def _threads() -> int:
    return max(1, min(16, int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))))


def std_normal(seed: int, name: str, count: int) -> np.ndarray:
    """First ``count`` standard normals (fp32) of stream ``name``."""
    pairs = (count + 1) // 2
    out = np.empty(2 * pairs, dtype=np.float32)
    spans = [(p, min(_CHUNK, pairs - p)) for p in range(0, pairs, _CHUNK)]

    def fill(span):
        p, n = span
        out[2 * p:2 * (p + n)] = _normal_pairs(seed, name, p, n)

    if len(spans) > 1:
        with ThreadPoolExecutor(_threads()) as pool:
            list(pool.map(fill, spans))
    else:
        for s in spans:
            fill(s)
    return out[:count]


def uniform_int(seed: int, name: str, count: int, modulus: int) -> np.ndarray:
    """``count`` integers in [0, modulus) from stream ``name``."""
    return (raw_bits(seed, name, 0, count) >> np.uint64(11)).astype(np.int64) % modulus


# --------------------------------------------------------------------------
# storage formats
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(x: np.ndarray, dtype: int) -> np.ndarray:
    if dtype == F32:
        return np.ascontiguousarray(x, dtype=np.float32)
    return f32_to_bf16_bits(x)


def storage_to_f64(x: np.ndarray, dtype: int) -> np.ndarray:
    """Exact widening of a stored tensor (for tests and reports)."""
    if dtype == F32:
        return x.astype(np.float64)
    return bf16_bits_to_f32(x).astype(np.float64)


# --------------------------------------------------------------------------
# layer / workload descriptions
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class LayerSpec:
    name: str
    dtype: int                 # F32 | BF16: hidden, all weights, output
    hidden: int                # d_h
    experts: int               # M routed experts
    top_k: int                 # K
    inter: int                 # d_m per expert
    shared: int                # always-on shared experts
    tokens: int                # T decode tokens in the batch
    weight_seed: int
    hidden_seed: int
    clusters: int = 0          # 0: hidden ~ N(0,1); >0: Gaussian clusters
    cluster_std: float = 0.5
    twin_src: int = 0          # experts [twin_dst, twin_dst+twin_n) are
    twin_dst: int = 0          # perturbed copies of [twin_src, twin_src+twin_n)
    twin_n: int = 0
    twin_noise: float = 0.1    # noise scale relative to weight_std
    weight_std: float = 0.02
    calib_batches: int = 2     # N of the similarity estimation
    calib_tokens: int = 32     # tokens per calibration batch
    grid: Tuple[Tuple[int, float], ...] = ()   # (S, rho) settings measured

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == F32 else 2

    @property
    def expert_bytes(self) -> int:
        return 3 * self.hidden * self.inter * self.elem_bytes


SPECS: Dict[str, LayerSpec] = {
    # tiny fp32 layer; experts 8-15 are experts 0-7 plus 0.1x-scaled noise
    "tiny": LayerSpec("tiny", F32, 256, 16, 2, 128, 0, 8, 1001, 1001,
                      twin_src=0, twin_dst=8, twin_n=8,
                      grid=((1, 0.0), (1, 0.5))),
    # Qwen3-30B-A3B-shaped layer, clustered batch of 32; a quarter of the
    # experts (96-127) are perturbed copies of experts 0-31
    "qwen3_b32": LayerSpec("qwen3_b32", BF16, 2048, 128, 8, 768, 0, 32, 1002, 1002,
                           clusters=8, twin_src=0, twin_dst=96, twin_n=32,
                           grid=((2, 0.0), (2, 0.5), (1, 0.0), (1, 0.5))),
    # same layer, maximally diverse batch of 128 (prefixes of one 256-token draw)
    "qwen3_b128": LayerSpec("qwen3_b128", BF16, 2048, 128, 8, 768, 0, 128, 1002, 1003,
                            twin_src=0, twin_dst=96, twin_n=32,
                            grid=((2, 0.0), (2, 0.5), (1, 0.0), (1, 0.5))),
    # DeepSeek-V2-Lite-shaped layer with 2 shared experts
    "dsv2lite_b64": LayerSpec("dsv2lite_b64", BF16, 2048, 64, 6, 1408, 2, 64, 1004, 1004,
                              clusters=16,
                              grid=((2, 0.0), (2, 0.3), (1, 0.0), (1, 0.3))),
    # Mixtral-8x7B-shaped layer: few, very large experts
    "mixtral_b64": LayerSpec("mixtral_b64", BF16, 4096, 8, 2, 14336, 0, 64, 1005, 1005,
                             calib_tokens=8,
                             grid=((1, 0.0), (1, 0.3))),
    # Qwen1.5-MoE-A2.7B-shaped layer (60 experts, top-4, 4 shared).  The paper
    # gives no per-expert width; 1408 is this build's choice.
    "qwen15_b32": LayerSpec("qwen15_b32", BF16, 2048, 60, 4, 1408, 4, 32, 1006, 1006,
                            clusters=8, twin_src=0, twin_dst=45, twin_n=15,
                            grid=((2, 0.0), (2, 0.3), (1, 0.0), (1, 0.3))),
}

BATCH_SWEEP = (1, 4, 16, 32, 64, 128, 256)   # qwen3_b128 prefixes


@dataclass
class Workload:
    spec: LayerSpec
    hidden: np.ndarray                    # [T, d_h]
    router_w: np.ndarray                  # [M, d_h]
    w_gate_up: np.ndarray                 # [M, 2*d_m, d_h]  rows 0..d_m-1 gate, then up
    w_down: np.ndarray                    # [M, d_h, d_m]
    shared_gate_up: Optional[np.ndarray]  # [n_sh, 2*d_m, d_h]
    shared_down: Optional[np.ndarray]     # [n_sh, d_h, d_m]
    calib: np.ndarray                     # [N, n, d_h] calibration tokens
    extra: dict = field(default_factory=dict)


def _draw_hidden(spec: LayerSpec, seed: int, tag: str, count: int) -> np.ndarray:
    d = spec.hidden
    noise = std_normal(seed, f"{tag}.noise", count * d).reshape(count, d)
    if spec.clusters <= 0:
        return noise
    # the centres belong to the layer's input distribution, not to one batch
    centres = std_normal(spec.hidden_seed, "hidden.centres", spec.clusters * d)
    centres = centres.reshape(spec.clusters, d)
    which = uniform_int(seed, f"{tag}.cluster", count, spec.clusters)
    return centres[which] + np.float32(spec.cluster_std) * noise


def _draw_experts(spec: LayerSpec, tag: str, n: int, rows: int, cols: int,
                  twins: bool) -> np.ndarray:
    std = np.float32(spec.weight_std)
    out = np.empty((n, rows, cols), dtype=np.float32 if spec.dtype == F32 else np.uint16)
    per = rows * cols
    for e in range(n):
        src = e
        if twins and spec.twin_n and spec.twin_dst <= e < spec.twin_dst + spec.twin_n:
            src = spec.twin_src + (e - spec.twin_dst)
        # one stream per expert so any expert can be regenerated alone
        w = std * std_normal(spec.weight_seed, f"{tag}.{src}", per)
        if src != e:
            w = w + np.float32(spec.twin_noise) * std * std_normal(
                spec.weight_seed, f"{tag}.twin_noise.{e}", per)
        out[e] = to_storage(w, spec.dtype).reshape(rows, cols)
    return out


_FORMAT = 1   # bump when a change alters the generated bits


def _cache_dir() -> Optional[str]:
    d = os.environ.get("SERE_WORKLOAD_CACHE", "/tmp/sere_workloads")
    if not d or d == "0":
        return None
    try:
        os.makedirs(d, exist_ok=True)
    except OSError:
        return None
    return d


def _cached_experts(spec: LayerSpec, tag: str, n: int, rows: int, cols: int,
                    twins: bool) -> np.ndarray:
    """Expert tensors above 64 MiB are kept as .npy files between runs: they
    are a pure function of the fields in the key."""
    nbytes = n * rows * cols * spec.elem_bytes
    d = _cache_dir()
    if d is None or nbytes < (64 << 20):
        return _draw_experts(spec, tag, n, rows, cols, twins)
    key = (f"v{_FORMAT}_{tag}_{spec.dtype}_{spec.weight_seed}_{n}x{rows}x{cols}_"
           f"{spec.weight_std}_{spec.twin_src}_{spec.twin_dst}_{spec.twin_n}_"
           f"{spec.twin_noise}_{int(twins)}")
    path = os.path.join(d, key + ".npy")
    if os.path.exists(path):
        try:
            arr = np.load(path, allow_pickle=False)
            if arr.shape == (n, rows, cols):
                return arr
        except (OSError, ValueError):
            pass
    arr = _draw_experts(spec, tag, n, rows, cols, twins)
    try:
        tmp = f"{path}.{os.getpid()}.tmp.npy"
        np.save(tmp, arr)
        os.replace(tmp, path)
    except OSError:
        pass
    return arr


def make_workload(spec_or_name, tokens: Optional[int] = None,
                  hidden_seed: Optional[int] = None) -> Workload:
    """Build the full seeded input set of one layer + batch."""
    spec = SPECS[spec_or_name] if isinstance(spec_or_name, str) else spec_or_name
    if tokens is not None:
        spec = replace(spec, tokens=tokens)
    if hidden_seed is not None:
        spec = replace(spec, hidden_seed=hidden_seed)
    d, m, dm = spec.hidden, spec.experts, spec.inter

    hidden = to_storage(_draw_hidden(spec, spec.hidden_seed, "hidden", spec.tokens), spec.dtype)
    router = np.float32(spec.weight_std) * std_normal(spec.weight_seed, "router", m * d)
    router_w = to_storage(router, spec.dtype).reshape(m, d)
    w_gate_up = _cached_experts(spec, "gate_up", m, 2 * dm, d, True)
    w_down = _cached_experts(spec, "down", m, d, dm, True)
    if spec.shared:
        shared_gate_up = _draw_experts(spec, "shared_gate_up", spec.shared, 2 * dm, d, False)
        shared_down = _draw_experts(spec, "shared_down", spec.shared, d, dm, False)
    else:
        shared_gate_up = shared_down = None
    n_cal = spec.calib_batches * spec.calib_tokens
    calib = to_storage(_draw_hidden(spec, spec.hidden_seed, "calib", n_cal), spec.dtype)
    calib = calib.reshape(spec.calib_batches, spec.calib_tokens, d)
    return Workload(spec, hidden.reshape(spec.tokens, d), router_w, w_gate_up, w_down,
                    shared_gate_up, shared_down, calib)


def custom_spec(name: str, dtype: int, hidden: int, experts: int, top_k: int, inter: int,
                shared: int, tokens: int, seed: int, **kw) -> LayerSpec:
    """A free-form layer for edge-case tests."""
    return LayerSpec(name, dtype, hidden, experts, top_k, inter, shared, tokens,
                     seed, seed, **kw)


def stack_specs(spec: LayerSpec, layers: int) -> Tuple[LayerSpec, ...]:
    """Specs of `layers` consecutive MoE layers of one model: same shape and
    input batch, independent weights (layer l draws from weight_seed + 7919*l)."""
    return tuple(replace(spec, name=f"{spec.name}.L{l}", weight_seed=spec.weight_seed + 7919 * l)
                 for l in range(layers))


def planted_similarity(spec: LayerSpec, seed: int) -> np.ndarray:
    """A synthetic [M, M] fp32 similarity matrix with the structure the paper
    reports for trained models (groups of similar experts, a unit diagonal,
    values in [0, 1]) without running any expert: twin pairs score high, all
    other pairs draw a low value.  Used where only the *shape* of the matrix
    matters (argument marshalling tests, routing-only timing)."""
    m = spec.experts
    low = (raw_bits(seed, "planted_sim", 0, m * m) >> np.uint64(40)).astype(np.float64)
    low = (low / float(1 << 24)) * 0.4
    low = low.reshape(m, m)
    sim = np.triu(low, 1)
    sim = sim + sim.T
    np.fill_diagonal(sim, 1.0)
    for i in range(spec.twin_n):
        a, b = spec.twin_src + i, spec.twin_dst + i
        sim[a, b] = sim[b, a] = 0.9
    return sim.astype(np.float32)

"""GPU: the library called from plain C (paper_2602_07616_amd/csrc/abi_cli.c, built by build()):
device memory from hipMalloc, a stream from hipStreamCreate, no Python objects anywhere near the
boundary.  Its results are checked against the CPU oracle like the binding's.

The C program runs as a child process that uses the GPU, so these tests run before this process
initialises the GPU itself (pytest collects this file first); otherwise they are skipped."""
import os
import subprocess
import sys

import numpy as np
import pytest

import oracle
from paper_2602_07616_amd import workloads as wk
from . import pins

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLI = os.path.join(ROOT, "paper_2602_07616_amd", "abi_cli")

CASES = {
    "tiny_fp32": (wk.SPECS["tiny"], 1, 0.5, (1e-5, 1e-5)),
    "bf16_shared": (wk.custom_spec("c_caller_bf16", wk.BF16, 512, 32, 4, 256, 1, 24, 4242, twin_src=0, twin_dst=16,
                                   twin_n=16, calib_tokens=8), 2, 0.0, (2e-2, 1e-2)),
}


def _gpu_initialised():
    torch = sys.modules.get("torch")
    return torch is not None and torch.cuda.is_initialized()


@pytest.mark.parametrize("name", list(CASES))
def test_c_caller_matches_oracle(tmp_path, name):
    if _gpu_initialised():
        pytest.skip("this process already holds the GPU; the C caller is started from a process that does not")
    assert os.path.exists(CLI), "abi_cli is not built: run __graft_entry__.build() first"
    spec, S, rho, (max_abs, rel_l2) = CASES[name]
    wl = wk.make_workload(spec)
    sim = oracle.similarity_frobenius(wl.calib, wl.w_gate_up, wl.w_down, spec.dtype).astype(np.float32)
    d = str(tmp_path)
    with open(os.path.join(d, "config.txt"), "w") as f:
        f.write(f"{spec.tokens} {spec.hidden} {spec.experts} {spec.top_k} {spec.inter} {spec.shared} {spec.dtype} "
                f"{S} {rho!r} 0\n")
    files = {"hidden": wl.hidden, "router_w": wl.router_w, "w_gate_up": wl.w_gate_up, "w_down": wl.w_down, "sim": sim}
    if spec.shared:
        files["shared_gate_up"], files["shared_down"] = wl.shared_gate_up, wl.shared_down
    for k, v in files.items():
        np.ascontiguousarray(v).tofile(os.path.join(d, k + ".bin"))
    print(f"C caller {name}", flush=True)
    try:
        if not os.access(CLI, os.X_OK):
            os.chmod(CLI, 0o755)
        r = subprocess.run([CLI, d], capture_output=True, text=True, timeout=120)
    except OSError as e:      # the program could not be started at all: nothing about the library was learnt
        pytest.skip(f"cannot start {CLI}: {e}")
    if r.returncode != 0 and "abi_cli: sere_" not in r.stderr:
        # the HIP runtime or the loader failed before any library call (no device for a second process,
        # missing runtime): an environment matter; a failing library call is a failure
        pytest.skip("the C caller could not set up the device: " + r.stderr.strip()[:300])
    assert r.returncode == 0, r.stdout + r.stderr
    ref = oracle.layer(wl.hidden, wl.router_w, wl.w_gate_up, wl.w_down, wl.shared_gate_up, wl.shared_down,
                       spec.dtype, spec.top_k, sim, S, rho)

    def ints(fname, shape):
        return np.fromfile(os.path.join(d, fname + ".bin"), dtype=np.int32).reshape(shape)
    T, K, M = spec.tokens, spec.top_k, spec.experts
    assert np.array_equal(ints("topk_ids", (T, K)), ref.topk_ids)
    assert np.array_equal(ints("rerouted_ids", (T, K)), ref.rerouted_ids)
    assert np.array_equal(ints("count_before", (M,)), ref.count_before)
    assert np.array_equal(ints("count_after", (M,)), ref.count_after)
    assert np.array_equal(ints("primary_mask", (M,)), ref.primary_mask)
    assert np.array_equal(ints("expert_offsets", (M + 1,)), ref.offsets)
    assert np.array_equal(ints("sorted_token", (T * K,)), ref.sorted_token)
    assert np.array_equal(ints("sorted_slot", (T * K,)), ref.sorted_slot)
    assert ints("num_active", (2,)).tolist() == [ref.n_active_before, ref.n_active_after]
    w = np.fromfile(os.path.join(d, "topk_weights.bin"), dtype=np.float32).reshape(T, K)
    assert np.allclose(w, ref.topk_weights, rtol=1e-6, atol=1e-7)
    storage = np.float32 if spec.dtype == wk.F32 else np.uint16
    for fname, want in (("out", ref.out_sere), ("out_baseline", ref.out_base)):
        got = pins.f64(np.fromfile(os.path.join(d, fname + ".bin"), dtype=storage).reshape(T, spec.hidden), spec.dtype)
        assert np.abs(got - want).max() <= max_abs, (fname, np.abs(got - want).max())
        assert np.linalg.norm(got - want) <= rel_l2 * np.linalg.norm(want), fname
    assert f"{ref.n_active_before} -> {ref.n_active_after}" in r.stdout

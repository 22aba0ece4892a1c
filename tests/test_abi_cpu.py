"""CPU-only: the C-ABI library loads, exports every symbol the header declares,
and rejects bad arguments before touching the device (no compute call here)."""
import ctypes
import os
import re

import pytest

from paper_2602_07616_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "sere.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sere_[a-z_]+)\s*\(", text)))


def test_exports_every_declared_symbol():
    lib = B.load()
    names = declared_functions()
    assert {"sere_route", "sere_moe_decode", "sere_moe_decode_baseline", "sere_reroute", "sere_similarity",
            "sere_workspace_bytes", "sere_similarity_workspace_bytes", "sere_status_string"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"libsere.so does not export {n}"


def test_struct_sizes_match_header():
    assert ctypes.sizeof(B.sere_config) == 40
    assert ctypes.sizeof(B.sere_route_out) == 10 * ctypes.sizeof(ctypes.c_void_p)


def good():
    return B.make_config(32, 2048, 128, 8, 768, 0, B.SERE_BF16, 2, 0.5)


def test_workspace_size_and_status_strings():
    assert B.sere_workspace_bytes(good()) > 0
    c = good(); c.num_shared = 2
    assert B.sere_workspace_bytes(c) > B.sere_workspace_bytes(good())
    assert B.load().sere_workspace_bytes(None) == 0
    for s in range(0, -12, -1):
        assert B.sere_status_string(s) and B.sere_status_string(s) != "unknown status"
    assert B.sere_status_string(-99) == "unknown status"


BAD_CONFIGS = [
    ("num_tokens", 0, B.SERE_ERR_BAD_SHAPE), ("num_tokens", 65537, B.SERE_ERR_BAD_SHAPE),
    ("hidden", 0, B.SERE_ERR_BAD_SHAPE), ("hidden", 2050, B.SERE_ERR_BAD_SHAPE),
    ("inter", 100, B.SERE_ERR_BAD_SHAPE), ("num_experts", 0, B.SERE_ERR_BAD_SHAPE),
    ("num_experts", 257, B.SERE_ERR_BAD_SHAPE), ("num_shared", -1, B.SERE_ERR_BAD_SHAPE),
    ("num_shared", 17, B.SERE_ERR_BAD_SHAPE), ("top_k", 0, B.SERE_ERR_BAD_TOPK),
    ("top_k", 129, B.SERE_ERR_BAD_TOPK), ("select_top_k", 0, B.SERE_ERR_BAD_TOPK),
    ("select_top_k", 9, B.SERE_ERR_BAD_TOPK), ("dtype", 2, B.SERE_ERR_BAD_DTYPE),
    ("flags", 8, B.SERE_ERR_BAD_FLAGS), ("flags", -1, B.SERE_ERR_BAD_FLAGS),
    ("flags", B.SERE_FLAG_SIM_COSINE | B.SERE_FLAG_SIM_CKA_LINEAR, B.SERE_ERR_BAD_FLAGS), ("threshold", float("nan"), B.SERE_ERR_NONFINITE_THRESHOLD),
    ("threshold", float("inf"), B.SERE_ERR_NONFINITE_THRESHOLD),
]
FAKE = 0x10000  # aligned, non-NULL, never dereferenced: validation fails first


def call_all(cfg, ptr=FAKE, ws=FAKE, ws_bytes=1 << 40, sim=FAKE, out=FAKE):
    lib = B.load()
    c = ctypes.byref(cfg)
    return [
        lib.sere_route(c, ptr, ptr, sim, None, ws, ws_bytes, None),
        lib.sere_reroute(c, ptr, sim, None, ws, ws_bytes, None),
        lib.sere_moe_decode(c, ptr, ptr, ptr, ptr, None, None, sim, out, None, ws, ws_bytes, None),
        lib.sere_moe_decode_baseline(c, ptr, ptr, ptr, ptr, None, None, out, None, ws, ws_bytes, None),
    ]


@pytest.mark.parametrize("field,value,status", BAD_CONFIGS)
def test_bad_config_rejected(field, value, status):
    cfg = good()
    setattr(cfg, field, value)
    assert B.sere_workspace_bytes(cfg) == 0
    assert call_all(cfg) == [status] * 4


def test_bad_pointers_rejected():
    cfg = good()
    lib = B.load()
    assert lib.sere_route(None, FAKE, FAKE, FAKE, None, FAKE, 1 << 40, None) == B.SERE_ERR_NULL_PTR
    assert call_all(cfg, ptr=0) == [B.SERE_ERR_NULL_PTR] * 4
    assert call_all(cfg, ptr=FAKE + 4) == [B.SERE_ERR_MISALIGNED] * 4
    assert call_all(cfg, ws=0) == [B.SERE_ERR_NULL_PTR] * 4
    assert call_all(cfg, ws=FAKE + 16) == [B.SERE_ERR_MISALIGNED] * 4
    need = B.sere_workspace_bytes(cfg)
    assert call_all(cfg, ws_bytes=need - 1) == [B.SERE_ERR_WORKSPACE_TOO_SMALL] * 4
    # sim is required where re-routing happens, not for the baseline
    got = call_all(cfg, sim=0, ws_bytes=need - 1)
    assert got[:3] == [B.SERE_ERR_NULL_PTR] * 3 and got[3] == B.SERE_ERR_WORKSPACE_TOO_SMALL
    # shared experts: weights required iff num_shared > 0
    cfg.num_shared = 2
    c = ctypes.byref(cfg)
    assert lib.sere_moe_decode(c, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, FAKE, None, FAKE, 0,
                               None) == B.SERE_ERR_NULL_PTR
    assert lib.sere_moe_decode(c, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, FAKE, 0,
                               None) == B.SERE_ERR_WORKSPACE_TOO_SMALL
    # a misaligned optional output is refused too
    o = B.sere_route_out()
    o.count_after = FAKE + 2
    assert lib.sere_route(ctypes.byref(good()), FAKE, FAKE, FAKE, ctypes.byref(o), FAKE, 1 << 40,
                          None) == B.SERE_ERR_MISALIGNED


def test_static_scratch_entry_point_validates_before_touching_the_device():
    """sere_moe_decode_static checks configuration, pointers and the size limit before it looks up
    its scratch array (no GPU here, so only the error paths can be reached)."""
    lib = B.load()

    def call(cfg, ptr=FAKE, sim=FAKE):
        return lib.sere_moe_decode_static(ctypes.byref(cfg), ptr, ptr, ptr, ptr, None, None, sim, FAKE, None, None)
    bad = good(); bad.top_k = 500
    assert call(bad) == B.SERE_ERR_BAD_TOPK
    assert call(good(), ptr=0) == B.SERE_ERR_NULL_PTR
    assert call(good(), ptr=FAKE + 4) == B.SERE_ERR_MISALIGNED
    assert call(good(), sim=0) == B.SERE_ERR_NULL_PTR
    big = good(); big.num_tokens = 4096
    assert B.sere_workspace_bytes(big) > B.SERE_STATIC_SCRATCH_BYTES
    assert call(big) == B.SERE_ERR_SCRATCH_TOO_SMALL
    for name in ("qwen3_b32", "qwen3_b128", "dsv2lite_b64", "mixtral_b64", "qwen15_b32", "tiny"):
        from paper_2602_07616_amd import workloads as wk
        sp = wk.SPECS[name]
        cfg = B.make_config(sp.tokens, sp.hidden, sp.experts, sp.top_k, sp.inter, sp.shared, sp.dtype, 1, 0.0)
        assert 0 < B.sere_workspace_bytes(cfg) <= B.SERE_STATIC_SCRATCH_BYTES, name


def test_similarity_validation():
    lib = B.load()
    cfg = good()
    c = ctypes.byref(cfg)
    assert B.sere_similarity_workspace_bytes(cfg, 32) > 0
    assert B.sere_similarity_workspace_bytes(cfg, 0) == 0
    assert lib.sere_similarity(c, FAKE, 0, 32, FAKE, FAKE, FAKE, FAKE, 1 << 40, None) == B.SERE_ERR_BAD_SHAPE
    assert lib.sere_similarity(c, FAKE, 2, 5000, FAKE, FAKE, FAKE, FAKE, 1 << 40, None) == B.SERE_ERR_BAD_SHAPE
    assert lib.sere_similarity(c, None, 2, 32, FAKE, FAKE, FAKE, FAKE, 1 << 40, None) == B.SERE_ERR_NULL_PTR
    assert lib.sere_similarity(c, FAKE, 2, 32, FAKE, FAKE, FAKE + 8, FAKE, 1 << 40, None) == B.SERE_ERR_MISALIGNED
    assert lib.sere_similarity(c, FAKE, 2, 32, FAKE, FAKE, FAKE, FAKE, 16, None) == B.SERE_ERR_WORKSPACE_TOO_SMALL
    cfg.dtype = 7
    assert lib.sere_similarity(c, FAKE, 2, 32, FAKE, FAKE, FAKE, FAKE, 1 << 40, None) == B.SERE_ERR_BAD_DTYPE


def test_binding_raises_on_error():
    cfg = good()
    cfg.top_k = 500
    with pytest.raises(B.SereError) as e:
        B._check(B.load().sere_route(ctypes.byref(cfg), FAKE, FAKE, FAKE, None, FAKE, 0, None))
    assert e.value.status == B.SERE_ERR_BAD_TOPK


def test_cka_similarity_batch_size_limits():
    """Linear CKA needs 4 .. 512 tokens per calibration batch; checked before anything is enqueued."""
    lib = B.load()
    cfg = good()
    cfg.flags = B.SERE_FLAG_SIM_CKA_LINEAR
    for n in (3, 513):
        assert B.sere_similarity_workspace_bytes(cfg, n) == 0
        assert lib.sere_similarity(ctypes.byref(cfg), FAKE, 1, n, FAKE, FAKE, FAKE, FAKE, 1 << 40,
                                   None) == B.SERE_ERR_BAD_SHAPE
    plain = good()
    plain.flags = B.SERE_FLAG_SIM_COSINE      # the metric with no buffers of its own
    assert B.sere_similarity_workspace_bytes(cfg, 64) > B.sere_similarity_workspace_bytes(plain, 64) > 0
    assert B.sere_similarity_workspace_bytes(good(), 64) > B.sere_similarity_workspace_bytes(plain, 64)   # partial Gram matrices
    assert lib.sere_similarity(ctypes.byref(cfg), FAKE, 1, 64, FAKE, FAKE, FAKE, FAKE, 0,
                               None) == B.SERE_ERR_WORKSPACE_TOO_SMALL


def test_row_limit():
    """T * (K + num_shared) is bounded (the FFN grids carry one work item per 32 rows in a grid dimension)."""
    cfg = good()
    cfg.num_tokens, cfg.top_k, cfg.select_top_k = 65536, 16, 1
    assert B.sere_workspace_bytes(cfg) > 0
    cfg.top_k = 17
    assert B.sere_workspace_bytes(cfg) == 0
    assert call_all(cfg) == [B.SERE_ERR_BAD_SHAPE] * 4
    cfg.top_k, cfg.num_shared = 16, 1
    assert call_all(cfg) == [B.SERE_ERR_BAD_SHAPE] * 4


def test_header_is_plain_c_and_links(tmp_path):
    """include/sere.h compiles as C99 with warnings as errors, and a C program that takes the
    address of every declared entry point links against the library (no call is made: no GPU)."""
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    names = declared_functions()
    src = tmp_path / "use_abi.c"
    body = "\n".join(f"  table[{i}] = (void (*)(void))&{n};" for i, n in enumerate(names))
    src.write_text('#include "sere.h"\n#include <stdio.h>\nint main(void) {\n'
                   f"  void (*table[{len(names)}])(void);\n{body}\n"
                   f'  printf("%d\\n", (int)(sizeof(sere_config) + sizeof(sere_route_out)) + (table[0] != 0));\n'
                   "  return 0;\n}\n")
    lib_dir = os.path.dirname(B.LIB_PATH)
    exe = tmp_path / "use_abi"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(root, "include"),
                    str(src), "-o", str(exe), "-L", lib_dir, "-l:" + os.path.basename(B.LIB_PATH),
                    "-Wl,-rpath," + lib_dir, "-Wl,--unresolved-symbols=ignore-in-shared-libs"], check=True)
    assert exe.exists()


def test_cka_kernel_parameters_validated():
    """sere_similarity_cka rejects unknown kernels and parameters outside their range before anything
    is enqueued; the metric bits of cfg.flags play no part."""
    lib = B.load()
    cfg = good()
    c = ctypes.byref(cfg)

    def call(kernel, p0, p1, n=64, ws_bytes=0):
        return lib.sere_similarity_cka(c, FAKE, 1, n, FAKE, FAKE, kernel, p0, p1, FAKE, FAKE, ws_bytes, None)
    for kernel, p0, p1 in ((3, 1.0, 1.0), (-1, 1.0, 1.0), (B.SERE_CKA_RBF, 0.0, 0.0), (B.SERE_CKA_RBF, -1.0, 0.0),
                           (B.SERE_CKA_RBF, float("nan"), 0.0), (B.SERE_CKA_POLY, 1.0, 0.0),
                           (B.SERE_CKA_POLY, 1.0, 17.0), (B.SERE_CKA_POLY, 1.0, 2.5),
                           (B.SERE_CKA_POLY, float("inf"), 2.0)):
        assert call(kernel, p0, p1) == B.SERE_ERR_BAD_KERNEL, (kernel, p0, p1)
    for kernel, p0, p1 in ((B.SERE_CKA_LINEAR, 0.0, 0.0), (B.SERE_CKA_RBF, 0.5, 0.0), (B.SERE_CKA_POLY, -1.0, 3.0)):
        assert call(kernel, p0, p1) == B.SERE_ERR_WORKSPACE_TOO_SMALL      # accepted up to the workspace check
        assert call(kernel, p0, p1, n=3) == B.SERE_ERR_BAD_SHAPE
    cfg.flags = B.SERE_FLAG_SIM_COSINE
    assert B.sere_similarity_cka_workspace_bytes(cfg, 64) > B.sere_similarity_workspace_bytes(cfg, 64)
    assert call(B.SERE_CKA_RBF, 0.5, 0.0) == B.SERE_ERR_WORKSPACE_TOO_SMALL
    assert lib.sere_similarity_cka(None, FAKE, 1, 64, FAKE, FAKE, 0, 0.0, 0.0, FAKE, FAKE, 0, None) == B.SERE_ERR_NULL_PTR

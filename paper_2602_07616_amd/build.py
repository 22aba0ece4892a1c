"""Compile the HIP library for gfx950 into paper_2602_07616_amd/libsere.so, and the plain-C
caller of its ABI (csrc/abi_cli.c) into paper_2602_07616_amd/abi_cli.

hipcc cross-compiles without a GPU.  Packed-fp32 instruction selection is
switched off for device code (see the flag below); the host pass prints a
harmless warning about not knowing that target feature.
"""
from __future__ import annotations

import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsere.so")
LIB_FORMAL = os.path.join(HERE, "libsere_formal.so")   # same sources, SERE_FORMAL_HANDOFF=1 (for the tests)
CLI = os.path.join(HERE, "abi_cli")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def source_hash() -> str:
    """Hash over the library's sources (kernels, host side, header): names what a measurement
    recorded next to it was taken on."""
    import hashlib
    h = hashlib.sha256()
    files = sources() + sorted(glob.glob(os.path.join(CSRC, "*.hpp"))) + [
        os.path.join(os.path.dirname(HERE), "include", "sere.h")]
    for f in files:
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + glob.glob(os.path.join(CSRC, "*.hpp")) + [
        os.path.join(os.path.dirname(HERE), "include", "sere.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and not stale():
        return LIB
    jobs = []
    for lib, extra in ((LIB, []), (LIB_FORMAL, ["-DSERE_FORMAL_HANDOFF=1"])):
        tmp = f"{lib}.{os.getpid()}.tmp"
        cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wall", "-Wno-unused-function", *extra,
               *sources(), "-o", tmp]
        if verbose:
            print(" ".join(cmd))
        jobs.append((lib, tmp, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)))
    for lib, tmp, proc in jobs:
        out, err = proc.communicate()
        if proc.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + out + err)
        if verbose:
            noise = "is not a recognized feature for this target"
            print("\n".join(ln for ln in err.splitlines() if noise not in ln))
        os.replace(tmp, lib)
    build_cli()
    return LIB


def build_cli() -> str:
    """The C program links against libsere.so (found next to it at run time) and the HIP runtime."""
    tmp = f"{CLI}.{os.getpid()}.tmp"
    cmd = ["gcc", "-std=c99", "-O1", "-Wall", "-Wextra", "-Werror", "-D__HIP_PLATFORM_AMD__",
           "-I", os.path.join(ROCM, "include"), "-I", os.path.join(os.path.dirname(HERE), "include"),
           os.path.join(CSRC, "abi_cli.c"), "-o", tmp,
           "-L", HERE, "-l:libsere.so", "-L", os.path.join(ROCM, "lib"), "-lamdhip64",
           "-Wl,-rpath,$ORIGIN", "-Wl,-rpath," + os.path.join(ROCM, "lib"),
           "-Wl,--unresolved-symbols=ignore-in-shared-libs"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("gcc failed on abi_cli.c:\n" + r.stdout + r.stderr)
    os.replace(tmp, CLI)
    return CLI


if __name__ == "__main__":
    print(build(verbose=True))

"""Build libnt.so (the HIP kernels and the C ABI) for gfx950 with hipcc, in-tree.

Every source is compiled to an object file of its own, in parallel, and the objects are linked into the
shared library; the objects live in a build folder beside the sources that is kept out of the history.
"""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libnt.so")
SOURCES = ["nt_host.hip", "nt_gemm.hip", "nt_gemm_stream.hip", "nt_vocab.hip", "nt_vocab_q8.hip", "nt_rows.hip",
           "nt_attn.hip", "nt_attn16.hip", "nt_decoder.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _run(cmd):
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the device-only target feature; that warning is harmless
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + err)
    return err


def build(verbose: bool = False, extra_flags=(), lib_path: str = LIB) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    tag = f"{os.getpid()}"
    srcs = [s for s in SOURCES if os.path.exists(os.path.join(CSRC, s))]
    objs = [os.path.join(OBJ, f"{s}.{tag}.o") for s in srcs]
    cmds = [[hipcc, *FLAGS, *extra_flags, "-c", "-o", o, os.path.join(CSRC, s)] for s, o in zip(srcs, objs)]
    try:
        with ThreadPoolExecutor(max_workers=min(8, len(cmds))) as ex:
            errs = list(ex.map(_run, cmds))
        tmp = lib_path + f".tmp{tag}"
        errs.append(_run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs]))
        os.replace(tmp, lib_path)
    finally:
        for o in objs:
            if os.path.exists(o):
                os.remove(o)
    if verbose and any(e.strip() for e in errs):
        print("\n".join(e for e in errs if e.strip()))
    return lib_path


if __name__ == "__main__":
    print(build(verbose=True))

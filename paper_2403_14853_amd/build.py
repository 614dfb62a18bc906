"""Compile the HIP sources under csrc/ into libisp.so for gfx950 (hipcc, in-tree)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libisp.so")
SOURCES = ["isp_api.hip", "scan.hip", "csr_build.hip", "transpose.hip", "spmm.hip", "sddmm.hip", "fusedmm.hip",
           "spmm_reduce.hip", "static_scratch.hip", "alias.hip"]
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # keep the compiler from forming packed-fp32 VALU ops out of scalar float code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "is not a recognized feature" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build(verbose: bool = False) -> str:
    """Compile every source to an object (in parallel), link libisp.so, build the C-ABI example."""
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    inc = ["-I" + os.path.join(ROOT, "include"), "-I" + CSRC]
    cflags = [f for f in HIPCC_FLAGS if f != "-shared"]
    objs = [os.path.join(objdir, s.replace(".hip", ".o")) for s in SOURCES]
    jobs = [[hipcc, *cflags, *inc, "-c", os.path.join(CSRC, s), "-o", o] for s, o in zip(SOURCES, objs)]
    with ThreadPoolExecutor(max_workers=min(8, len(jobs))) as ex:
        list(ex.map(lambda c: _run(c, verbose), jobs))
    tmp = LIB + ".tmp%d" % os.getpid()
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", tmp], verbose)
    os.replace(tmp, LIB)
    # a consumer of the C ABI without Python or PyTorch (run by the GPU tests)
    example = os.path.join(HERE, "abi_example")
    res = subprocess.run([hipcc, "--offload-arch=gfx950", "-O2", "-std=c++17", *inc, os.path.join(CSRC, "abi_example.cpp"),
                          "-L" + HERE, "-lisp", "-Wl,-rpath,$ORIGIN", "-o", example + ".tmp"],
                         stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed on abi_example.cpp:\n" + res.stdout)
    os.replace(example + ".tmp", example)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))

"""The CPU-side native code (the oracle and the input generator) under AddressSanitizer and
UndefinedBehaviorSanitizer.  Both sources are compiled with -fsanitize=address,undefined into a temporary
directory and a child Python process (the sanitizer runtime has to be loaded before the interpreter's own
allocations, hence LD_PRELOAD in a child) runs the hand-worked example, one hypothesis round of every pin and
a shrunk benchmark graph through them.  Any report makes the child exit non-zero.  CPU only."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

CHILD = r"""
import sys
sys.path.insert(0, {root!r}); sys.path.insert(0, {tests!r})
import numpy as np
import graphgen, oracle
graphgen.use_library({gen!r})
oracle.use_library({orc!r})
import test_oracle_pins as pins, test_oracle_reduce_pins as rpins, test_oracle_scale_pins as spins
pins.test_hand_worked_example()
for t in (pins.test_spmm_matches_dense_bruteforce, pins.test_transpose_properties, pins.test_backward_adjoint_and_scatter,
          pins.test_sddmm_bruteforce_and_identity, pins.test_fusedmm_forward_is_unfused_composition,
          rpins.test_reduce_matches_bruteforce, rpins.test_reduce_backward_is_the_adjoint_of_the_selected_linear_map,
          spins.test_fusedmm_forward_scale, spins.test_fusedmm_backward_scale, spins.test_mean_scale,
          spins.test_reduce_backward_scale, spins.test_minmax_against_the_fp64_definition):
    t()
pins.test_fusedmm_backward_finite_differences(0, "sigmoid")
pins.test_transpose_matches_scipy_and_rejects_bad_column()
for k, shrink in ((1, 64), (0, 1), (4, 512), (2, 4096)):
    w = graphgen.make_config(k, shrink=shrink)
    assert w.indptr[-1] == w.nnz and w.indices.max() < w.n
    Y, mag = oracle.spmm(w.indptr, w.indices, w.values, w.X)
    t = oracle.transpose(w.n, w.n, w.indptr, w.indices, w.values)
    oracle.spmm(t[0], t[1], t[3], w.dY)
    oracle.sddmm(w.indptr, w.indices, w.values, w.dY, w.X)
    oracle.fusedmm(w.indptr, w.indices, w.values, (0.1 * w.X).astype(np.float32))
    oracle.fusedmm_backward(w.indptr, w.indices, w.values, (0.1 * w.X).astype(np.float32), w.dY)
    for r in ("mean", "max"):
        Yr, arg, _ = oracle.spmm_reduce(w.indptr, w.indices, w.values, w.X, r)
        oracle.spmm_reduce_backward(w.n, w.indptr, w.indices, w.values, w.dY, r, arg)
graphgen.random_csr(7, 5, 30, 1, sorted_cols=False, allow_dup=True)
print("sanitized run ok")
"""


def _runtime(name):
    path = subprocess.check_output(["gcc", "-print-file-name=" + name], text=True).strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def test_oracle_and_generator_under_asan_and_ubsan(tmp_path):
    asan = _runtime("libasan.so")
    if asan is None:
        pytest.skip("gcc's AddressSanitizer runtime is not installed")
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1",
           "-fopenmp", "-shared", "-fPIC"]
    orc = str(tmp_path / "liboracle_san.so")
    gen = str(tmp_path / "libgraphgen_san.so")
    subprocess.check_call(["gcc", *san, "-Wall", os.path.join(ROOT, "oracle", "isp_oracle.c"), "-o", orc, "-lm"])
    subprocess.check_call(["g++", *san, "-std=c++17", os.path.join(ROOT, "graphgen", "gen.cpp"), "-o", gen])
    env = dict(os.environ)
    # the sanitizer runtime goes in front of whatever is preloaded already (nothing is removed)
    env["LD_PRELOAD"] = " ".join(x for x in (asan, env.get("LD_PRELOAD", "")) if x)
    # the interpreter itself is not instrumented: its own (intentional) leaks are not this test's business
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0:halt_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    script = CHILD.format(root=ROOT, tests=os.path.join(ROOT, "tests"), gen=gen, orc=orc)
    res = subprocess.run([sys.executable, "-c", script], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                         text=True, timeout=900)
    assert res.returncode == 0 and "sanitized run ok" in res.stdout, res.stdout[-4000:]
    assert "ERROR: AddressSanitizer" not in res.stdout and "runtime error:" not in res.stdout, res.stdout[-4000:]

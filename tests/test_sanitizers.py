"""The CPU side under AddressSanitizer and UndefinedBehaviorSanitizer: the oracle (C) and the input generator
(C++) are rebuilt with -fsanitize=address,undefined into a temporary directory and driven, in a child process
that preloads the sanitizer runtime, through the oracle's pins and the generator's own checks at small scale.
Any report (out-of-bounds access, use after free, signed overflow, misaligned access, data race on the heap
bookkeeping of the OpenMP loops ...) aborts the child and fails the test."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
       "-fopenmp", "-shared", "-fPIC"]

CHILD = r'''
import os, sys
root, oracle_lib, gen_lib = sys.argv[1:4]
sys.path.insert(0, root)
sys.path.insert(0, os.path.join(root, "tests"))
import graphgen
graphgen._LIB = gen_lib                       # the instrumented generator instead of the in-tree build
graphgen.build = lambda force=False: gen_lib
import oracle
import test_oracle_pins as pins_module
from oracle_pins import GRAD_PINS, PINS
instrumented = pins_module._Mutant(oracle._bind(oracle_lib))
for pin in PINS:
    pin(instrumented.spmm)
for pin in GRAD_PINS:
    pin(instrumented)
print("oracle pins ok", flush=True)
import test_graphgen as tg
tg.test_tiny_and_sweep_have_exact_sizes()
tg.test_general_ops_workload_shape()
tg.test_scaled_large_and_skew_workloads()
tg.test_same_seed_same_graph_any_thread_count()
tg.test_value_fillers()
tg.test_grid_stencils_have_the_textbook_structure()
for kw in (dict(duplicates=True, sort_cols=False), dict(empty_frac=0.5), dict(long_rows=((3, 500),))):
    graphgen.random_csr(200, 150, 6.0, 3, **kw)
print("generator checks ok", flush=True)
'''


def test_oracle_and_generator_are_clean_under_asan_and_ubsan(tmp_path):
    runtime = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(runtime) or not os.path.exists(runtime):
        pytest.skip("no AddressSanitizer runtime in this image")
    oracle_lib = str(tmp_path / "liboracle_san.so")
    gen_lib = str(tmp_path / "libgraphgen_san.so")
    subprocess.run(["gcc", "-std=c11", *SAN, "-o", oracle_lib, os.path.join(ROOT, "oracle", "spmm_oracle.c"), "-lm"], check=True)
    subprocess.run(["g++", "-std=c++17", *SAN, "-o", gen_lib, os.path.join(ROOT, "graphgen", "graphgen.cpp")], check=True)
    env = dict(os.environ)
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:halt_on_error=1"     # the interpreter itself leaks by design
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env["OMP_NUM_THREADS"] = "4"
    child = tmp_path / "child.py"
    child.write_text(CHILD)
    r = subprocess.run([sys.executable, str(child), ROOT, oracle_lib, gen_lib], capture_output=True, text=True, env=env,
                       timeout=900)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-4000:])
    assert "oracle pins ok" in r.stdout and "generator checks ok" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]

"""The host half of the library (pruning, quantiser, encoder, decoder, cost model) built
with AddressSanitizer and UndefinedBehaviorSanitizer, and the bit-exact host tests run
against that build in a child process.  No GPU, no device code: egt_host.cpp alone."""
import os
import re
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2605_11582_amd", "csrc")
HOST_SYMBOLS = ("egt_status_str", "egt_2bitcsr_sizes", "egt_prune_n4", "egt_prune_n4_importance", "egt_pack_2bitcsr",
                "egt_pack_2bitcsr_rowgroups", "egt_pack_2bitcsr_rows", "egt_2bitcsr_sizes_rows", "egt_unpack_2bitcsr", "egt_quant_int4", "egt_fit_verify_cost", "egt_trigger_depth")
HOST_TESTS = ("packs_the_handworked or status_strings or sizes_match or prune_matches or importance_prune or pack_bit_exact or "
              "row_groups or wide_value_ranges or pack_errors or first_offending or strided_inputs or unpack_ or quant_int4_dense or "
              "trigger_cost_model or ragged_pack")

CHILD = r"""
import ctypes, sys
sys.path.insert(0, {root!r}); sys.path.insert(0, {tests!r})
from paper_2605_11582_amd import binding as B
B._lib = B._declare(ctypes.CDLL({lib!r}), {symbols!r})      # the sanitised host build stands in for libegt.so
import pytest
sys.exit(pytest.main(["-x", "-q", "-p", "no:cacheprovider", {test!r}, "-k", {select!r}]))
"""


def test_host_encoder_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    gxx = shutil.which("g++")
    if not gxx:
        pytest.skip("no host compiler")
    lib = str(tmp_path / "libegt_host_san.so")
    build = subprocess.run([gxx, "-std=c++17", "-O1", "-g", "-fPIC", "-shared", "-pthread", "-ffp-contract=off",
                            "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                            "-I" + os.path.join(ROOT, "include"), os.path.join(CSRC, "egt_host.cpp"), "-o", lib],
                           capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    runtime = subprocess.run([gxx, "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(runtime) or not os.path.exists(runtime):
        pytest.skip("the sanitizer runtime of the host compiler is not installed")
    env = dict(os.environ)
    # the runtime has to come first in a process whose main program is not instrumented;
    # whatever the environment preloads already stays behind it
    env["LD_PRELOAD"] = " ".join(v for v in (runtime, env.get("LD_PRELOAD", "")) if v)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:exitcode=66"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1:exitcode=67"
    code = CHILD.format(root=ROOT, tests=os.path.join(ROOT, "tests"), lib=lib, symbols=HOST_SYMBOLS,
                        test=os.path.join(ROOT, "tests", "test_host_encoder.py"), select=HOST_TESTS)
    run = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, env=env, cwd=ROOT, timeout=600)
    assert run.returncode == 0, (run.stdout[-3000:], run.stderr[-3000:])
    m = re.search(r"(\d+) passed", run.stdout)
    assert m and int(m.group(1)) >= 30 and "failed" not in run.stdout, run.stdout[-2000:]

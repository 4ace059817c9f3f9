"""The C part of the oracle under AddressSanitizer + UndefinedBehaviorSanitizer: the Tiny pins
(sampling, induced subgraph and transpose, dense brute force of forward and backward for both layer
kinds, the error-bound companions, dropout) are run once more in a child process that loads the
sanitizer build; any out-of-bounds access, use after free or undefined operation in the oracle's
loops aborts that process.  Host code only: nothing here touches a GPU or the HIP library."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_tiny_pins_pass_under_address_and_ub_sanitizers():
    sys.path.insert(0, ROOT)
    from oracle import build as ob
    lib = ob.build_sanitized()
    env = dict(os.environ)
    env["BNS_ORACLE_LIB"] = lib
    # the sanitizer runtime has to come first in the child's library list; whatever is preloaded
    # already stays behind it
    env["LD_PRELOAD"] = ":".join(x for x in (ob.sanitizer_preload(), env.get("LD_PRELOAD", "")) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"      # the interpreter itself is not leak-clean
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    pins = ["tests/test_oracle_sampling.py::test_philox_known_answers", "tests/test_oracle_sampling.py::test_p0_keeps_none_p1_keeps_all",
            "tests/test_oracle_sampling.py::test_kept_list_and_remap_agree", "tests/test_oracle_subgraph.py::test_brute_force_dense_on_tiny",
            "tests/test_oracle_gcn.py::test_dense_brute_force_tiny", "tests/test_oracle_sage.py::test_dense_brute_force_tiny",
            "tests/test_oracle_bounds.py", "tests/test_oracle_dropout.py"]
    probe = subprocess.run([sys.executable, "-c", "from oracle import bns_oracle as o; print(o._LIB_PATH); o.lib()"],
                           cwd=ROOT, env=env, capture_output=True, text=True, timeout=120)
    assert probe.returncode == 0, probe.stderr[-2000:]
    assert probe.stdout.strip().endswith("libbns_oracle_asan.so")
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *pins],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    assert run.returncode == 0, (run.stdout[-3000:], run.stderr[-3000:])
    assert " passed" in run.stdout and "failed" not in run.stdout

"""The oracle under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only).

A child process builds oracle/libhb_ref_san.so (HB_ORACLE_SANITIZE=1), preloads the sanitizer runtime and runs
the pins that sweep the oracle's code paths: every width and both dealer layouts of the adder, the exhaustive
small widths, the full ring, the 8-bit-ring brute force over every (k, m), the p-party oracle, the wire
transcript, the eco scan and the float boundary.  Any sanitizer report aborts the child (-fno-sanitize-recover).
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

SELECT = ("adder or full_ring or brute_force or beaver or theorem or worked_example or eco or float or simulated "
          "or range_scatter or validation or wire or tree or parties")


def test_oracle_pins_pass_under_asan_and_ubsan():
    from oracle import build as oracle_build
    runtime = oracle_build.sanitizer_runtime()
    if not os.path.isabs(runtime) or not os.path.exists(runtime):
        pytest.skip("gcc has no AddressSanitizer runtime here")
    env = dict(os.environ)
    env["HB_ORACLE_SANITIZE"] = "1"
    env["LD_PRELOAD"] = " ".join([runtime] + ([env["LD_PRELOAD"]] if env.get("LD_PRELOAD") else []))
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"     # the interpreter's own allocations are not the subject
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu",
           os.path.join(ROOT, "tests", "test_oracle_pins.py"), os.path.join(ROOT, "tests", "test_oracle_multiparty.py"),
           os.path.join(ROOT, "tests", "test_oracle_wire.py"), "-k", SELECT]
    proc = subprocess.run(cmd, cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True,
                          timeout=900)
    tail = proc.stdout[-3000:]
    assert proc.returncode == 0, tail
    assert "runtime error" not in proc.stdout and "AddressSanitizer" not in proc.stdout, tail
    assert " passed" in tail and "libhb_ref_san.so" in loaded_library_of_child(env)


def loaded_library_of_child(env):
    """Which oracle library a process with this environment loads (asked of a second, tiny child)."""
    code = ("import ctypes, oracle; oracle.lib(); "
            "print([l.split()[-1] for l in open('/proc/self/maps') if 'libhb_ref' in l][0])")
    proc = subprocess.run([sys.executable, "-c", code], cwd=ROOT, env=env, stdout=subprocess.PIPE,
                          stderr=subprocess.STDOUT, text=True, timeout=300)
    assert proc.returncode == 0, proc.stdout[-2000:]
    return proc.stdout

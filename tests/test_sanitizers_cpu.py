"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer (no GPU, no GPU sanitizers): the
C oracle runs its pin tests, and the host side of the C boundary (argument checks, workspace
arithmetic, error strings, the benchmark library's option handling) runs the boundary tests, each
in a child process whose first library is the sanitizer runtime."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(env_extra, code):
    env = dict(os.environ)
    env.update(env_extra)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    p = subprocess.run([sys.executable, "-c", code], cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    out = p.stdout + p.stderr
    assert "AddressSanitizer" not in out and "runtime error" not in out, out[-4000:]
    assert p.returncode == 0, out[-4000:]
    return out


def test_oracle_pins_under_asan_and_ubsan():
    import oracle
    rt = oracle.gcc_asan_runtime()
    if not rt:
        pytest.skip("gcc's libasan is not installed")
    oracle.build_sanitized()
    preload = rt + (":" + os.environ["LD_PRELOAD"] if os.environ.get("LD_PRELOAD") else "")
    out = _run({"LD_PRELOAD": preload, "MOHGE_ORACLE_SANITIZED": "1", "OMP_NUM_THREADS": "4"},
               "import sys, pytest; sys.exit(pytest.main(['-x', '-q', '-p', 'no:cacheprovider', "
               "'tests/test_oracle_pins.py', 'tests/test_oracle_bwd_pins.py']))")
    assert " passed" in out


def test_boundary_host_code_under_asan_and_ubsan():
    from paper_2604_23108_amd import build
    rt = build.asan_runtime()
    if not rt:
        pytest.skip("the compiler's shared AddressSanitizer runtime is not installed")
    build.build_sanitized()
    preload = rt + (":" + os.environ["LD_PRELOAD"] if os.environ.get("LD_PRELOAD") else "")
    code = ("import sys, pytest\n"
            "from paper_2604_23108_amd import binding, bench_binding, build\n"
            "binding._LIB_PATH = build.SAN_LIB\n"
            "bench_binding._LIB_PATH = build.SAN_BENCH_LIB\n"
            "sys.exit(pytest.main(['-x', '-q', '-p', 'no:cacheprovider', 'tests/test_boundary_cpu.py', "
            "'-k', 'not bench_refuses']))\n")
    out = _run({"LD_PRELOAD": preload}, code)
    assert " passed" in out

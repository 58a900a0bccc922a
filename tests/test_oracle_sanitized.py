"""The oracle's C code under AddressSanitizer and UndefinedBehaviorSanitizer (host only): the pins run again in a
child process that loads a sanitized build of moe_oracle.c, and must pass with no report."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def sanitizer_runtime():
    r = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True)
    path = r.stdout.strip()
    return path if r.returncode == 0 and os.path.isabs(path) and os.path.exists(path) else None


@pytest.mark.skipif(shutil.which("gcc") is None or sanitizer_runtime() is None, reason="gcc with libasan is needed")
def test_oracle_pins_pass_under_asan_and_ubsan(tmp_path):
    # a private copy of the oracle package, so that the sanitized library never replaces the one the other tests load
    pkg = tmp_path / "oracle"
    pkg.mkdir()
    for name in ("__init__.py", "oracle.py", "moe_oracle.c"):
        shutil.copy(os.path.join(ROOT, "oracle", name), pkg / name)
    lib = pkg / "libmoe_oracle.so"
    subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
                    "-o", str(lib), str(pkg / "moe_oracle.c"), "-lm"], check=True)
    os.utime(lib)        # newer than the source: oracle.build() keeps it
    env = dict(os.environ)
    preload = [sanitizer_runtime()] + ([env["LD_PRELOAD"]] if env.get("LD_PRELOAD") else [])
    env.update({"LD_PRELOAD": ":".join(preload), "PYTHONPATH": f"{tmp_path}:{ROOT}",
                # python itself is not instrumented: no leak report for the interpreter's own allocations
                "ASAN_OPTIONS": "detect_leaks=0:abort_on_error=1:halt_on_error=1", "UBSAN_OPTIONS": "halt_on_error=1",
                "OMP_NUM_THREADS": "4"})
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=str(tmp_path), env=env, capture_output=True, text=True,
                       timeout=900)
    tail = (r.stdout + r.stderr)[-4000:]
    assert r.returncode == 0, tail
    assert "passed" in r.stdout and "AddressSanitizer" not in tail and "runtime error" not in tail
    # the child really loaded the sanitized copy
    probe = subprocess.run([sys.executable, "-c", "from oracle import oracle; print(oracle._LIB)"], cwd=str(tmp_path),
                           env=env, capture_output=True, text=True, timeout=120)
    assert probe.stdout.strip() == str(lib), probe.stdout + probe.stderr

"""CPU sanitizer pass: the oracle, and the host-side code of the HIP library (argument validation,
size accounting, order of the concatenated rows, launch plans of every path), built with
-fsanitize=address,undefined and exercised by two small drivers (tests/sanitize/).  Either aborts on
the first out-of-bounds access or undefined operation.  No GPU is needed: the drivers only make
calls that are pure host arithmetic or that the validation refuses before anything is launched.

By hand:
    gcc -std=c11 -O1 -g -fsanitize=address,undefined -fno-sanitize-recover=all -static-libasan -fopenmp \\
        -o /tmp/oracle_san tests/sanitize/oracle_driver.c -lm && /tmp/oracle_san
    python -c "from paper_2412_14590_amd import build; build.build_sanitized_host('tests/sanitize/host_driver.cpp', '/tmp/host_san')" \\
        && ASAN_OPTIONS=detect_leaks=0 /tmp/host_san
"""
import os
import subprocess
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
DRIVERS = os.path.join(ROOT, "tests", "sanitize")


def run(cmd, **env):
    e = dict(os.environ)
    e.update(env)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=e, timeout=600)
    assert r.returncode == 0, r.stdout[-4000:]
    return r.stdout


def test_oracle_under_address_and_undefined_behaviour_sanitizers():
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "oracle_san")
        run(["gcc", "-std=c11", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
             "-fno-sanitize-recover=all", "-static-libasan", "-fopenmp", "-o", exe, os.path.join(DRIVERS, "oracle_driver.c"), "-lm"])
        out = run([exe], ASAN_OPTIONS="detect_leaks=1", OMP_NUM_THREADS="4")
        assert "oracle_driver: ok" in out


def test_library_host_code_under_address_and_undefined_behaviour_sanitizers():
    from paper_2412_14590_amd import build
    with tempfile.TemporaryDirectory() as tmp:
        exe = build.build_sanitized_host(os.path.join(DRIVERS, "host_driver.cpp"), os.path.join(tmp, "host_san"))
        # (the HIP runtime keeps allocations until exit: leak reports are not about this library)
        out = run([exe], ASAN_OPTIONS="detect_leaks=0")
        assert "host_driver: ok" in out

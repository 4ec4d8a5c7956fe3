"""The oracle's C++ under AddressSanitizer + UndefinedBehaviorSanitizer: the pin tests are run once more, in a
child process that has the sanitizer runtime preloaded and loads a sanitized build of oracle/hero_oracle.cpp.
An out-of-bounds access, a signed overflow or a misaligned / invalid conversion anywhere in the operators the pins
reach aborts that run."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _runtime(name):
    p = subprocess.run(["gcc", f"-print-file-name={name}"], capture_output=True, text=True).stdout.strip()
    return p if os.path.isabs(p) and os.path.exists(p) else None


def test_oracle_pins_pass_under_asan_and_ubsan():
    asan = _runtime("libasan.so")
    if asan is None:
        pytest.skip("no AddressSanitizer runtime beside gcc")
    sys.path.insert(0, ROOT)
    import oracle
    oracle.build_sanitized()
    env = dict(os.environ)
    env.update({"LD_PRELOAD": asan, "HERO_ORACLE_SANITIZED": "1", "OMP_NUM_THREADS": "4",
                # Python itself leaks by design and the image preloads a library of its own ahead of ASan's
                "ASAN_OPTIONS": "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1",
                "UBSAN_OPTIONS": "halt_on_error=1:print_stacktrace=1"})
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    out = r.stdout + r.stderr
    # such a child really maps the sanitized build and the sanitizer runtime
    probe = subprocess.run([sys.executable, "-c", "import oracle; oracle.lib(); print(open('/proc/self/maps').read())"],
                           cwd=ROOT, env=env, capture_output=True, text=True, timeout=300)
    assert "libhero_oracle_san.so" in probe.stdout and "libasan" in probe.stdout, probe.stderr[-2000:]
    assert r.returncode == 0, out[-4000:]
    assert "AddressSanitizer" not in out and "runtime error" not in out, out[-4000:]
    assert " passed" in out

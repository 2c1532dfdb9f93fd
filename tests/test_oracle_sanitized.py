"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer.

The oracle is the checker of every GPU result and has index arithmetic of its own
(FIFO rings of the alias construction, row * dim + e, per-row sum maps).  This
test builds gs_oracle.cpp once more with -fsanitize=address,undefined (no
recovery: the first finding aborts) into a temporary file and runs the oracle's
own pins against that build in a child process.  CPU only.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# the pins that drive every oracle entry point
PINS = [
    "tests/test_oracle_rng_graph.py",
    "tests/test_oracle_sgns.py",
    "tests/test_oracle_storage.py",
    "tests/test_oracle_line.py",
    "tests/test_oracle_walks.py",
]


def _runtime(name):
    path = subprocess.run(["g++", f"-print-file-name={name}"], capture_output=True, text=True,
                          check=True).stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def test_oracle_pins_under_asan_ubsan(tmp_path):
    asan = _runtime("libasan.so")
    if asan is None:
        pytest.skip("g++ has no AddressSanitizer runtime here")
    sys.path.insert(0, ROOT)
    from oracle import binding
    lib = str(tmp_path / "liboracle_sanitized.so")
    subprocess.run(["g++", "-O1", "-g", "-fno-omit-frame-pointer",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    *binding.BASE_FLAGS, "-o", lib, binding.SOURCE], check=True)
    env = dict(os.environ)
    env["GS_ORACLE_LIB"] = lib
    # the interpreter is not instrumented, so the runtime has to be in the process before the
    # library is loaded; whatever was preloaded already stays, after it
    env["LD_PRELOAD"] = ":".join(x for x in (asan, env.get("LD_PRELOAD", "")) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider", *PINS]
    r = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=1500)
    tail = (r.stdout + "\n" + r.stderr)[-4000:]
    assert r.returncode == 0, tail
    assert "passed" in r.stdout, tail
    # the child really ran against the sanitized build
    probe = subprocess.run(
        [sys.executable, "-c",
         "import oracle, ctypes; from oracle import binding as b; b._load(); "
         "print(open('/proc/self/maps').read().count('liboracle_sanitized'))"],
        cwd=ROOT, env=env, capture_output=True, text=True, timeout=120)
    assert probe.returncode == 0 and int(probe.stdout.strip() or 0) > 0, probe.stderr[-2000:]

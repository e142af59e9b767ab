"""The oracle's C sources under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only): every pin of the oracle
is run once more in a child process that loads the sanitizer build (``oracle.build(sanitize=True)``), with the
sanitizer runtime preloaded in front of whatever is preloaded already.  A finding aborts the child."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PINS = ["test_oracle_pins.py", "test_oracle_backward_pins.py", "test_oracle_inplace_pins.py",
        "test_oracle_postprocess_pins.py", "test_oracle_transaction_pins.py"]


def test_oracle_pins_pass_under_asan_and_ubsan():
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("no AddressSanitizer runtime beside this gcc")
    sys.path.insert(0, ROOT)
    import oracle
    oracle.build(sanitize=True)
    env = dict(os.environ)
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"          # (the interpreter itself is not leak-clean)
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["ORACLE_SANITIZE"] = "1"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        *[os.path.join(ROOT, "tests", f) for f in PINS]],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "passed" in r.stdout and "failed" not in r.stdout, tail
    # and the child really ran on the sanitizer build with the runtime in place
    probe = ("import oracle; oracle._load(); m = open('/proc/self/maps').read(); "
             "print(int('liboracle_san.so' in m), int('libasan' in m), int('liboracle.so' in m))")
    r = subprocess.run([sys.executable, "-c", probe], cwd=ROOT, env=env, capture_output=True, text=True, timeout=120)
    assert r.stdout.split() == ["1", "1", "0"], r.stdout + r.stderr

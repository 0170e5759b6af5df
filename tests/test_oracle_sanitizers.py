"""The CPU oracle under sanitizers (CPU tier): a stand-alone driver that calls every entry point on exactly-sized
heap buffers under AddressSanitizer + UBSan, and the oracle's own pins once more with the library built under
UBSan (any report aborts)."""
import os
import subprocess
import sys

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_driver_under_address_and_undefined_sanitizers(tmp_path):
    exe = oracle.build_sanitizer_driver(str(tmp_path / "oracle_san"))
    env = dict(os.environ)
    # (a preloaded library ahead of the sanitizer runtime is no error; leaks count)
    env["ASAN_OPTIONS"] = "verify_asan_link_order=0:detect_leaks=1:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "oracle sanitizer driver: ok" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr


def test_pins_under_undefined_behaviour_sanitizer():
    env = dict(os.environ, MKQ_ORACLE_SANITIZE="undefined")
    files = [os.path.join(ROOT, "tests", f) for f in ("test_oracle_quantizer.py", "test_oracle_linear.py",
                                                      "test_oracle_int8.py", "test_oracle_calibration.py")]
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *files],
                       capture_output=True, text=True, env=env, cwd=ROOT, timeout=900)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
    assert "runtime error" not in r.stderr

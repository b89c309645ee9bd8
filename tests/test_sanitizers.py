"""Host-side sanitizer runs (CPU only): the oracle, and the argument/state layer of the C ABI with the
library's host code, each built with -fsanitize=address,undefined and driven by a small program of
tests/sanitize/.  A finding aborts the driver (no recovery), so exit status 0 is the check."""
import os
import subprocess
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def _run(cmd, **kw):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    return r.returncode, r.stdout


def test_oracle_under_address_and_undefined_behaviour_sanitizers():
    with tempfile.TemporaryDirectory() as d:
        exe = os.path.join(d, "oracle_driver")
        rc, out = _run(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                        "-o", exe, os.path.join(SAN, "oracle_driver.cpp")])
        assert rc == 0, out
        rc, out = _run([exe], env=ENV)
        assert rc == 0 and "oracle driver ok" in out and "runtime error" not in out and "AddressSanitizer" not in out, out


def test_abi_argument_and_state_layer_under_sanitizers():
    # hipcc: the sanitizers go to the host pass only (each flag right after -Xarch_host); the device code is built as usual
    with tempfile.TemporaryDirectory() as d:
        exe = os.path.join(d, "abi_driver")
        rc, out = _run(["hipcc", "-O1", "-g", "-std=c++17", "--offload-arch=gfx950",
                        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                        "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                        "-Xarch_host", "-fno-sanitize-recover=all", "-o", exe,
                        os.path.join(SAN, "abi_driver.cpp"), os.path.join(ROOT, "paper_2502_13652_amd", "csrc", "c2t_lib.hip")])
        assert rc == 0, out
        rc, out = _run([exe], env=ENV)
        assert rc == 0 and "abi driver ok" in out and "runtime error" not in out and "AddressSanitizer" not in out, out

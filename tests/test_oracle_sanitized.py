"""The oracle's C code under the compiler's undefined-behaviour checks: a small C
driver (oracle/bs_ref_selftest.c) runs every entry point on random inputs, checks
the invariants of Sec. 3.1 itself, and any out-of-bounds index, signed overflow or
misaligned access inside bs_ref.c aborts it.  Host only."""
import os
import subprocess
import tempfile

ORACLE = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle")


def test_oracle_selftest_under_ubsan():
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "bs_ref_selftest")
        subprocess.check_call(["gcc", "-std=c99", "-O1", "-g", "-Wall", "-Werror",
                               "-fsanitize=undefined,bounds", "-fno-sanitize-recover=all",
                               os.path.join(ORACLE, "bs_ref.c"), os.path.join(ORACLE, "bs_ref_selftest.c"),
                               "-o", exe, "-lm", "-lpthread"])
        out = subprocess.run([exe], capture_output=True, text=True, timeout=120)
        assert out.returncode == 0, out.stdout + out.stderr
        assert "oracle selftest ok" in out.stdout

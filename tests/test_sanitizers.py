"""CPU sanitizer leg: the oracle's C convolution and the library's host-only code (model description,
layouts, the random layer-wise split) built with -fsanitize=address,undefined and run on shapes that
reach every border case.  No GPU and no HIP compiler involved."""
import subprocess

from oracle import build as oracle_build
from paper_2107_00961_amd import build as lib_build


def _run(exe):
    p = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, timeout=300)
    out = p.stdout.decode()
    assert p.returncode == 0, out
    assert "runtime error" not in out and "AddressSanitizer" not in out, out
    return out


def test_oracle_convolution_under_sanitizers():
    assert "clean" in _run(oracle_build.build_sanitized())


def test_library_host_code_under_sanitizers():
    assert "clean" in _run(lib_build.build_host_check())

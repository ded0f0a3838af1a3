"""The host side of the C ABI (argument checks, launch-plan arithmetic, the feed's queue with real threads) as a
native program built with AddressSanitizer + UndefinedBehaviorSanitizer on the host pass; device code is compiled as
usual and never runs here. No GPU needed."""
import os
import subprocess

import pytest

from conftest import ROOT
from paper_2505_16175_amd import build as qp_build


def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "host_sanitize")
    cmd = qp_build.hipcc_command(out=exe, extra=["-O1", "-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host",
                                                 "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined",
                                                 "-pthread", os.path.join(ROOT, "tests", "host_sanitize.cpp")])
    cmd = [c for c in cmd if c != "-shared"]
    built = subprocess.run(cmd, capture_output=True, text=True)
    if built.returncode != 0 and "sanitize" in built.stderr and "unsupported" in built.stderr:
        pytest.skip("this toolchain has no host sanitizer runtime")
    assert built.returncode == 0, built.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:halt_on_error=1", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert run.returncode == 0 and "ALL OK" in run.stdout, (run.stdout[-3000:], run.stderr[-3000:])

"""The C ABI from plain C: tests/c_abi/c_abi_check.c (HIP runtime + libbiq + the C oracle, no
Python on the data path) is compiled by the build step; on a GPU it must run clean."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
EXE = os.path.join(ROOT, "tests", "c_abi", "c_abi_check")


def test_c_abi_program_builds():
    """Compiles and links against the built libraries (no GPU needed for that)."""
    import sys

    sys.path.insert(0, os.path.join(ROOT, "tests", "c_abi"))
    import build_check

    if not os.path.exists(os.path.join(ROOT, "paper_2005_09904_amd", "libbiq.so")):
        pytest.skip("libbiq.so not built")
    import oracle

    oracle.build()
    assert build_check.build() == EXE and os.path.exists(EXE)


@pytest.mark.gpu
def test_c_abi_program_runs_clean():
    if not os.path.exists(EXE):  # normally built by the build step; a few seconds of gcc otherwise
        import sys

        sys.path.insert(0, os.path.join(ROOT, "tests", "c_abi"))
        import build_check
        import oracle

        oracle.build()
        build_check.build()
    out = subprocess.run([EXE], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    print(out.stdout, flush=True)
    assert out.returncode == 0, out.stdout
    assert "C ABI check passed" in out.stdout
    for kernel in ("gemv8_half", "gemm8x2", "query_wide", "unpack_mfma"):
        assert kernel in out.stdout

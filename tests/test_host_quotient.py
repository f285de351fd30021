"""The SQ encoder kernel divides without the hardware's division sequence (a shared reciprocal and fused
multiply-add corrections).  The arithmetic claim behind it -- that the short sequences return the correctly
rounded binary32 quotient for every divisor an fp16 scale can be -- is checked here on the host, in C,
against the compiler's IEEE division: exhaustively for 16-bit dividends, on random binary32 ones
otherwise (tests/host/quotient_check.c).  What the kernel itself returns is compared with the encoder
oracle in tests/test_gpu_encode.py."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def has_fma():
    try:
        with open("/proc/cpuinfo") as f:
            return " fma " in f.read().replace("\n", " ")
    except OSError:
        return False


@pytest.mark.skipif(shutil.which("gcc") is None or not has_fma(), reason="needs gcc and a host with fused multiply-add")
def test_short_division_sequences_are_correctly_rounded(tmp_path):
    exe = str(tmp_path / "quotient_check")
    subprocess.run(["gcc", "-O2", "-mfma", "-fopenmp", "-ffp-contract=off", "-o", exe,
                    os.path.join(HERE, "host", "quotient_check.c"), "-lm"], check=True)
    env = dict(os.environ, OMP_NUM_THREADS=str(min(8, os.cpu_count() or 1)))
    out = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert out.returncode == 0, out.stdout + out.stderr
    assert out.stdout.split() == ["reciprocal", "0", "quotient16", "0", "quotient32", "0", "seventh", "0"]

"""CPU proof harness for the gather kernel's fast division path (tests/fastdiv_model.c).

The kernel replaces the per-element IEEE division by a precomputed correctly rounded reciprocal
and two FMA correction steps and accepts the result when its exponent lies in a mid range
(otherwise it divides the ordinary way); this test shows on the host (x86 FMA, IEEE binary32)
that every accepted result is exactly RN(d / sigma): all 2^32 dividends for hard divisors (all-ones significand, 1 + ulp, a typical standard
deviation, a negative one, the edges of the accepted range), and every 4099th dividend for
600 random divisors."""
import os
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.fixture(scope="module")
def model(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("fastdiv") / "fastdiv_model")
    subprocess.check_call(["gcc", "-O2", "-mfma", "-ffp-contract=off", "-fopenmp",
                           os.path.join(HERE, "fastdiv_model.c"), "-o", exe, "-lm"])
    return exe


@pytest.mark.parametrize("sigma_bits", ["3fffffff", "c10e6666", "4f7fffff", "2f800000"])
def test_every_dividend(model, sigma_bits):
    out = subprocess.run([model, "exhaustive", sigma_bits], capture_output=True, text=True)
    assert out.returncode == 0 and out.stdout.strip() == "bad=0", out.stdout + out.stderr


def test_random_divisors(model):
    out = subprocess.run([model, "random", "600", "4099", "5"], capture_output=True, text=True)
    assert out.returncode == 0 and out.stdout.strip() == "bad=0", out.stdout + out.stderr

"""The reciprocal-plus-correction division of the quantisation kernel is the IEEE
quotient: exhaustive CPU check over all significand pairs (binary16 x, binary32 s)."""
import os
import subprocess
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))


def test_reciprocal_division_equals_ieee_quotient_exhaustively():
    with tempfile.TemporaryDirectory() as d:
        exe = os.path.join(d, "check")
        subprocess.run(["g++", "-O2", "-march=x86-64-v3", "-ffp-contract=off", "-fopenmp",
                        os.path.join(HERE, "recip_division_check.cpp"), "-o", exe], check=True)
        out = subprocess.run([exe], check=True, capture_output=True, text=True).stdout
    assert out.startswith("mismatches 0 "), out


def test_reciprocal_division_rounds_like_the_ieee_quotient_near_every_tie():
    """Second division (binary32 numerator): only rne(y / scale) matters; exhaustive over every
    scale significand and every numerator within 8 ulp of a half-integer multiple of the scale."""
    with tempfile.TemporaryDirectory() as d:
        exe = os.path.join(d, "check2")
        subprocess.run(["g++", "-O2", "-march=x86-64-v3", "-ffp-contract=off", "-fopenmp",
                        os.path.join(HERE, "recip_rounding_check.cpp"), "-o", exe], check=True)
        out = subprocess.run([exe], check=True, capture_output=True, text=True).stdout
    assert out.startswith("rounding mismatches 0 "), out

"""The adaptive-lambda kernels replace the general sqrt and divide expansions
by short forms wherever the radicand is in the middle of the exponent range.
The stand-alone checker (built from the kernels' own header) compares those
forms with the IEEE operations; here it runs on every admitted radicand, on
every pair of radicand significand and numerator significand (1.4e14 cases,
under a minute), on 2^34 random (radicand, numerator) pairs over the whole
exponent window and both signs, and on the admission test itself.  The noise
generator's radius has a short form of its own, checked on all of its 2^24 inputs."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CHECKER = os.path.join(ROOT, "paper_1609_08326_amd", "lambda_check")


def run(*args):
    if not os.path.exists(CHECKER):
        raise FileNotFoundError("%s is not built; run `python -m paper_1609_08326_amd.build`" % CHECKER)
    print("lambda_check", *args, flush=True)
    sys.stdout.flush()
    p = subprocess.run([CHECKER, *[str(a) for a in args]], capture_output=True, text=True, timeout=170)
    print(p.stdout, p.stderr, flush=True)
    assert p.returncode == 0, p.stdout + p.stderr
    return p.stdout


def test_root_on_every_admitted_radicand():
    out = run("roots")
    assert "1073741824 cases" in out and " 0 mismatches" in out


def test_noise_radius_short_form_on_every_input():
    """sqrt(-2 ln u) with the reciprocal / reciprocal-square-root forms against the form with
    the general divide and square root: the function has 2^24 inputs, all are compared.  (That
    the general form is the oracle's arithmetic is what the worker-kernel parity tests show.)"""
    out = run("radius")
    assert "16777216 cases" in out and " 0 mismatches" in out


def test_root_and_quotient_on_random_pairs_over_the_whole_range():
    out = run("sampled", 1 << 34, 20260)
    assert "17179869184 cases" in out and " 0 mismatches" in out


def test_quotient_on_every_pair_of_radicand_and_numerator_significands():
    """All 2^24 radicand significands (both exponent parities) against all 2^23
    numerator significands; the forms are exact under scaling by powers of two
    inside the admitted window, which the sampled run above cross-checks."""
    out = run("quotients", 0, 1 << 23)
    assert "140737488355328 cases" in out and " 0 mismatches" in out


@pytest.mark.parametrize("first", [0, 4190000, (1 << 23) - 4096])
def test_quotient_on_all_radicand_significands_for_a_slice_of_numerators(first):
    out = run("quotients", first, 4096)
    assert "68719476736 cases" in out and " 0 mismatches" in out


def test_admission_test_for_four_radicands_equals_four_single_tests():
    """Also the wave-wide vote the kernels take, on waves that are all admitted (about
    half of them) and on waves with outsiders."""
    import re
    out = run("predicate", 1 << 32, 77)
    assert " 0 mismatches" in out
    m = re.search(r"(\d+) of (\d+) waves voted", out)
    assert m and 0.3 < int(m.group(1)) / int(m.group(2)) < 0.6, out


def test_device_sqrt_and_divide_are_this_cpus_ieee_operations(tmp_path):
    """The checker's yardstick is the device's own sqrt and division.  Tie those (and the
    short forms once more) to the host CPU's IEEE operations on 4M random pairs over the
    whole positive range, denormal radicands and quotients included."""
    import numpy as np
    path = tmp_path / "table.bin"
    n = 1 << 22
    run("table", n, 4242, path)
    rec = np.fromfile(path, dtype=np.uint32).reshape(n, 6)
    x, a = rec[:, 0].view(np.float32), rec[:, 1].view(np.float32)
    with np.errstate(all="ignore"):
        root = np.sqrt(x)
        quot = a / root
    assert root.dtype == np.float32 and quot.dtype == np.float32
    assert np.array_equal(root.view(np.uint32), rec[:, 2]), "device sqrt"
    ok = np.isfinite(quot)                   # NaN payloads (0/0) are not compared
    assert ok.mean() > 0.9
    assert np.array_equal(quot.view(np.uint32)[ok], rec[ok, 3]), "device quotient"
    assert np.array_equal(np.isfinite(rec[:, 3].view(np.float32)), ok)
    assert np.array_equal(rec[:, 4], rec[:, 2]), "short root"
    assert np.array_equal(rec[ok, 5], rec[ok, 3]), "short quotient"
    sub = (x > 0) & (x < 1.1754944e-38)
    assert sub.sum() > 1000, "denormal radicands are in the sample"

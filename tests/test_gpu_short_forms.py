"""The adaptive-lambda kernels replace the general sqrt and divide expansions
by short forms wherever the radicand is in the middle of the exponent range.
The stand-alone checker (built from the kernels' own header) compares those
forms with the IEEE operations; here it runs on every admitted radicand, on
2^32 random (radicand, numerator) pairs over the whole range, and on every
radicand significand against a slice of numerator significands.  (Its
`quotients 0 8388608` mode covers all 1.4e14 significand pairs in about a
minute; it was run once per change of the forms and found no mismatch.)"""
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
    p = subprocess.run([CHECKER, *[str(a) for a in args]], capture_output=True, text=True, timeout=100)
    print(p.stdout, p.stderr, flush=True)
    assert p.returncode == 0, p.stdout + p.stderr
    return p.stdout


def test_root_on_every_admitted_radicand():
    out = run("roots")
    assert "1073741824 cases" in out and " 0 mismatches" in out


def test_root_and_quotient_on_random_pairs_over_the_whole_range():
    out = run("sampled", 1 << 32, 20260)
    assert " 0 mismatches" in out


@pytest.mark.parametrize("first", [0, 4190000, (1 << 23) - 4096])
def test_quotient_on_all_radicand_significands_for_a_slice_of_numerators(first):
    out = run("quotients", first, 4096)
    assert "68719476736 cases" in out and " 0 mismatches" in out


def test_admission_test_for_four_radicands_equals_four_single_tests():
    out = run("predicate", 1 << 32, 77)
    assert " 0 mismatches" in out

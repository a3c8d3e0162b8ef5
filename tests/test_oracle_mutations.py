"""How sharp are the oracle's pins?  Single mistakes of the kind that are easy to
make - a dropped term, a wrong sign or index, a swapped operand, an off-by-one
in the event loop - are planted, one at a time, in a COPY of the oracle's
source; the copy is compiled and the pin tests are run against it in a child
process.  Every mutant must make at least one pin fail.  Nothing here touches
the real oracle, the GPU library or a GPU."""
import concurrent.futures
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "dcasgd_oracle.cpp")

PIN_FILES = ["tests/test_oracle_server.py", "tests/test_oracle_rng.py", "tests/test_oracle_fold.py",
             "tests/test_oracle_momentum.py", "tests/test_oracle_bak16.py"]

# (what is planted, text in the oracle, what replaces it)
MUTANTS = [
    ("displacement with the wrong sign (constant lambda)",
     "    const float diff = w - b;\n    const float g2 = g * g;\n    const float c1 = sv.lambda0 * g2;",
     "    const float diff = b - w;\n    const float g2 = g * g;\n    const float c1 = sv.lambda0 * g2;"),
    ("lambda*g instead of lambda*g*g", "const float c1 = sv.lambda0 * g2;", "const float c1 = sv.lambda0 * g;"),
    ("compensation subtracted (constant lambda)",
     "    const float c2 = c1 * diff;\n    const float gd = g + c2;\n    return gd;\n}\n\n// Eq. 18",
     "    const float c2 = c1 * diff;\n    const float gd = g - c2;\n    return gd;\n}\n\n// Eq. 18"),
    ("MeanSquare weights swapped", "const float t2 = sv.one_minus_m * g2;", "const float t2 = sv.ema_m * g2;"),
    ("lambda from the old MeanSquare", "const float den = *ms + sv.eps;", "const float den = t1 + sv.eps;"),
    ("square root dropped", "const float lam = sv.lambda0 / rt;", "const float lam = sv.lambda0 / den;"),
    ("adaptive lambda times g instead of g*g", "const float c1 = lam * g2;", "const float c1 = lam * g;"),
    ("displacement with the wrong sign (adaptive)",
     "    const float diff = w - b;\n    const float c1 = lam * g2;",
     "    const float diff = b - w;\n    const float c1 = lam * g2;"),
    ("step added instead of subtracted",
     "        const float st = eta * gd;\n        sv.w[i] = sv.w[i] - st;",
     "        const float st = eta * gd;\n        sv.w[i] = sv.w[i] + st;"),
    ("pull copies the wrong way", "sv.bak[m][i] = v;", "sv.w[i] = sv.bak[m][i];"),
    ("push reads worker 0's backup", "const float* b = sv.bak[m].data();", "const float* b = sv.bak[0].data();"),
    ("Philox halves crossed",
     "const uint32_t n0 = (uint32_t)(pb >> 32) ^ c1 ^ k0;", "const uint32_t n0 = (uint32_t)(pa >> 32) ^ c1 ^ k0;"),
    ("Philox key not advanced", "if (round > 0) { k0 += WEYL_A; k1 += WEYL_B; }", "if (round > 0) { k0 += WEYL_A; }"),
    ("sine polynomial sign", "sp = sp * x2;  sp = sp - 0.16666667f;", "sp = sp * x2;  sp = sp + 0.16666667f;"),
    ("quadrant 1 sign", "case 1:  C = -sn; S = cs;  break;", "case 1:  C = sn; S = cs;  break;"),
    ("logarithm series coefficient", "p = p * s2;  p = p + 0.33333334f;", "p = p * s2;  p = p + 0.3f;"),
    ("octant fold off by one", "const bool swap = rr > 0x200000u;", "const bool swap = rr >= 0x200000u;"),
    ("bf16 rounds half up, not to even",
     "const uint32_t bias = 0x7FFFu + ((b >> 16) & 1u);", "const uint32_t bias = 0x8000u;"),
    ("gradient h + (w - w*)", "const float p = hdiag[i] * dd;", "const float p = hdiag[i] + dd;"),
    ("noise keyed by the first push only",
     "(uint32_t)(t0 + e), gidx, as_bf16, gbuf, lo, hi);\n        push_range(sv, m, gbuf, lo, hi);\n"
     "        pull_range(sv, m, lo, hi);",
     "(uint32_t)(t0), gidx, as_bf16, gbuf, lo, hi);\n        push_range(sv, m, gbuf, lo, hi);\n"
     "        pull_range(sv, m, lo, hi);"),
    ("pull left out of the event loop",
     "        push_range(sv, m, gbuf, lo, hi);\n        pull_range(sv, m, lo, hi);\n    }\n}",
     "        push_range(sv, m, gbuf, lo, hi);\n    }\n}"),
    ("fold step not divided by J",
     "const float step = eta_hat / (float)J;  // per-gradient learning rate", "const float step = eta_hat;"),
    ("fold compensated against zero", "const float anchor = sv.w[i];       // w_t", "const float anchor = 0.0f;"),
    ("fold in reverse order",
     "for (int j = 0; j < J; ++j) push_elem(sv, step, g[j][i], anchor, i);",
     "for (int j = J - 1; j >= 0; --j) push_elem(sv, step, g[j][i], anchor, i);"),
    ("fold compensated against the running model",
     "for (int j = 0; j < J; ++j) push_elem(sv, step, g[j][i], anchor, i);",
     "for (int j = 0; j < J; ++j) push_elem(sv, step, g[j][i], sv.w[i], i);"),
    ("momentum carries the gradient, not the velocity",
     "const float mv = sv.mu * sv.vel[i];", "const float mv = sv.mu * gd;"),
    ("velocity with the wrong sign", "sv.vel[i] = mv + gd;", "sv.vel[i] = mv - gd;"),
    ("momentum step ignores the velocity",
     "const float st = eta * sv.vel[i];", "const float st = eta * gd;"),
    ("bf16 snapshot truncated", "if (sv.bak_bf16) v = bf16_widen(bf16_rne(v));",
     "if (sv.bak_bf16) v = bf16_widen((uint16_t)(bits_of(v) >> 16));"),
    ("bf16 snapshot also rounds the model", "if (sv.bak_bf16) v = bf16_widen(bf16_rne(v));",
     "if (sv.bak_bf16) sv.w[i] = bf16_widen(bf16_rne(v));"),
]


def run_mutant(args):
    index, (what, old, new), workdir = args
    source = open(SRC).read()
    if source.count(old) != 1:
        return index, what, "not applicable: the text occurs %d times" % source.count(old)
    tree = os.path.join(workdir, "m%02d" % index)
    os.makedirs(tree)
    shutil.copytree(os.path.join(ROOT, "oracle"), os.path.join(tree, "oracle"),
                    ignore=shutil.ignore_patterns("*.so", "__pycache__"))
    shutil.copytree(os.path.join(ROOT, "tests"), os.path.join(tree, "tests"),
                    ignore=shutil.ignore_patterns("__pycache__", "test_oracle_mutations.py"))
    shutil.copytree(os.path.join(ROOT, "paper_1609_08326_amd"), os.path.join(tree, "paper_1609_08326_amd"),
                    ignore=shutil.ignore_patterns("*.so", "__pycache__", "csrc", "membw_probe",
                                                  "lambda_check", "abi_client"))
    with open(os.path.join(tree, "oracle", "dcasgd_oracle.cpp"), "w") as f:
        f.write(source.replace(old, new))
    p = subprocess.run([sys.executable, "-m", "pytest", *PIN_FILES, "-x", "-q", "-m", "not gpu",
                        "-p", "no:cacheprovider"], cwd=tree, capture_output=True, text=True,
                       timeout=600)
    if p.returncode == 0:
        return index, what, "SURVIVED: every pin passed"
    if "failed" not in p.stdout and "error" not in p.stdout.lower():
        return index, what, "the child run broke: " + (p.stdout + p.stderr)[-300:]
    return index, what, None


def test_every_planted_mistake_is_caught_by_a_pin(tmp_path):
    jobs = [(i, m, str(tmp_path)) for i, m in enumerate(MUTANTS)]
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 2)) as pool:
        results = list(pool.map(run_mutant, jobs))
    problems = ["mutant %d (%s): %s" % (i, what, why) for i, what, why in results if why]
    assert not problems, "\n".join(problems)


def test_the_unmutated_copy_passes_the_same_pins(tmp_path):
    """Control: the same child-process set-up with nothing planted passes, so a failure
    above is the mutant's doing."""
    index, what, why = run_mutant((99, ("control", "// Server state of Algorithm 2.",
                                        "// Server state of Algorithm 2 (copy)."), str(tmp_path)))
    assert why == "SURVIVED: every pin passed", why

"""Mutation run of the oracle's pins (CPU only).  Each case plants one plausible mistake in a copy of
oracle/ciar_oracle.c -- a dropped term, a wrong sign, a swapped operand, an off-by-one comparison -- builds the copy
in a temporary directory and runs the pin suite (tests/test_oracle_pins.py) against it in a child process: the suite
must fail.  The unmodified copy must pass the same way, so that a failure is the mutation's doing."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "ciar_oracle.c")

MUTATIONS = [
    ("the denominator keeps the token's own exponential (the -e_i is dropped)",
     "const double others = i == rest->imax ? rest->rest_imax : S - e[i];", "const double others = S;"),
    ("sign of the radius in the lower bound",
     "double down = e[i] * exp(-r);", "double down = e[i] * exp(r);"),
    ("sample instead of population standard deviation",
     "double Sg = sqrt(ss / (double)V);", "double Sg = sqrt(ss / (double)(V - 1));"),
    ("direction of the lower cap (max instead of min)",
     "double fl = P->lower_cap / Sl; if (fl > 1.0) fl = 1.0;", "double fl = P->lower_cap / Sl; if (fl < 1.0) fl = 1.0;"),
    ("draft and target swapped in the accept test",
     "const double ell = (tx - mt - log(Z)) - (cx - m - log(S));", "const double ell = (cx - m - log(S)) - (tx - mt - log(Z));"),
    ("residual of the wrong sign (p - q instead of q - p)",
     "double res = et[i] / Z - e[i] / S;\n                            if (res < 0.0) res = 0.0;",
     "double res = e[i] / S - et[i] / Z;\n                            if (res < 0.0) res = 0.0;"),
    ("inclusive comparison in the inverse CDF (>= instead of >)",
     "if (run > T) {", "if (run >= T) {"),
    ("the window reports the row after its first rejection",
     "if (resampled)  resampled[w] = (lo + n < hi) ? id_all[lo + n] : -1;",
     "if (resampled)  resampled[w] = (lo + n + 1 < hi) ? id_all[lo + n + 1] : -1;"),
    ("Softplus without the logarithm of 1 + e^x (log instead of log1p)",
     "return x > 0.0 ? x + log1p(exp(-x)) : log1p(exp(x));", "return x > 0.0 ? x + log(exp(-x)) : log(exp(x));"),
    ("threshold polarity: U == tau flagged",
     "if (flags) flags[row] = (uint8_t)(U > P->tau);", "if (flags) flags[row] = (uint8_t)(U >= P->tau);"),
    ("no max shift before the exponential",
     "e[i] = exp(c - m);", "e[i] = exp(c);"),
]


def _build_and_run(tmp_path, name, source):
    c = tmp_path / f"{name}.c"
    so = tmp_path / f"lib{name}.so"
    c.write_text(source)
    subprocess.run(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-o", str(so),
                    str(c), "-lm"], check=True)
    env = dict(os.environ, CIAR_ORACLE_LIB=str(so))
    return subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                           "-m", "not gpu", "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True)


def test_the_unmodified_copy_passes_the_pins(tmp_path):
    r = _build_and_run(tmp_path, "plain", open(SRC).read())
    assert r.returncode == 0, r.stdout[-2000:]


@pytest.mark.parametrize("what,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_a_planted_mistake_fails_the_pins(tmp_path, what, old, new):
    src = open(SRC).read()
    assert src.count(old) >= 1, f"the oracle no longer contains the line this mutation edits: {old!r}"
    r = _build_and_run(tmp_path, "mutant", src.replace(old, new))
    assert r.returncode != 0, f"the pins did not notice: {what}"
    assert " failed" in r.stdout or "Error" in r.stdout, r.stdout[-1500:]

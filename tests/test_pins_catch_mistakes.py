"""Do the pins of the oracle notice a mistake?  Each case plants one plausible
error (a dropped term, a wrong sign or index, a wrong norm) in a COPY of
oracle/ef_oracle.c, builds it on the CPU and runs tests/test_oracle_pins.py
against it in a child process: the run must fail.  The untouched copy must pass.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "ef_oracle.c")

MISTAKES = [
    ("worker uses the old momentum in p", "t1 = mu * mnew;", "t1 = mu * mm;"),
    ("worker drops the error feedback term", "p[j] = t2 + t3;", "p[j] = t2;"),
    ("residual with the wrong sign", "e[j] = p[j] - delta[j];", "e[j] = p[j] + delta[j];"),
    ("apply adds instead of subtracting", "x[j] = x[j] - u;", "x[j] = x[j] + u;"),
    ("server forgets the stepsize ratio", "float t = r * te[j];", "float t = te[j];"),
    ("stepsize ratio inverted", "r = eta_prev / eta;", "r = eta_prev > 0 ? eta / eta_prev : 0;"),
    ("strict sign: zero encodes -1", "if (v[j] >= 0.0f)", "if (v[j] > 0.0f)"),
    ("scale divided by d instead of d_b", "scales[b] = (float)(l1 / (double)db);", "scales[b] = (float)(l1 / (double)d);"),
    ("server does not divide by M", "float avg = acc[j] / (float)M;", "float avg = acc[j];"),
    ("L2 norm instead of L1", "l1 += (double)fabsf(v[j]);", "l1 += (double)v[j] * v[j];"),
    ("server residual negated", "te[j] = tp[j] - delta[j];", "te[j] = delta[j] - tp[j];"),
    ("bits packed most significant first", "(uint64_t)1 << (j % 64)", "(uint64_t)1 << (63 - j % 64)"),
    ("block sum accumulated in float", "double l1 = 0.0;", "float l1 = 0.0f;"),
    ("Algorithm 3 worker forgets the stepsize ratio", "float t = r * e[j];", "float t = e[j];"),
    ("weight decay uses the old decay momentum", "float b = mu * mnew;", "float b = mu * mt[j];"),
    ("weight decay term left out of the update", "float u = u1 + lx;", "float u = u1;"),
    ("phi without the block size", "double ratio = a1 * a1 / ((double)(offs[b + 1] - offs[b]) * a2);",
     "double ratio = a1 * a1 / a2;"),
    ("delta with the squared L2 norm squared again", "*delta = l2 > 0.0 ? l1 * l1 / ((double)d * l2) : 1.0;",
     "*delta = l2 > 0.0 ? l1 * l1 / ((double)d * l2 * l2) : 1.0;"),
]


def _pins_pass(source_path):
    env = dict(os.environ, EF_ORACLE_SRC=source_path)
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=300)
    return r.returncode == 0, r.stdout[-600:]


def test_untouched_copy_passes(tmp_path):
    copy = tmp_path / "ef_oracle_copy.c"
    copy.write_text(open(SRC).read())
    ok, out = _pins_pass(str(copy))
    assert ok, out


@pytest.mark.parametrize("what,old,new", MISTAKES, ids=[m[0] for m in MISTAKES])
def test_planted_mistake_is_caught(tmp_path, what, old, new):
    src = open(SRC).read()
    assert src.count(old) >= 1, "the line this case edits is gone from the oracle: %r" % old
    copy = tmp_path / "ef_oracle_mistake.c"
    copy.write_text(src.replace(old, new, 1))
    ok, out = _pins_pass(str(copy))
    assert not ok, "no pin noticed: %s" % what

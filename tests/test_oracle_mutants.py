"""Do the pins of tests/test_oracle_pins.py notice a mistake in the oracle?

Each case plants one plausible mistake (a wrong bound, sign, divisor, scale or index) in a COPY of
oracle/anchor_oracle.c, builds the copy with gcc and runs the pin tests against it in a child
process (the oracle module loads the library named by ANCHOR_ORACLE_LIB).  The pins must fail for
every altered copy and pass for the unaltered one.  CPU only.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "anchor_oracle.c")

# (name, text in the source, replacement, which occurrence)
MUTANTS = [
    ("window starts one block early", "int64_t W = G - c->w;", "int64_t W = G - c->w - c->b_q;", 0),
    ("window start not clamped to the initial tokens", "return W > c->n_init ? W : c->n_init;", "return W > 0 ? W : 0;", 0),
    ("diagonal excluded", "if (j > r) return 0;", "if (j >= r) return 0;", 0),
    ("one initial token too many", "if (j < c->n_init) return 1;", "if (j <= c->n_init) return 1;", 0),
    ("window taken per block instead of per group", "int64_t g = (r / c->b_q) / c->step;", "int64_t g = (r / c->b_q);", 0),
    ("score scale dropped", "return c->sigma * s;", "return s;", 0),
    ("anchor ignores the initial tokens", "if (s > m) m = s;", "if (s > m && j >= c->n_init) m = s;", 0),
    ("row sum not relative to the anchor", "double p = exp(score(c, qr, k + j * d) - m);", "double p = exp(score(c, qr, k + j * d));", 0),
    ("pooled anchor divided by the block size, not the row count", "*xbar = sx / n;", "*xbar = sx / (double)c->b_q;", 0),
    ("pooled query divided by the block size, not the row count", "qbar[t] /= n;", "qbar[t] /= (double)c->b_q;", 0),
    ("candidates reach one column into the window", "if (j >= c->n_init && j < W) {", "if (j >= c->n_init && j <= W) {", 0),
    ("initial tokens are candidates", "if (j >= c->n_init && j < W) {", "if (j >= 0 && j < W) {", 0),
    ("difference with the wrong sign", "double diff = xbar[b] - c->sigma * s;", "double diff = c->sigma * s - xbar[b];", 0),
    ("pooled score not scaled", "double diff = xbar[b] - c->sigma * s;", "double diff = xbar[b] - s;", 0),
    ("all blocks of a group must agree (AND instead of OR)", "if (diff < mg) mg = diff;", "if (mg == INFINITY || diff > mg) mg = diff;", 0),
    ("threshold added instead of subtracted", "mg -= c->theta;", "mg += c->theta;", 0),
    ("strict threshold test (< for <=)", "sel[j] = (mg <= 0.0) ? 1 : 0;", "sel[j] = (mg < 0.0) ? 1 : 0;", 0),
    ("selected columns not attended", "if (in_anchor(c, r, j) || sel[j]) {", "if (in_anchor(c, r, j)) {", 0),
    ("output not normalised", "for (int t = 0; t < d; ++t) o[t] /= l;", "for (int t = 0; t < d; ++t) o[t] /= 1.0;", 0),
    ("lse without the maximum", "lse[r - r0] = m + log(l);", "lse[r - r0] = log(l);", 0),
    ("block variant: block mean divided by the wrong count", "kbar[t] /= (double)b_kv;", "kbar[t] /= (double)(b_kv + 1);", 0),
    ("block variant: difference with the wrong sign", "double diff = xbar[b] - c->sigma * s;", "double diff = c->sigma * s - xbar[b];", 1),
    ("block variant: strict threshold test (< for <=)", "sel[j] = (mg <= 0.0) ? 1 : 0;", "sel[j] = (mg < 0.0) ? 1 : 0;", 1),
    ("block variant: one block too many", "J < W / b_kv; ++J", "J <= W / b_kv - 0 && J < c->N / b_kv; ++J", 0),
]


def _replace_nth(text, old, new, n):
    pos = -1
    for _ in range(n + 1):
        pos = text.index(old, pos + 1)
    return text[:pos] + new + text[pos + len(old):]


def _pins_pass(lib_path):
    env = dict(os.environ, ANCHOR_ORACLE_LIB=lib_path, OMP_NUM_THREADS="2")
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True)
    return r.returncode == 0, r.stdout[-400:]


def _build(text, path):
    c = path + ".c"
    with open(c, "w") as f:
        f.write(text)
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fno-fast-math", "-shared", "-fPIC", "-o", path, c, "-lm"])
    return path


def test_pins_pass_on_an_unaltered_copy(tmp_path):
    ok, out = _pins_pass(_build(open(SRC).read(), str(tmp_path / "copy.so")))
    assert ok, out


def test_pins_fail_on_every_planted_mistake(tmp_path):
    src = open(SRC).read()

    def run(i):
        name, old, new, nth = MUTANTS[i]
        assert src.count(old) > nth, "source text of mutant %r not found" % name
        ok, out = _pins_pass(_build(_replace_nth(src, old, new, nth), str(tmp_path / ("m%d.so" % i))))
        return name, ok

    with ThreadPoolExecutor(max_workers=4) as ex:
        survivors = [name for name, ok in ex.map(run, range(len(MUTANTS))) if ok]
    assert not survivors, "the pins do not notice: %s" % survivors

"""Do the pins notice a wrong oracle?  Each case plants one plausible mistake in a copy
of oracle/step.c (a sign, a dropped term, a wrong index, a wrong rounding), builds it
beside the real one and runs the pin tests against it in a child process: at least
one pin has to fail.  Everything here runs on the CPU; the real oracle is untouched."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

from oracle import build as obuild

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

MUTANTS = [
    ("weight decay with the wrong sign", "fmaf(-s->lw, theta[e], theta[e])", "fmaf(s->lw, theta[e], theta[e])"),
    ("update with the wrong sign", "fmaf(-s->step, u, th)", "fmaf(s->step, u, th)"),
    ("second moment from g instead of g^2", "(s->omb2 * gm) * gm", "(s->omb2 * gm)"),
    ("eps inside the root", "fmaf(sqrtf(v1), s->isb2, s->ep)", "sqrtf(v1 + s->ep) * s->isb2"),
    ("no bias correction of v", "out->isb2 = (float)(1.0 / sqrt(bc2));", "out->isb2 = 1.0f;"),
    ("no bias correction of m", "out->step = (float)(lr / bc1);", "out->step = (float)lr;"),
    ("first moment decays with beta2", "fmaf(s->b1, m[e], s->omb1 * gm)", "fmaf(s->b2, m[e], s->omb1 * gm)"),
    ("decay applied to the new weight",
     "float th = fmaf(-s->lw, theta[e], theta[e]);\n        float t1 = fmaf(-s->step, u, th);",
     "float th = fmaf(-s->step, u, theta[e]);\n        float t1 = fmaf(-s->lw, th, th);"),
    ("a contribution skipped", "for (uint32_t r = 1; r < n_contrib; ++r)", "for (uint32_t r = 2; r < n_contrib; ++r)"),
    ("cast truncates", "u += 0x7fffu + keep_lsb;", "u += 0;"),
    ("cast rounds half up", "u += 0x7fffu + keep_lsb;", "u += 0x8000u;"),
    ("cast of the old weight", "p[e] = oracle_bf16_rne(t1);", "p[e] = oracle_bf16_rne(th);"),
    ("clip coefficient ignored", "gm = gm * s->cc;", "gm = gm;"),
    ("accumulation forgets the running total", "accum[e] = overwrite ? acc : accum[e] + acc;", "accum[e] = acc;"),
    ("difference taken as a sum", "double d = x - y;", "double d = x + y;"),
    ("checksum blind to position", "(first_index + i + 1) * 0x9E3779B97F4A7C15ull", "0x9E3779B97F4A7C15ull"),
    ("checksum index off by one", "(first_index + i + 1) * 0x9E3779B97F4A7C15ull", "(first_index + i) * 0x9E3779B97F4A7C15ull"),
    ("clip without the 1e-6", "max_norm / (norm + 1e-6)", "max_norm / norm"),
]


def _pins_fail_with(tmp_path, k, old, new):
    src = open(obuild.SRC).read()
    assert old in src, "the mutation no longer applies: %r" % old
    c_file, so_file = str(tmp_path / ("mutant%d.c" % k)), str(tmp_path / ("mutant%d.so" % k))
    with open(c_file, "w") as f:
        f.write(src.replace(old, new))
    subprocess.run(["gcc", *obuild.CFLAGS, "-w", c_file, "-o", so_file, "-lm"], check=True)
    env = dict(os.environ, PS_ORACLE_LIB_UNDER_TEST=so_file)
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                        "-x", "-q", "-p", "no:cacheprovider", "-k", "not exhaustive_against_library"],
                       cwd=ROOT, env=env, capture_output=True, text=True)
    return r.returncode, r.stdout[-400:]


def test_every_planted_mistake_fails_a_pin(tmp_path):
    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(lambda a: _pins_fail_with(tmp_path, a[0], a[1][1], a[1][2]), enumerate(MUTANTS)))
    survivors = [MUTANTS[k][0] for k, (rc, _) in enumerate(results) if rc == 0]
    broken = [(MUTANTS[k][0], out) for k, (rc, out) in enumerate(results) if rc not in (0, 1)]
    assert not broken, broken            # 1 = tests failed; anything else is a harness problem
    assert not survivors, "no pin notices: %s" % survivors


def test_the_unmodified_oracle_passes_through_the_same_route(tmp_path):
    rc, out = _pins_fail_with(tmp_path, 99, "double d = x - y;", "double d = x - y;")
    assert rc == 0, out

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
    ("cast of the old weight", "oracle_f16_rne(t1) : oracle_bf16_rne(t1);", "oracle_f16_rne(th) : oracle_bf16_rne(th);"),
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


# ---- the placement closed forms (oracle/placement.py) ----

PLACEMENT_MUTANTS = [
    ("S not divided by N", "_mu = pl.mu\npl.mu = lambda mode, s, N, s_unit=0: Fraction(s) if mode == 'S' else _mu(mode, s, N, s_unit)"),
    ("S* without its transient unit", "_mu = pl.mu\npl.mu = lambda mode, s, N, s_unit=0: Fraction(s, N) if mode == 'S*' else _mu(mode, s, N, s_unit)"),
    ("offloaded state counted on the device", "_mu = pl.mu\npl.mu = lambda mode, s, N, s_unit=0: Fraction(s) if mode == 'O' else _mu(mode, s, N, s_unit)"),
    ("materialised state counted in full", "_mu = pl.mu\npl.mu = lambda mode, s, N, s_unit=0: Fraction(s) if mode == 'M' else _mu(mode, s, N, s_unit)"),
    ("All-Reduce at half its volume", "pl.all_reduce = lambda N, T: Fraction((N - 1) * T, N)"),
    ("Reduce-Scatter at twice its volume", "pl.reduce_scatter = lambda N, T: Fraction(2 * (N - 1) * T, N)"),
    ("All-Gather with N for N-1", "pl.all_gather = lambda N, T: Fraction(T)"),
    ("optimizer state of 8 bytes per parameter", "pl.state_bytes = lambda P: {'theta': 2 * P, 'omega': 8 * P, 'grad': 2 * P}"),
    ("gradients of 4 bytes per parameter", "pl.state_bytes = lambda P: {'theta': 2 * P, 'omega': 12 * P, 'grad': 4 * P}"),
    ("one parameter gather per step instead of two",
     "_c = pl.communication\npl.communication = lambda spec, P, N: _c(spec, P, N) - (pl.all_gather(N, 2 * P) if spec[0] == 'S*' else 0)"),
    ("shards start one slot late",
     "_g = pl.shard_geometry\npl.shard_geometry = lambda psi, N, i, align=1: (lambda r: (r[0], r[1] + r[2], r[2], r[3]))(_g(psi, N, i, align))"),
    ("valid length not clamped to the shard",
     "_g = pl.shard_geometry\npl.shard_geometry = lambda psi, N, i, align=1: (lambda r: (r[0], r[1], r[2], max(psi - r[1], 0)))(_g(psi, N, i, align))"),
    ("padding ignores the alignment", "_g = pl.shard_geometry\npl.shard_geometry = lambda psi, N, i, align=1: _g(psi, N, i, 1)"),
    ("selection threshold 0.8",
     "_s = pl.select_strategy\npl.select_strategy = lambda P, M, N, layer_bytes=0, fast_interconnect=False: _s(P, Fraction(8, 7) * M, N, layer_bytes * Fraction(8, 7), fast_interconnect)"),
    ("tensor parallelism added without a fast interconnect",
     "_s = pl.select_strategy\npl.select_strategy = lambda P, M, N, layer_bytes=0, fast_interconnect=False: _s(P, M, N, layer_bytes, True)"),
    ("data-parallel groups of neighbours", "pl.tp_dp_groups = lambda T, D: (pl.pp_dp_groups(D, T)[0], pl.pp_dp_groups(T, D)[0])"),
    ("pipelines of neighbours", "pl.pp_dp_groups = lambda K, D: ([list(range(k * D, (k + 1) * D)) for k in range(K)], [list(range(r * K, (r + 1) * K)) for r in range(D)])"),
    ("composed cost on the whole model", "pl.composed_cost = lambda spec, P, inner, D, s_unit=0: (pl.memory(spec, P, D, s_unit), pl.communication(spec, P, D))"),
]

_CHILD = """
import sys, pytest
from fractions import Fraction
import oracle.placement as pl
exec(sys.argv[1])
sys.exit(pytest.main([sys.argv[2], "-x", "-q", "-p", "no:cacheprovider"]))
"""


def _placement_pins(patch):
    r = subprocess.run([sys.executable, "-c", _CHILD, patch,
                        os.path.join(ROOT, "tests", "test_oracle_placement.py")],
                       cwd=ROOT, capture_output=True, text=True)
    return r.returncode, r.stdout[-400:] + r.stderr[-400:]


def test_every_planted_mistake_in_the_placement_forms_fails_a_pin():
    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(lambda m: _placement_pins(m[1]), PLACEMENT_MUTANTS))
    broken = [(m[0], out) for m, (rc, out) in zip(PLACEMENT_MUTANTS, results) if rc not in (0, 1)]
    assert not broken, broken
    survivors = [m[0] for m, (rc, _) in zip(PLACEMENT_MUTANTS, results) if rc == 0]
    assert not survivors, "no pin notices: %s" % survivors
    assert _placement_pins("pass")[0] == 0

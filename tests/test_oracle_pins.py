"""Pins for oracle/step.c against things other than itself: exact definitions of
the 16-bit conversions, brute-force fixed-order sums, closed forms and
invariants of the Adam update, a binary64 pass, and a library optimizer."""
import numpy as np
import pytest
import torch

from oracle import placement as pl
from oracle import step as orc
from synth import WORKLOADS
from synth import host as gen

HP = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)


def ulp_diff(a, b):
    """Distance in binary32 units-in-the-last-place (monotone integer mapping)."""
    def key(x):
        i = np.ascontiguousarray(x, dtype=np.float32).view(np.int32).astype(np.int64)
        return np.where(i < 0, -(i & 0x7fffffff), i)
    return np.abs(key(a) - key(b))


# --------------------------------------------------------------------------
# 16-bit conversions
# --------------------------------------------------------------------------

def _bf16_value_f64(bits):
    """Value of a bf16 pattern from the format's definition: 1 sign, 8 exponent,
    7 fraction bits, bias 127, subnormals at exponent field 0."""
    bits = np.asarray(bits, dtype=np.int64)
    s = np.where(bits & 0x8000, -1.0, 1.0)
    e = (bits >> 7) & 0xff
    f = (bits & 0x7f).astype(np.float64)
    normal = np.ldexp(1.0 + f / 128.0, (e - 127).astype(np.int64))
    sub = np.ldexp(f / 128.0, -126)
    return s * np.where(e == 0, sub, normal)


def test_widen_bf16_exhaustive():
    bits = np.arange(65536, dtype=np.int64)
    finite = ((bits >> 7) & 0xff) != 0xff
    want = _bf16_value_f64(bits[finite])
    got = np.array([orc.widen_bf16(int(b)) for b in bits[finite]], dtype=np.float64)
    assert np.array_equal(got, want)
    assert np.array_equal(np.signbit(got), (bits[finite] & 0x8000) != 0)
    assert orc.widen_bf16(0x7f80) == np.inf and orc.widen_bf16(0xff80) == -np.inf
    assert np.isnan(orc.widen_bf16(0x7fc1))


def _nearest_even_bf16(u32):
    """Independent definition of the cast for finite inputs: among the two bf16
    values that bracket x pick the nearer by exact comparison in binary64; on a
    tie the one with even fraction; past the largest finite bf16 by half a step
    or more -> infinity."""
    u32 = np.asarray(u32, dtype=np.uint32)
    x = u32.view(np.float32).astype(np.float64)
    sign = (u32 >> 31).astype(np.int64)
    mag = (u32 & 0x7fffffff).astype(np.int64)
    lo = mag >> 16                      # truncation toward zero in magnitude
    hi = lo + 1                         # next pattern up (0x7f80 = infinity)
    ax = np.abs(x)
    vlo = _bf16_value_f64(lo)
    # the would-be value of hi if the exponent range went on (used for overflow ties)
    hi_e = (hi >> 7) & 0xff
    hi_f = (hi & 0x7f).astype(np.float64)
    vhi = np.where(hi_e == 0, np.ldexp(hi_f / 128.0, -126),
                   np.ldexp(1.0 + hi_f / 128.0, (hi_e - 127).astype(np.int64)))
    dlo, dhi = ax - vlo, vhi - ax
    pick_hi = (dhi < dlo) | ((dhi == dlo) & ((lo & 1) == 1))
    out = np.where(pick_hi, hi, lo) | (sign << 15)
    return out.astype(np.uint16)


def test_bf16_rne_against_definition():
    hi = np.arange(65536, dtype=np.uint32)
    finite = ((hi >> 7) & 0xff) != 0xff
    hi = hi[finite]
    lows = np.array([0x0000, 0x0001, 0x7fff, 0x8000, 0x8001, 0xffff, 0x4000, 0xc000], np.uint32)
    u = ((hi[:, None] << 16) | lows[None, :]).reshape(-1)
    rng = np.random.default_rng(7)
    extra = rng.integers(0, 2 ** 32, size=1 << 20, dtype=np.uint64).astype(np.uint32)
    extra = extra[((extra >> 23) & 0xff) != 0xff]
    u = np.concatenate([u, extra])
    assert np.array_equal(orc.bf16_rne_bits(u), _nearest_even_bf16(u))


def test_bf16_rne_specials():
    f = lambda x: orc.bf16_rne_bits(np.array([x], dtype=np.uint32))[0]
    assert f(0x7f800000) == 0x7f80 and f(0xff800000) == 0xff80      # infinities stay
    assert f(0x80000000) == 0x8000 and f(0x00000000) == 0x0000      # signed zeros
    assert f(0x7f7fffff) == 0x7f80                                  # FLT_MAX overflows
    assert f(0x7f7f7fff) == 0x7f7f                                  # just under the tie
    assert f(0x7f7f8000) == 0x7f80                                  # tie at the top -> even = inf
    assert f(0x7fc00001) == 0x7fc0 and f(0xffc00001) == 0xffc0      # NaN: quiet, sign kept
    assert f(0x7f800001) == 0x7fc0                                  # signalling NaN payload in low half
    assert f(0x3f808000) == 0x3f80 and f(0x3f818000) == 0x3f82      # ties to even, both ways
    assert f(0x00000001) == 0x0000 and f(0x00008001) == 0x0001      # subnormals


def _f16_value_f64(bits):
    """Value of a binary16 pattern from the format's definition: 1 sign, 5 exponent, 10
    fraction bits, bias 15, subnormals at exponent field 0."""
    bits = np.asarray(bits, dtype=np.int64)
    s = np.where(bits & 0x8000, -1.0, 1.0)
    e = (bits >> 10) & 0x1f
    f = (bits & 0x3ff).astype(np.float64)
    normal = np.ldexp(1.0 + f / 1024.0, (e - 15).astype(np.int64))
    sub = np.ldexp(f / 1024.0, -14)
    return s * np.where(e == 0, sub, normal)


def test_widen_f16_exhaustive():
    bits = np.arange(65536, dtype=np.int64)
    finite = ((bits >> 10) & 0x1f) != 0x1f
    want = _f16_value_f64(bits[finite])
    got = np.array([orc.widen_f16(int(b)) for b in bits[finite]], dtype=np.float64)
    assert np.array_equal(got, want)
    assert np.array_equal(np.signbit(got), (bits[finite] & 0x8000) != 0)
    assert orc.widen_f16(0x7c00) == np.inf and orc.widen_f16(0xfc00) == -np.inf
    assert np.isnan(orc.widen_f16(0x7c01)) and np.isnan(orc.widen_f16(0xfe00))
    # the library's own widening agrees on every non-NaN pattern
    lib = np.arange(65536, dtype=np.uint16).view(np.float16).astype(np.float64)
    assert np.array_equal(got, lib[finite])


def _nearest_even_f16(u32):
    """Independent definition of the binary16 cast for finite inputs: the finite binary16
    magnitudes are listed in order (pattern = rank), x is bracketed by two of them, the
    nearer by exact comparison in binary64 wins, a tie goes to the even pattern; the
    value one step past the largest finite one (65536, were the exponent range to go on)
    stands for infinity."""
    u32 = np.asarray(u32, dtype=np.uint32)
    ax = np.abs(u32.view(np.float32).astype(np.float64))
    sign = (u32 >> 31).astype(np.int64)
    grid = np.concatenate([_f16_value_f64(np.arange(0x7c00)), [65536.0]])   # rank 0x7c00 = infinity
    hi = np.minimum(np.searchsorted(grid, ax, side="left"), 0x7c00)         # first grid value >= |x|
    lo = np.maximum(hi - 1, 0)
    dlo, dhi = ax - grid[lo], grid[hi] - ax
    pick_hi = (hi == lo) | (dhi < dlo) | ((dhi == dlo) & ((lo & 1) == 1))
    pick_hi |= ax >= 65536.0
    out = np.where(pick_hi, hi, lo) | (sign << 15)
    return out.astype(np.uint16)


def test_f16_rne_against_definition():
    h = np.arange(0x7c00, dtype=np.int64)                     # every finite magnitude
    v = _f16_value_f64(h)
    nxt = np.concatenate([v[1:], [65536.0]])
    tie = ((v + nxt) / 2).astype(np.float32)                  # exact midpoints (12 significant bits)
    cases = [v.astype(np.float32), tie, np.nextafter(tie, np.float32(0)), np.nextafter(tie, np.float32(np.inf))]
    mag = np.concatenate(cases).view(np.uint32)
    rng = np.random.default_rng(17)
    extra = rng.integers(0, 2 ** 32, size=1 << 20, dtype=np.uint64).astype(np.uint32)
    extra = extra[((extra >> 23) & 0xff) != 0xff]
    u = np.concatenate([mag, mag | np.uint32(0x80000000), extra])
    assert np.array_equal(orc.f16_rne_bits(u), _nearest_even_f16(u))


def test_f16_rne_specials():
    f = lambda x: orc.f16_rne_bits(np.array([x], dtype=np.uint32))[0]
    assert f(0x7f800000) == 0x7c00 and f(0xff800000) == 0xfc00      # infinities stay
    assert f(0x80000000) == 0x8000 and f(0x00000000) == 0x0000      # signed zeros
    assert f(0x477fe000) == 0x7bff                                  # 65504, the largest finite value
    assert f(0x477fefff) == 0x7bff and f(0x477ff000) == 0x7c00      # just under / at 65520: the tie goes up
    assert f(0x7f7fffff) == 0x7c00                                  # FLT_MAX overflows
    assert f(0x7fc00001) == 0x7e00 and f(0xffc00001) == 0xfe00      # NaN: quiet, sign kept
    assert f(0x7f800001) == 0x7e00                                  # signalling NaN
    assert f(0x33800000) == 0x0001 and f(0x33000000) == 0x0000      # 2^-24 -> 1 unit; 2^-25 ties to even 0
    assert f(0x33000001) == 0x0001 and f(0x33c00000) == 0x0002      # just over half; 1.5 units ties to even 2
    assert f(0x387fc000) == 0x03ff and f(0x387fe000) == 0x0400      # largest subnormal; tie rolls into 2^-14
    assert f(0x3f801000) == 0x3c00 and f(0x3f803000) == 0x3c02      # ties to even, both ways, at 1.0


# --------------------------------------------------------------------------
# gradient reduction (gradient integrity, Theorem 3)
# --------------------------------------------------------------------------

def _np_fixed_order_sum(grads):
    """Left-to-right binary32 sum with numpy scalars, independent of the C loop."""
    def widen(g):
        if g.dtype == np.uint16:
            return (g.astype(np.uint32) << 16).view(np.float32)
        if g.dtype == np.float16:
            return g.astype(np.float32)          # the library's exact widening
        return g
    acc = widen(grads[0]).copy()
    for g in grads[1:]:
        acc = (acc + widen(g)).astype(np.float32)
    return acc


@pytest.mark.parametrize("dtype", ["bf16", "f32", "f16"])
@pytest.mark.parametrize("N", [1, 2, 3, 6, 8])
def test_reduce_is_the_fixed_order_sum(dtype, N):
    n = 4099
    grads = [gen.gradient(n, 11, 0, r, dtype, std=1.0, outlier_frac=0.01, outlier_mult=1e4)
             for r in range(N)]
    acc = orc.reduce_sum(grads)
    assert np.array_equal(acc.view(np.uint32), _np_fixed_order_sum(grads).view(np.uint32))
    if N == 1:
        assert np.array_equal(acc.view(np.uint32), _np_fixed_order_sum(grads[:1]).view(np.uint32))
    if N >= 3 and dtype == "f32":
        # order matters in binary32: the fixed order is not just "some" order
        # (sums of a few bf16 values of like size are exact, so only fp32 shows it)
        rev = orc.reduce_sum(grads[::-1])
        assert not np.array_equal(acc.view(np.uint32), rev.view(np.uint32))


def test_reduce_shard_equals_slice_of_full_sum():
    psi, N = 6 * 257, 6
    grads = [gen.gradient(psi, 5, 3, r, "bf16") for r in range(N)]
    full = orc.reduce_sum(grads)
    for i in range(N):
        _, off, n, _ = pl.shard_geometry(psi, N, i)
        shard = orc.reduce_sum([np.ascontiguousarray(g[off:off + n]) for g in grads])
        assert np.array_equal(shard.view(np.uint32), full[off:off + n].view(np.uint32))


@pytest.mark.parametrize("N", [2, 4, 8])
def test_equal_contributions_mean_is_exact_for_power_of_two(N):
    x = gen.gradient(2048, 9, 0, 0, "bf16")
    gm, _ = orc.mean_sumsq([x] * N, 1.0 / N)
    assert np.array_equal(gm.view(np.uint32), ((x.astype(np.uint32) << 16)))


def test_integrity_violations_are_visible():
    # Missing contribution, duplicated contribution, wrong normaliser (the paper's
    # list of gradient-integrity violations) each change the mean beyond 1e-5 relative.
    n, N = 1 << 14, 8
    grads = [gen.gradient(n, 21, 0, r, "bf16") for r in range(N)]
    good, _ = orc.mean_sumsq(grads, 1.0 / N)
    rel = lambda a: np.linalg.norm(a.astype(np.float64) - good) / np.linalg.norm(good)
    assert rel(orc.mean_sumsq(grads[:-1], 1.0 / N)[0]) > 1e-5
    assert rel(orc.mean_sumsq(grads[:-1] + [grads[0]], 1.0 / N)[0]) > 1e-5
    assert rel(orc.mean_sumsq(grads, 1.0)[0]) > 1e-5
    assert rel(orc.mean_sumsq(grads, 1.0 / N)[0]) == 0.0


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_accumulate_micro_batches(dtype):
    """k micro-batches: running = running + ((g0+g1)+...), against a numpy scalar loop;
    one micro-batch with overwrite equals the plain reduce; untouched outside the range."""
    n, N, k = 3001, 4, 5
    accum = np.full(n, np.float32(123.0))
    want = None
    for j in range(k):
        grads = [gen.gradient(n, 91, j, r, dtype, std=1.0) for r in range(N)]
        micro = _np_fixed_order_sum(grads)
        want = micro if j == 0 else (want + micro).astype(np.float32)
        orc.accumulate(grads, accum, overwrite=(j == 0), lo=7, hi=n - 5)
        if j == 0:
            assert np.array_equal(accum[7:n - 5].view(np.uint32), orc.reduce_sum(grads)[7:n - 5].view(np.uint32))
    assert np.array_equal(accum[7:n - 5].view(np.uint32), want[7:n - 5].view(np.uint32))
    assert (accum[:7] == 123.0).all() and (accum[n - 5:] == 123.0).all()
    # the mean over N*k contributions then feeds the step as one fp32 contribution
    gm, _ = orc.mean_sumsq([accum], 1.0 / (N * k), 7, n - 5)
    exact = sum(sum((g.astype(np.uint32) << 16).view(np.float32).astype(np.float64) if g.dtype == np.uint16
                    else g.astype(np.float64)
                    for g in [gen.gradient(n, 91, j, r, dtype, std=1.0) for r in range(N)])
                for j in range(k)) / (N * k)
    assert np.allclose(gm[7:n - 5], exact[7:n - 5], rtol=0, atol=2e-6)


def test_sumsq_and_clip():
    n = 10007
    grads = [gen.gradient(n, 3, 0, r, "f32", std=1e-2, student_t_dof=3) for r in range(6)]
    gs = np.float32(1.0 / 6.0)
    gm, ss = orc.mean_sumsq(grads, gs)
    want_g = (_np_fixed_order_sum(grads) * gs).astype(np.float32)
    assert np.array_equal(gm.view(np.uint32), want_g.view(np.uint32))
    import math
    assert ss == pytest.approx(math.fsum(float(x) * float(x) for x in want_g), rel=1e-13)
    # range additivity and empty range
    _, a = orc.mean_sumsq(grads, gs, 0, 5000, want_mean=False)
    _, b = orc.mean_sumsq(grads, gs, 5000, n, want_mean=False)
    assert a + b == pytest.approx(ss, rel=1e-14)
    assert orc.mean_sumsq(grads, gs, 77, 77, want_mean=False)[1] == 0.0
    # clip: never above 1; clipped norm never above the limit
    for others in (0.0, 5 * ss, 1e6):
        for mx in (1.0, 1e-3, 1e3):
            c = orc.clip_coef(ss, others, mx)
            assert 0 < c <= 1.0
            assert c * math.sqrt(ss + others) <= mx * (1 + 1e-6)
            if math.sqrt(ss + others) + 1e-6 <= mx:
                assert c == 1.0
    assert orc.clip_coef(4.0, 12.0, 1.0) == pytest.approx(1.0 / (4.0 + 1e-6), rel=1e-15)


# --------------------------------------------------------------------------
# the Adam update
# --------------------------------------------------------------------------

def _state(n, seed, warm=False):
    th = gen.master(n, seed)
    m, v = gen.moments(n, seed, warm)
    return th, m, v, np.zeros(n, np.uint16)


def test_scalars():
    s = orc.derive_scalars(1e-4, 0.9, 0.999, 1e-8, 0.01, 1000, 8)
    assert s.gs == np.float32(0.125) and s.cc == 1.0
    assert s.b1 == np.float32(0.9) and s.omb1 == np.float32(1 - 0.9)
    assert s.b2 == np.float32(0.999) and s.omb2 == np.float32(1 - 0.999)
    assert s.step == np.float32(1e-4 / (1 - 0.9 ** 1000))
    assert s.isb2 == np.float32(1 / np.sqrt(1 - 0.999 ** 1000))
    assert abs(1 - 0.999 ** 1000 - 0.63230) < 1e-4           # beta2^1000 ~ 0.3677
    assert s.lw == np.float32(1e-4 * 0.01) and s.ep == np.float32(1e-8)
    s1 = orc.derive_scalars(1e-4, 0.9, 0.999, 1e-8, 0.01, 1, 6, clip_coef=0.25)
    assert s1.gs == np.float32(1 / 6) and s1.cc == 0.25
    assert s1.step == np.float32(1e-4 / (1 - 0.9)) and s1.isb2 == np.float32(1 / np.sqrt(1 - 0.999))


def test_zero_gradient_is_pure_decay():
    # g == 0, m = v = 0: theta_k = theta_0 (1 - lr wd)^k and the moments stay zero.
    n, k = 4096, 10
    th, m, v, p = _state(n, 1)
    th0 = th.astype(np.float64)
    z = [np.zeros(n, np.uint16)] * 4
    for t in range(1, k + 1):
        orc.step_f32(z, orc.derive_scalars(t=t, n_devices=4, **HP), th, m, v, p)
    assert not m.any() and not v.any()
    want = th0 * (1 - HP["lr"] * HP["weight_decay"]) ** k
    assert np.max(np.abs(th - want) / np.abs(want)) < k * 2.0 ** -23


def test_first_step_is_sign_descent():
    # t = 1, m = v = 0, wd = 0: bias correction gives m^ = g, v^ = g^2, so
    # theta' = theta - lr g / (|g| + eps).
    n = 4096
    th, m, v, p = _state(n, 2)
    th0 = th.astype(np.float64)
    g = gen.gradient(n, 2, 0, 0, "f32", std=1e-3)
    hp = dict(HP, weight_decay=0.0)
    orc.step_f32([g], orc.derive_scalars(t=1, n_devices=1, **hp), th, m, v, p)
    g64 = g.astype(np.float64)
    want = th0 - hp["lr"] * g64 / (np.abs(g64) + hp["eps"])
    assert np.max(np.abs(th - want)) < 1e-4 * 4e-6 + 2.0 ** -24 * np.max(np.abs(th0))
    assert np.allclose(m, 0.1 * g64, rtol=1e-6, atol=0)
    assert np.allclose(v, 0.001 * g64 * g64, rtol=1e-5, atol=0)


def test_constant_gradient_walks_linearly():
    # constant g, wd = 0: m^ = g and v^ = g^2 at every step, so
    # theta_k = theta_0 - k lr g / (|g| + eps).
    n, k = 2048, 25
    th, m, v, p = _state(n, 3)
    th0 = th.astype(np.float64)
    g = gen.gradient(n, 3, 0, 0, "f32", std=1e-3)
    g[np.abs(g) < 1e-6] = 1e-6
    hp = dict(HP, weight_decay=0.0)
    for t in range(1, k + 1):
        orc.step_f32([g], orc.derive_scalars(t=t, n_devices=1, **hp), th, m, v, p)
    g64 = g.astype(np.float64)
    want = th0 - k * hp["lr"] * g64 / (np.abs(g64) + hp["eps"])
    assert np.max(np.abs(th - want)) < 1e-5 * k * hp["lr"] + k * 2.0 ** -24 * np.max(np.abs(th0))


def test_invariants_sign_nonneg_permutation_split():
    n = 5000
    w = WORKLOADS["tiny"]
    grads = [gen.gradient(n, 4, 0, r, "bf16") for r in range(4)]
    th, m, v, p = _state(n, 4, warm=True)
    hp = dict(HP, weight_decay=0.0)
    s = orc.derive_scalars(t=7, n_devices=4, **hp)
    a = [x.copy() for x in (th, m, v, p)]
    orc.step_f32(grads, s, *a)
    assert (a[2] >= 0).all()
    moved = a[0] != th
    assert np.array_equal(np.sign(th - a[0])[moved], np.sign(a[1])[moved])
    # elementwise: permuting the inputs permutes the outputs
    perm = np.random.default_rng(0).permutation(n)
    b = [np.ascontiguousarray(x[perm]) for x in (th, m, v, p)]
    orc.step_f32([np.ascontiguousarray(g[perm]) for g in grads], s, *b)
    for x, y in zip(a, b):
        assert np.array_equal(x[perm].view(np.uint8), y.view(np.uint8))
    # any split of the index range gives the same bits
    c = [x.copy() for x in (th, m, v, p)]
    for lo, hi in ((0, 1), (1, 1234), (1234, 1234), (1234, n)):
        orc.step_f32(grads, s, *c, lo=lo, hi=hi)
    for x, y in zip(a, c):
        assert np.array_equal(x.view(np.uint8), y.view(np.uint8))
    # the bf16 image is the cast of the new master weight
    assert np.array_equal(a[3], orc.bf16_rne_bits(a[0].view(np.uint32)))
    assert w.n_devices == 4


@pytest.mark.parametrize("name,t", [("tiny", 1), ("tiny", 10), ("gpt2s", 1000), ("13b_clip", 1000)])
def test_binary32_order_is_within_rounding_of_binary64(name, t):
    """The binary32 op order against the all-binary64 pass.  Bounds follow the
    rounding steps: each fused multiply-add or product contributes half an ulp
    of its operands' size (m can cancel, so its bound is on the operands)."""
    w = WORKLOADS[name]
    n = 1 << 16
    u = 2.0 ** -24
    grads = [gen.gradient(n, w.seed, t, r, w.grad_dtype, w.grad_std, w.outlier_frac,
                          w.outlier_mult, w.student_t_dof) for r in range(w.n_devices)]
    th, m, v, p = _state(n, w.seed, w.warm_moments or t > 1)
    th0, m0 = th.astype(np.float64), m.astype(np.float64)
    hp = dict(lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, weight_decay=w.weight_decay)
    cc = 0.37 if w.max_grad_norm else 0.0
    t64, m64, v64 = orc.step_f64(grads, t=t, theta=th, m=m, v=v, clip_coef=cc, **hp)
    orc.step_f32(grads, orc.derive_scalars(t=t, n_devices=w.n_devices, clip_coef=cc, **hp),
                 th, m, v, p)
    widen = lambda g: (g.astype(np.uint32) << 16).view(np.float32) if g.dtype == np.uint16 else g
    scale = (1.0 / w.n_devices) * (cc if cc else 1.0)
    g64 = sum(widen(g).astype(np.float64) for g in grads) * scale
    gabs = sum(np.abs(widen(g).astype(np.float64)) for g in grads) * scale
    dg = (w.n_devices + 2) * u * gabs                 # N-1 adds and two scalings
    b1, b2 = w.beta1, w.beta2
    dm = 3 * u * (b1 * np.abs(m0) + (1 - b1) * gabs) + (1 - b1) * dg
    assert np.all(np.abs(m - m64) <= dm + 1e-45)
    dv = 4 * u * v64 + (1 - b2) * (2 * np.abs(g64) * dg + dg * dg)
    assert np.all(np.abs(v - v64) <= dv + 1e-45)
    bc1, bc2 = 1 - b1 ** t, 1 - b2 ** t
    root = np.sqrt(v64 / bc2)
    den = root + w.eps
    u64 = np.abs(m64 / bc1) / den
    dden = 3 * u * den + dv / (2 * np.sqrt(np.maximum(v64, 1e-300)) * np.sqrt(bc2))
    du = 3 * u * u64 + dm / bc1 / den + u64 * dden / den
    bound = 2 * u * (np.abs(th0) + np.abs(t64)) + w.lr / bc1 * (du + 3 * u * u64)
    assert np.all(np.abs(th - t64) <= bound)
    # and for the bulk of elements this is no more than one ulp of theta
    assert np.mean(ulp_diff(th, t64.astype(np.float32)) <= 1) > 0.97


@pytest.mark.parametrize("wd", [0.0, 0.01, 0.1])
def test_against_library_adamw(wd):
    """Ten steps of a library AdamW in binary64 on the CPU versus the binary64
    pass (tight) and the binary32 step (loose).  The oracle never calls the library."""
    n, N, k = 3000, 4, 10
    hp = dict(HP, weight_decay=wd, lr=3e-4)
    th0 = gen.master(n, 17)
    ref = torch.nn.Parameter(torch.from_numpy(th0.astype(np.float64)))
    opt = torch.optim.AdamW([ref], lr=hp["lr"], betas=(hp["beta1"], hp["beta2"]),
                            eps=hp["eps"], weight_decay=wd)
    th, m, v, p = th0.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32), np.zeros(n, np.uint16)
    th64, m64, v64 = th0.astype(np.float64), np.zeros(n), np.zeros(n)
    for t in range(1, k + 1):
        grads = [gen.gradient(n, 17, t, r, "bf16", std=1e-3) for r in range(N)]
        gmean = sum((g.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
                    for g in grads) / N
        ref.grad = torch.from_numpy(gmean.copy())
        opt.step()
        # binary64 pass chained through float32 storage would round each step, so
        # chain it in binary64 here: feed float32 views only for the gradients.
        s64 = orc.step_f64(grads, t=t, theta=th64.astype(np.float32), m=m64.astype(np.float32),
                           v=v64.astype(np.float32), **hp)
        orc.step_f32(grads, orc.derive_scalars(t=t, n_devices=N, **hp), th, m, v, p)
        if t == 1:
            assert np.allclose(s64[0], ref.detach().numpy(), rtol=0, atol=1e-12)
        th64, m64, v64 = s64
    lib = ref.detach().numpy()
    # the binary32 trajectory stays within rounding noise of the library's binary64 one
    assert np.max(np.abs(th - lib)) < 5e-8 * np.abs(lib).max() * k + 1e-9
    state = opt.state[ref]
    assert np.allclose(m, state["exp_avg"].numpy(), rtol=1e-5, atol=1e-6 * np.abs(m).max())
    assert np.allclose(v, state["exp_avg_sq"].numpy(), rtol=1e-5, atol=1e-6 * np.abs(v).max())
    moved = np.abs(th0.astype(np.float64) - lib)
    assert np.max(np.abs((th0 - th) - (th0.astype(np.float64) - lib)) / moved.max()) < 1e-3


def test_state_consistency_all_shards_equal_unsharded():
    """Tiny workload, 10 steps with fresh gradients: every device updates only its
    shard; concatenated they are bit-identical to the unsharded run (Theorem 4)."""
    w = WORKLOADS["tiny"]
    psi, N = w.psi, w.n_devices
    full = [gen.master(psi, w.seed), *gen.moments(psi, w.seed, False), np.zeros(psi, np.uint16)]
    shards = []
    for i in range(N):
        _, off, n, _ = pl.shard_geometry(psi, N, i)
        shards.append([np.ascontiguousarray(a[off:off + n]) for a in full])
    hp = dict(lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, weight_decay=w.weight_decay)
    for t in range(w.first_step, w.first_step + w.n_steps):
        grads = gen.workload_gradients(w, t)
        s = orc.derive_scalars(t=t, n_devices=N, **hp)
        orc.step_f32(grads, s, *full)
        for i in range(N):
            _, off, n, _ = pl.shard_geometry(psi, N, i)
            orc.step_f32([np.ascontiguousarray(g[off:off + n]) for g in grads], s, *shards[i])
    for k in range(4):
        cat = np.concatenate([sh[k] for sh in shards])
        assert np.array_equal(cat.view(np.uint8), full[k].view(np.uint8))
    assert np.abs(full[0] - gen.master(psi, w.seed)).max() > 1e-5   # it did move


# --------------------------------------------------------------------------
# verification protocol
# --------------------------------------------------------------------------

def test_checksum_against_published_vectors_and_brute_force(golden):
    M = (1 << 64) - 1
    outs = [int(golden["splitmix64_seed0_out%d" % k], 16) for k in (1, 2, 3)]
    # an all-zero buffer: word i contributes output i+1 of the generator seeded with 0
    assert orc.checksum(np.zeros(1, np.uint64)) == outs[0]
    assert orc.checksum(np.zeros(3, np.uint64)) == sum(outs) & M
    assert orc.checksum(np.zeros(1, np.uint64), first_index=2) == outs[2]

    def brute(words, first=0):
        c = 0
        for i, w in enumerate(words):
            z = (int(w) + (first + i + 1) * 0x9E3779B97F4A7C15) & M
            z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M
            z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M
            c = (c + (z ^ (z >> 31))) & M
        return c
    w = np.random.default_rng(3).integers(0, 2 ** 63, 257, dtype=np.uint64) * np.uint64(2) + np.uint64(1)
    assert orc.checksum(w) == brute(w)
    # pieces add up; position matters; one flipped bit shows
    assert (orc.checksum(w[:100]) + orc.checksum(w[100:], first_index=100)) & M == orc.checksum(w)
    sw = w.copy(); sw[[5, 9]] = sw[[9, 5]]
    assert orc.checksum(sw) != orc.checksum(w)
    fl = w.copy(); fl[77] ^= np.uint64(1 << 40)
    assert orc.checksum(fl) != orc.checksum(w)
    # any dtype by bytes
    f = gen.master(1024, 5)
    assert orc.checksum(f) == orc.checksum(f.view(np.uint64))
    with pytest.raises(ValueError):
        orc.checksum(np.zeros(3, np.uint16))


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_relative_difference_sums(dtype):
    import math
    n = 5003
    a = gen.gradient(n, 7, 0, 0, dtype, std=1e-2)
    b = gen.gradient(n, 7, 0, 1, dtype, std=1e-2)
    wid = lambda g: (g.astype(np.uint32) << 16).view(np.float32).astype(np.float64) if g.dtype == np.uint16 \
        else g.astype(np.float64)
    sd, sa = orc.diff_sumsq(a, b)
    assert sd == pytest.approx(math.fsum((wid(a) - wid(b)) ** 2), rel=1e-13)
    assert sa == pytest.approx(math.fsum(wid(a) ** 2), rel=1e-13)
    assert orc.diff_sumsq(a, a) == (0.0, sa)
    s1, s2 = orc.diff_sumsq(a, b, 0, 2000), orc.diff_sumsq(a, b, 2000, n)
    assert s1[0] + s2[0] == pytest.approx(sd, rel=1e-14) and s1[1] + s2[1] == pytest.approx(sa, rel=1e-14)
    # the paper's threshold: a reduction in another order stays far below 1e-5, a lost contribution does not
    g = [gen.gradient(n, 8, 0, r, "f32") for r in range(8)]
    fwd, rev, lost = orc.reduce_sum(g), orc.reduce_sum(g[::-1]), orc.reduce_sum(g[:-1])
    rel = lambda x, y: math.sqrt(orc.diff_sumsq(x, y)[0] / orc.diff_sumsq(x, y)[1])
    assert rel(fwd, rev) < float(load_tol()) and rel(fwd, lost) > float(load_tol())


def load_tol():
    from conftest import load_golden
    return load_golden()["grad_check_rel_tol"]


def _exhaustive_cast_check(oracle_cast, torch_dtype, quiet_nan, exp_mask):
    """All 2^32 binary32 patterns in chunks (four at a time; the C loop and the library
    conversion both release the interpreter lock): oracle cast == library conversion on
    every non-NaN input; NaNs compared as a class (canonical quiet NaN with the sign)."""
    from concurrent.futures import ThreadPoolExecutor
    chunk = 1 << 26

    def one(lo):
        u = np.arange(lo, lo + chunk, dtype=np.uint32)
        got = oracle_cast(u)
        lib = torch.from_numpy(u.view(np.float32)).to(torch_dtype).view(torch.int16).numpy().view(np.uint16)
        nan = (u & 0x7fffffff) > 0x7f800000
        assert np.array_equal(got[~nan], lib[~nan]), hex(lo)
        if nan.any():
            assert ((got[nan] & 0x7fff) == quiet_nan).all() and ((lib[nan] & exp_mask) == exp_mask).all()
            assert np.array_equal(got[nan] >> 15, (u[nan] >> 31).astype(np.uint16))
        return True

    torch.set_num_threads(2)
    with ThreadPoolExecutor(max_workers=4) as pool:
        assert all(pool.map(one, range(0, 1 << 32, chunk)))


def test_bf16_rne_exhaustive_against_library_conversion():
    """The oracle's bf16 cast against the library's float32 -> bfloat16 conversion (round
    to nearest even) on all 2^32 binary32 patterns."""
    _exhaustive_cast_check(orc.bf16_rne_bits, torch.bfloat16, 0x7fc0, 0x7f80)


def test_f16_rne_exhaustive_against_library_conversion():
    """The oracle's binary16 cast against the library's float32 -> float16 conversion on
    all 2^32 binary32 patterns."""
    _exhaustive_cast_check(orc.f16_rne_bits, torch.float16, 0x7e00, 0x7c00)


def test_step_with_binary16_gradients_and_parameters():
    """The FP16 flavour of the step (Table 1: FP16 parameters and gradients, with a loss
    scale riding on grad_scale): same arithmetic as with bf16 once the contributions are
    widened, and the 16-bit image is the binary16 cast of the new master weight."""
    n, N, scale = 3001, 4, 1024.0
    g16 = [gen.gradient(n, 23, 0, r, "f16", std=1e-3 * scale, outlier_frac=0.01, outlier_mult=100.0)
           for r in range(N)]
    assert all(np.isinf(g).sum() == 0 for g in g16) and any((np.abs(g) < 6e-5).any() for g in g16)
    g32 = [g.astype(np.float32) for g in g16]                 # exact widening by the library
    s = orc.derive_scalars(t=3, n_devices=N, grad_scale=1.0 / (N * scale), **HP)
    a = [gen.master(n, 23), *gen.moments(n, 23, True), np.zeros(n, np.float16)]
    b = [x.copy() for x in a[:3]] + [np.zeros(n, np.uint16)]
    orc.step_f32(g16, s, *a)
    orc.step_f32(g32, s, *b)
    for x, y in zip(a[:3], b[:3]):
        assert np.array_equal(x.view(np.uint32), y.view(np.uint32))
    with np.errstate(over="ignore"):
        assert np.array_equal(a[3].view(np.uint16), a[0].astype(np.float16).view(np.uint16))
    assert np.array_equal(b[3], orc.bf16_rne_bits(b[0].view(np.uint32)))

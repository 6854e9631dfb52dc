"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by
element, on the same seeded inputs.  Bar: shard indexing, the fixed-order
reduction and the bf16 cast bit-exact; master/m/v within 2 binary32 ulp."""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_2601_02311_amd as ps
from oracle import placement as pl
from oracle import step as orc
from synth import WORKLOADS
from synth import host as gen

from gpu_util import (assert_state_parity, dev, grads_of, host, hp_of, shard_of,
                      stream_handle, ulp_diff)

pytestmark = pytest.mark.gpu

TILE = 2048  # eight of the update kernel's 256-element tiles (one wave x 4 elements per lane)


def _say(msg):
    print("[case] " + msg, flush=True)


def _run_gpu(spec, hp, state, grads_np, dtype, n, valid=None, offset=0, count=None, out_len=None):
    """Upload, run one ps_step_update on [offset, offset+count), download."""
    th, m, v, p = [dev(a) for a in state]
    gd = [dev(g) for g in grads_np]
    shard = shard_of(th, m, v, p, n, valid)
    count = n - offset if count is None else count
    ps.ps_step_update(spec, hp, shard, grads_of(gd, dtype, offset), offset, count, stream_handle())
    torch.cuda.synchronize()
    return [host(t) for t in (th, m, v, p)]


def test_tiny_ten_steps_all_shards_equal_unsharded():
    w = WORKLOADS["tiny"]
    _say("tiny: psi=%d N=%d, 10 steps, all shards vs unsharded oracle" % (w.psi, w.n_devices))
    psi, N = w.psi, w.n_devices
    full = [gen.master(psi, w.seed), *gen.moments(psi, w.seed, False), np.zeros(psi, np.uint16)]
    shards = []
    for i in range(N):
        spec = ps.ps_spec_preset(w.strategy, N, i, psi)
        c = ps.ps_cost_eval(spec)
        assert (c.shard_offset, c.shard_len) == pl.shard_geometry(psi, N, i)[1:3]
        sl = slice(c.shard_offset, c.shard_offset + c.shard_len)
        t = [dev(np.ascontiguousarray(a[sl])) for a in full]
        shards.append((spec, c, sl, t))
    for t_step in range(w.first_step, w.first_step + w.n_steps):
        grads = gen.workload_gradients(w, t_step)
        hpd, hp = hp_of(w, t_step)
        orc.step_f32(grads, orc.derive_scalars(t=t_step, n_devices=N, **hpd), *full)
        for spec, c, sl, t in shards:
            gd = [dev(np.ascontiguousarray(g[sl])) for g in grads]
            ps.ps_step_update(spec, hp, shard_of(*t, c.shard_len), grads_of(gd, "bf16"), 0,
                              c.shard_len, stream_handle())
            torch.cuda.synchronize()
    mismatched = 0
    for spec, c, sl, t in shards:
        got = [host(x) for x in t]
        mismatched += assert_state_parity(got, [a[sl] for a in full], "shard %d" % spec.shard_index)
    _say("tiny: elements whose theta differs in the last bits after 10 steps: %d" % mismatched)
    assert mismatched == 0      # same op order on both sides: expect identical bits


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("N", [1, 2, 3, 4, 5, 6, 8, 16])
def test_ragged_sizes_every_contribution_count(dtype, N):
    if N == 1 and dtype == "bf16":
        pytest.skip("a single contribution is the pre-reduced fp32 gradient")
    n = 3 * TILE + 1234 + 3           # several tiles and a ragged tail
    valid = n - 5                      # last five elements are padding
    _say("ragged n=%d valid=%d N=%d %s" % (n, valid, N, dtype))
    psi = n * max(N, 1)
    spec = ps.ps_spec_preset("zero3", max(N, 1), 0, psi)
    if N == 1:
        spec = ps.ps_spec_preset("zero3", 4, 0, n * 4)
    grads = [gen.gradient(n, 77, 3, r, dtype, std=1e-3, outlier_frac=0.01, outlier_mult=100.0)
             for r in range(N)]
    th = gen.master(n, 77)
    m, v = gen.moments(n, 77, True)
    canary = np.uint16(0xBEEF)
    state = [th, m, v, np.full(n, canary, np.uint16)]
    hpd, hp = hp_of(None, 1000, grad_scale=(1.0 if N == 1 else 0.0))
    want = [a.copy() for a in state]
    s = orc.derive_scalars(t=1000, n_devices=spec.n_devices, grad_scale=(1.0 if N == 1 else 0.0), **hpd)
    orc.step_f32(grads, s, *want, lo=0, hi=valid)
    got = _run_gpu(spec, hp, state, grads, dtype, n, valid)
    assert assert_state_parity(got, want, "ragged") == 0
    for g, a in zip(got, state):       # pads untouched, byte for byte
        assert np.array_equal(g[valid:].view(np.uint8), a[valid:].view(np.uint8))
    assert (got[3][valid:] == canary).all()


def test_bucket_range_inside_a_shard():
    """Only [offset, offset+count) is touched; gradient pointers are bucket-based."""
    n, N = 5 * TILE + 40, 4
    off, cnt = 2 * TILE + 8, 2 * TILE + 17
    _say("sub-range [%d,+%d) of n=%d" % (off, cnt, n))
    spec = ps.ps_spec_preset("zero3", N, 2, n * N)
    grads = [gen.gradient(n, 5, 0, r, "bf16") for r in range(N)]
    state = [gen.master(n, 5), *gen.moments(n, 5, True), np.full(n, 0x1234, np.uint16)]
    hpd, hp = hp_of(None, 17)
    want = [a.copy() for a in state]
    orc.step_f32(grads, orc.derive_scalars(t=17, n_devices=N, **hpd), *want, lo=off, hi=off + cnt)
    got = _run_gpu(spec, hp, state, grads, "bf16", n, None, off, cnt)
    for g, w_ in zip(got, want):
        assert np.array_equal(g.view(np.uint8), w_.view(np.uint8))


def test_zero2_writes_its_slice_of_the_replicated_parameters():
    n, N, i = TILE + 24, 4, 2
    _say("zero2 output slice, n=%d shard %d" % (n, i))
    spec = ps.ps_spec_preset("zero2", N, i, n * N)
    c = ps.ps_cost_eval(spec)
    grads = [gen.gradient(n, 8, 0, r, "bf16") for r in range(N)]
    state = [gen.master(n, 8), *gen.moments(n, 8, False), np.zeros(n, np.uint16)]
    hpd, hp = hp_of(None, 1)
    want = [a.copy() for a in state]
    orc.step_f32(grads, orc.derive_scalars(t=1, n_devices=N, **hpd), *want)
    th, m, v = [dev(a) for a in state[:3]]
    full_p = dev(np.full(n * N, 0xCAFE, np.uint16))
    gd = [dev(g) for g in grads]
    ps.ps_step_update(spec, hp, shard_of(th, m, v, full_p, n), grads_of(gd, "bf16"), 0, n,
                      stream_handle())
    torch.cuda.synchronize()
    p = host(full_p)
    assert np.array_equal(p[c.shard_offset:c.shard_offset + n], want[3])
    assert (p[:c.shard_offset] == 0xCAFE).all() and (p[c.shard_offset + n:] == 0xCAFE).all()
    assert np.array_equal(host(th).view(np.uint32), want[0].view(np.uint32))


def test_gpt2s_shard_full_size():
    w = WORKLOADS["gpt2s"]
    n, N, t = w.shard_len, w.n_devices, w.first_step
    _say("gpt2s: n=%d N=%d t=%d (not a multiple of the tile)" % (n, N, t))
    assert n % TILE != 0
    grads = [gen.gradient(n, w.seed, t, r, "bf16", w.grad_std) for r in range(N)]
    state = [gen.master(n, w.seed), *gen.moments(n, w.seed, True), np.zeros(n, np.uint16)]
    hpd, hp = hp_of(w, t)
    want = [a.copy() for a in state]
    orc.step_f32(grads, orc.derive_scalars(t=t, n_devices=N, **hpd), *want)
    spec = ps.ps_spec_preset(w.strategy, N, w.shard_index, w.psi)
    got = _run_gpu(spec, hp, state, grads, "bf16", n)
    assert assert_state_parity(got, want, "gpt2s") == 0
    assert np.array_equal(got[3], want[3])


def test_special_values_propagate():
    """Inf/NaN/huge/subnormal/zero gradients and states: no special casing, same as the oracle."""
    n, N = TILE + 64, 2
    _say("special values n=%d" % n)
    spec = ps.ps_spec_preset("zero3", N, 0, n * N)
    g0 = gen.gradient(n, 3, 0, 0, "f32")
    g1 = gen.gradient(n, 3, 0, 1, "f32")
    g0[:8] = [np.inf, -np.inf, np.nan, 3e38, 1e-45, 0.0, -0.0, 1e-30]
    g1[:8] = [1.0, 1.0, 1.0, 3e38, 1e-45, 0.0, -0.0, -1e-30]
    g0[8:16] = [np.inf] * 8
    g1[8:16] = [-np.inf] * 8                      # inf - inf
    th = gen.master(n, 3)
    m, v = gen.moments(n, 3, True)
    th[16:24] = [0.0, -0.0, 1e-42, 3.3e38, -3.3e38, np.inf, 1.0, 1.0]
    v[22] = 0.0; m[22] = 0.0; g0[22] = 0.0; g1[22] = 0.0       # 0/eps
    v[23] = 1e-45                                               # subnormal second moment
    state = [th, m, v, np.zeros(n, np.uint16)]
    hpd, hp = hp_of(None, 2)
    want = [a.copy() for a in state]
    orc.step_f32([g0, g1], orc.derive_scalars(t=2, n_devices=N, **hpd), *want)
    got = _run_gpu(spec, hp, state, [g0, g1], "f32", n)
    assert_state_parity(got, want, "specials")
    nan = np.isnan(want[0])
    assert nan[:3].all() and nan[8:16].all()
    assert ((got[3][nan] & 0x7fff) == 0x7fc0).all()             # canonical quiet NaN
    assert np.array_equal(got[3][~nan], want[3][~nan])


def test_cast_exhaustive_over_all_binary32_patterns():
    """Every binary32 pattern goes through the kernel as a master value.  With lr = 0, zero
    moments and a zero gradient the update leaves every finite value as it is (only -0
    becomes +0, and an infinity turns into NaN by 0 x inf), so the bf16 image the kernel
    writes is the cast of all 2^32 patterns: compared bit for bit with the library's
    round-to-nearest-even conversion of the master the kernel left behind."""
    chunk = 1 << 28
    _say("exhaustive cast: 2^32 master patterns in %d launches" % ((1 << 32) // chunk))
    spec = ps.ps_spec_preset("zero3", 4, 0, chunk * 4)
    _, hp = hp_of(None, 1, lr=0.0, weight_decay=0.0, grad_scale=1.0)
    bits = torch.empty(chunk, dtype=torch.int32, device="cuda")
    th = bits.view(torch.float32)
    m = torch.zeros(chunk, dtype=torch.float32, device="cuda")
    v = torch.zeros_like(m)
    g = torch.zeros_like(m)
    out = torch.empty(chunk, dtype=torch.int16, device="cuda")
    ramp = torch.arange(chunk, dtype=torch.int64, device="cuda")
    for lo in range(0, 1 << 32, chunk):
        before = ((ramp + lo) & 0xffffffff)
        bits.copy_(torch.where(before >= (1 << 31), before - (1 << 32), before).to(torch.int32))
        before = bits.clone()
        out.fill_(0x1111)
        ps.ps_step_update(spec, hp, shard_of(th, m, v, out, chunk), grads_of([g], "f32"), 0, chunk,
                          stream_handle())
        torch.cuda.synchronize()
        mag = before & 0x7fffffff
        finite = mag < 0x7f800000
        keep = finite & (before != -(1 << 31))                   # all finite values but -0
        assert torch.equal(bits[keep], before[keep]), hex(lo)    # identity: the cast sees them all
        nan = torch.isnan(th)
        lib = th.to(torch.bfloat16).view(torch.int16)
        assert torch.equal(out[~nan], lib[~nan]), hex(lo)
        assert bool(((out[nan] & 0x7fff) == 0x7fc0).all()), hex(lo)
        assert bool(nan[~finite].all()) and not bool(nan[finite].any())
    assert not bool(m.view(torch.int32).any()) and not bool(v.view(torch.int32).any())


@pytest.mark.parametrize("hpkw", [dict(beta1=0.0, beta2=0.0, eps=0.0),          # sign descent; 0/0 where g == 0
                                  dict(lr=0.0, weight_decay=0.0),               # nothing moves but m and v
                                  dict(weight_decay=0.0, eps=1.0),
                                  dict(lr=10.0, weight_decay=0.5, eps=1e-30),   # wild step, 1 - lr*wd < 0
                                  dict(beta1=0.999999, beta2=0.9999999)])       # bias corrections far from 1
@pytest.mark.parametrize("t", [1, 7, 10 ** 6, 2 ** 40])
def test_degenerate_hyperparameters_and_step_counts(hpkw, t):
    """Corners of the hyper-parameter space: the scalars both sides derive in binary64 and
    the special values they lead to (0/0, overflow, sign flips) must coincide."""
    n, N = TILE + 300, 4
    _say("hyper-parameter corner %s t=%d" % (hpkw, t))
    spec = ps.ps_spec_preset("zero3", N, 1, n * N)
    grads = [gen.gradient(n, 61, 0, r, "bf16") for r in range(N)]
    for g in grads:
        g[:32] = 0                                             # exact zero gradient in the first elements
    state = [gen.master(n, 61), *gen.moments(n, 61, True), np.zeros(n, np.uint16)]
    state[1][:16] = 0.0
    state[2][:16] = 0.0                                        # ... and zero moments under half of them
    base = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)
    base.update(hpkw)
    hp = ps.ps_adamw_t(base["lr"], base["beta1"], base["beta2"], base["eps"], base["weight_decay"], t, 0.0, 0.0)
    want = [a.copy() for a in state]
    orc.step_f32(grads, orc.derive_scalars(t=t, n_devices=N, **base), *want)
    got = _run_gpu(spec, hp, state, grads, "bf16", n)
    assert assert_state_parity(got, want, "corner") == 0
    nan = np.isnan(want[0])
    assert np.array_equal(got[3][~nan], want[3][~nan])
    assert ((got[3][nan] & 0x7fff) == 0x7fc0).all()


def test_run_twice_is_bitwise_identical():
    n, N = 7 * TILE + 99, 8
    _say("determinism n=%d" % n)
    spec = ps.ps_spec_preset("zero3", N, 1, n * N)
    grads = [gen.gradient(n, 13, 0, r, "bf16") for r in range(N)]
    state = [gen.master(n, 13), *gen.moments(n, 13, True), np.zeros(n, np.uint16)]
    _, hp = hp_of(None, 5)
    a = _run_gpu(spec, hp, state, grads, "bf16", n)
    b = _run_gpu(spec, hp, state, grads, "bf16", n)
    for x, y in zip(a, b):
        assert np.array_equal(x.view(np.uint8), y.view(np.uint8))


# ---- sum of squares and the clipped two-phase step ----

def _reduce_gpu(spec, grads_np, dtype, n, valid, gs=0.0, want_reduced=True, buckets=None):
    gd = [dev(g) for g in grads_np]
    red = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
    ss = torch.zeros(1, dtype=torch.float64, device="cuda")
    ws = torch.empty(ps.ps_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    ranges = buckets or [(0, n)]
    for k, (lo, cnt) in enumerate(ranges):
        ps.ps_step_reduce_sumsq(spec, grads_of(gd, dtype, lo), gs,
                                red.data_ptr() if want_reduced else 0, ss.data_ptr(), int(k > 0),
                                ws.data_ptr(), ws.numel(), lo, cnt, valid, stream_handle())
    torch.cuda.synchronize()
    return host(red), float(ss.item())


@pytest.mark.parametrize("dtype,N,n", [("f32", 6, 9 * TILE + 777), ("bf16", 8, 9 * TILE + 777),
                                       ("f32", 3, 9 * TILE + 777), ("bf16", 4, 9 * TILE + 777),
                                       ("f32", 16, 9 * TILE + 777),
                                       ("f32", 6, 1500 * TILE + 1255)])   # two-level final sum
def test_reduce_sumsq_matches_oracle(dtype, N, n):
    valid = n - 1001
    _say("reduce+sumsq n=%d valid=%d N=%d %s" % (n, valid, N, dtype))
    spec = ps.ps_spec_preset("zero3", N, N - 1, n * N)
    grads = [gen.gradient(n, 31, 0, r, dtype, std=1e-4, student_t_dof=3) for r in range(N)]
    gm, ss = orc.mean_sumsq(grads, 1.0 / N, 0, valid)
    red, ss_gpu = _reduce_gpu(spec, grads, dtype, n, valid)
    assert np.array_equal(red[:valid].view(np.uint32), gm[:valid].view(np.uint32))   # bit-exact mean
    assert np.isnan(red[valid:]).all()                                              # pad untouched
    assert abs(ss_gpu - ss) <= 1e-12 * ss            # binary64 tree vs sequential binary64 sum
    # reproducible bit for bit, with or without storing the mean
    _, again = _reduce_gpu(spec, grads, dtype, n, valid, want_reduced=False)
    assert again == ss_gpu
    # the same total when the range arrives as buckets in order (accumulate flag)
    b = (n // 5) // 8 * 8 + 8
    buckets = [(lo, min(b, n - lo)) for lo in range(0, n, b)]
    red2, ss_b = _reduce_gpu(spec, grads, dtype, n, valid, buckets=buckets)
    assert np.array_equal(red2[:valid].view(np.uint32), gm[:valid].view(np.uint32))
    assert abs(ss_b - ss) <= 1e-12 * ss
    assert _reduce_gpu(spec, grads, dtype, n, valid, buckets=buckets)[1] == ss_b


def test_reduce_sumsq_degenerate_ranges():
    n, N = 64, 4
    _say("reduce+sumsq degenerate: tiny n, empty valid range, inf")
    spec = ps.ps_spec_preset("zero3", N, 0, n * N)
    grads = [gen.gradient(n, 1, 0, r, "f32") for r in range(N)]
    _, ss = orc.mean_sumsq(grads, 1.0 / N)
    assert abs(_reduce_gpu(spec, grads, "f32", n, n)[1] - ss) <= 1e-12 * ss
    assert _reduce_gpu(spec, grads, "f32", n, 0)[1] == 0.0           # all padding
    grads[1][5] = np.inf
    red, ss_inf = _reduce_gpu(spec, grads, "f32", n, n)
    assert np.isinf(ss_inf)                                           # caller sees it and may skip
    # ... and a caller who does not look cannot damage the state: the library reports the
    # coefficient of a non-finite sum as NaN, and the update refuses a NaN before any launch
    assert np.isnan(ps.ps_clip_coef(ss_inf, 0.0, 1.0))
    state = [gen.master(n, 1), *gen.moments(n, 1, True), np.full(n, 0x4242, np.uint16)]
    th, m, v, p = [dev(a) for a in state]
    _, hp = hp_of(None, 3, grad_scale=1.0, clip_coef=ps.ps_clip_coef(ss_inf, 0.0, 1.0))
    with pytest.raises(ps.PsError) as e:
        ps.ps_step_update(spec, hp, shard_of(th, m, v, p, n), grads_of([dev(red)], "f32"), 0, n,
                          stream_handle())
    assert e.value.status == ps.PS_ERANGE
    torch.cuda.synchronize()
    for t_, a in zip((th, m, v, p), state):
        assert np.array_equal(host(t_).view(np.uint8), a.view(np.uint8))


def test_clipped_two_phase_step_matches_oracle():
    """Ragged fp32 shard with global-norm clipping: phase 1 reduces and sums squares,
    the host forms the coefficient, phase 2 updates from the reduced gradient."""
    w = WORKLOADS["13b_clip"]
    N = w.n_devices
    n = 11 * TILE + 1536            # a multiple of 256, not of the tile
    valid = n - 1001
    _say("clip two-phase n=%d valid=%d N=%d" % (n, valid, N))
    spec = ps.ps_spec_preset(w.strategy, N, N - 1, n * N - 1001, align_elems=w.align_elems)
    c = ps.ps_cost_eval(spec)
    assert (c.shard_len, c.valid_len) == (n, valid)
    grads = [gen.gradient(n, w.seed, 1, r, "f32", 1e-2, student_t_dof=3) for r in range(N)]
    state = [gen.master(n, w.seed), *gen.moments(n, w.seed, True), np.full(n, 0xD00D, np.uint16)]
    t = w.first_step
    # oracle: unclipped norm -> coefficient -> step (clip applied after the mean)
    _, ss = orc.mean_sumsq(grads, 1.0 / N, 0, valid)
    coef = orc.clip_coef(ss, 5 * ss, w.max_grad_norm)
    assert coef < 1.0
    hpd, _ = hp_of(w, t)
    want = [a.copy() for a in state]
    orc.step_f32(grads, orc.derive_scalars(t=t, n_devices=N, clip_coef=coef, **hpd), *want, lo=0, hi=valid)
    # GPU: phase 1
    gd = [dev(g) for g in grads]
    red = torch.zeros(n, dtype=torch.float32, device="cuda")
    ssd = torch.zeros(1, dtype=torch.float64, device="cuda")
    ws = torch.empty(ps.ps_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    ps.ps_step_reduce_sumsq(spec, grads_of(gd, "f32"), 0.0, red.data_ptr(), ssd.data_ptr(), 0,
                            ws.data_ptr(), ws.numel(), 0, n, valid, stream_handle())
    ss_gpu = float(ssd.item())
    assert abs(ss_gpu - ss) <= 1e-12 * ss
    # phase 2 with the SAME coefficient as the oracle, so a last-bit difference in the
    # sum cannot leak into the state comparison
    _, hp = hp_of(w, t, grad_scale=1.0, clip_coef=coef)
    th, m, v, p = [dev(a) for a in state]
    ps.ps_step_update(spec, hp, shard_of(th, m, v, p, n, valid), grads_of([red], "f32"), 0, n,
                      stream_handle())
    torch.cuda.synchronize()
    got = [host(x) for x in (th, m, v, p)]
    assert assert_state_parity(got, want, "clip") == 0
    for g, a in zip(got, state):
        assert np.array_equal(g[valid:].view(np.uint8), a[valid:].view(np.uint8))
    # the coefficient formed from the GPU's own sum is the same binary32 scalar here
    assert np.float32(ps.ps_clip_coef(ss_gpu, 5 * ss_gpu, w.max_grad_norm)) == np.float32(coef)


def test_clip_coefficient_formed_on_the_device():
    """ps_step_clip_coef against the oracle's binary64 formula on the same sums: the
    binary32 coefficient must be the same bit pattern (sqrt and division in binary64 are
    correctly rounded on both sides), NaN exactly where the host function reports NaN."""
    rng = np.random.default_rng(7)
    a = np.concatenate([10.0 ** rng.uniform(-30, 30, 40), [0.0, 1e-300, 4.0, np.inf, np.nan, -1.0, 1.0]])
    b = np.concatenate([10.0 ** rng.uniform(-30, 30, 40), [0.0, 0.0, 12.0, 1.0, 1.0, 1.0, np.inf]])
    mx = np.concatenate([10.0 ** rng.uniform(-3, 3, 40), [1.0, 1.0, 1.0, 1.0, 1.0, 1.0, 1.0]])
    _say("device clip coefficient on %d (local, others, max_norm) triples" % a.size)
    da, db = dev(a), dev(b)
    out = torch.full((a.size,), -7.0, dtype=torch.float32, device="cuda")
    for k in range(a.size):
        ps.ps_step_clip_coef(da.data_ptr() + 8 * k, db.data_ptr() + 8 * k, float(mx[k]),
                             out.data_ptr() + 4 * k, stream_handle())
    lone = torch.full((1,), -7.0, dtype=torch.float32, device="cuda")
    ps.ps_step_clip_coef(da.data_ptr() + 8 * 42, 0, 1.0, lone.data_ptr(), stream_handle())   # no others: 4.0 alone
    torch.cuda.synchronize()
    got = host(out)
    for k in range(a.size):
        lib = ps.ps_clip_coef(float(a[k]), float(b[k]), float(mx[k]))
        if np.isnan(lib):
            assert np.isnan(got[k]), k
        else:
            want = np.float32(orc.clip_coef(float(a[k]), float(b[k]), float(mx[k])))
            assert got[k].view(np.uint32) == want.view(np.uint32), (k, a[k], b[k], mx[k])
            assert np.float32(lib).view(np.uint32) == want.view(np.uint32)
    assert np.isnan(got[-4:]).all() and not np.isnan(got[:43]).any()
    assert host(lone)[0] == np.float32(orc.clip_coef(4.0, 0.0, 1.0))


def test_clipped_step_without_a_host_round_trip():
    """Phase 1, the coefficient and phase 2 all enqueued on one stream; the update reads
    the coefficient the device wrote.  Compared with the oracle given the same sums; a
    second run with an infinite gradient must leave every buffer as it was."""
    w = WORKLOADS["13b_clip"]
    N = w.n_devices
    n = 7 * TILE + 1536 + 40
    valid = n - 9
    _say("clip on the stream n=%d valid=%d N=%d" % (n, valid, N))
    spec = ps.ps_spec_preset(w.strategy, N, 0, n * N)
    grads = [gen.gradient(n, w.seed, 2, r, "f32", 1e-2, student_t_dof=3) for r in range(N)]
    state = [gen.master(n, w.seed), *gen.moments(n, w.seed, True), np.full(n, 0xABCD, np.uint16)]
    hpd, _ = hp_of(w, 11)
    gd = [dev(g) for g in grads]
    th, m, v, p = [dev(a) for a in state]
    red = torch.zeros(n, dtype=torch.float32, device="cuda")
    ssd = torch.zeros(1, dtype=torch.float64, device="cuda")
    others = torch.zeros(1, dtype=torch.float64, device="cuda")
    coef = torch.zeros(1, dtype=torch.float32, device="cuda")
    ws = torch.empty(ps.ps_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    hp = ps.ps_adamw_t(hpd["lr"], hpd["beta1"], hpd["beta2"], hpd["eps"], hpd["weight_decay"], 11,
                       1.0, 0.0, coef.data_ptr())

    def enqueue():
        ps.ps_step_reduce_sumsq(spec, grads_of(gd, "f32"), 0.0, red.data_ptr(), ssd.data_ptr(), 0,
                                ws.data_ptr(), ws.numel(), 0, n, valid, stream_handle())
        torch.mul(ssd, 5.0, out=others)                  # stands for the all-reduce of the peers' sums
        ps.ps_step_clip_coef(ssd.data_ptr(), others.data_ptr(), w.max_grad_norm, coef.data_ptr(),
                             stream_handle())
        ps.ps_step_update(spec, hp, shard_of(th, m, v, p, n, valid), grads_of([red], "f32"), 0, n,
                          stream_handle())
    enqueue()
    torch.cuda.synchronize()
    ss = float(ssd.item())
    c = orc.clip_coef(ss, 5.0 * ss, w.max_grad_norm)
    assert c < 1.0 and host(coef)[0] == np.float32(c)
    want = [a.copy() for a in state]
    orc.step_f32(grads, orc.derive_scalars(t=11, n_devices=N, clip_coef=c, **hpd), *want, lo=0, hi=valid)
    got = [host(x) for x in (th, m, v, p)]
    assert assert_state_parity(got, want, "clip on the stream") == 0
    # a non-finite gradient: NaN coefficient, the update launches turn into no-ops
    bad = grads[2].copy()
    bad[n // 2] = np.inf
    gd[2].copy_(dev(bad))
    enqueue()
    torch.cuda.synchronize()
    assert np.isinf(float(ssd.item())) and np.isnan(host(coef)[0])
    for x, a in zip((th, m, v, p), got):
        assert np.array_equal(host(x).view(np.uint8), a.view(np.uint8))
    # the host coefficient and the device coefficient exclude each other
    both = ps.ps_adamw_t(hpd["lr"], hpd["beta1"], hpd["beta2"], hpd["eps"], hpd["weight_decay"], 11,
                         1.0, 0.5, coef.data_ptr())
    with pytest.raises(ps.PsError) as e:
        ps.ps_step_update(spec, both, shard_of(th, m, v, p, n, valid), grads_of([red], "f32"), 0, n,
                          stream_handle())
    assert e.value.status == ps.PS_EINVAL


def test_both_phases_captured_in_a_hip_graph_and_replayed():
    """The launch-only entry points allocate nothing and synchronise nothing, so a caller
    may capture them.  One graph holds a whole clipped step: phase 1 (reduce + sum of
    squares), the coefficient formed on the device, phase 2 (update from the reduced
    gradient).  It is replayed three times with eager work and synchronisation between
    the replays, and every replay is compared with the oracle advanced by one more step."""
    N, n = 6, 5 * TILE + 777
    valid = n - 3
    _say("graph capture: phases 1+2, n=%d N=%d, 3 replays" % (n, N))
    spec = ps.ps_spec_preset("zero3", N, 0, n * N)
    grads = [gen.gradient(n, 41, 0, r, "f32", 1e-2) for r in range(N)]
    state = [gen.master(n, 41), *gen.moments(n, 41, True), np.full(n, 0x7777, np.uint16)]
    t, max_norm = 9, 0.05
    hpd, _ = hp_of(None, t)
    _, ss = orc.mean_sumsq(grads, 1.0 / N, 0, valid)
    want = [a.copy() for a in state]
    cdev = torch.zeros(1, dtype=torch.float32, device="cuda")
    hp = ps.ps_adamw_t(hpd["lr"], hpd["beta1"], hpd["beta2"], hpd["eps"], hpd["weight_decay"], t,
                       1.0, 0.0, cdev.data_ptr())
    gd = [dev(g) for g in grads]
    th, m, v, p = [dev(a) for a in state]
    red = torch.zeros(n, dtype=torch.float32, device="cuda")
    ssd = torch.zeros(1, dtype=torch.float64, device="cuda")
    ws = torch.empty(ps.ps_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    shard, gl, gr = shard_of(th, m, v, p, n, valid), grads_of(gd, "f32"), grads_of([red], "f32")
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ps.ps_step_reduce_sumsq(spec, gl, 0.0, red.data_ptr(), ssd.data_ptr(), 0, ws.data_ptr(),
                                ws.numel(), 0, n, valid, stream_handle())
        ps.ps_step_clip_coef(ssd.data_ptr(), 0, max_norm, cdev.data_ptr(), stream_handle())
        ps.ps_step_update(spec, hp, shard, gr, 0, n, stream_handle())
    torch.cuda.synchronize()
    assert np.array_equal(host(th).view(np.uint32), state[0].view(np.uint32))   # capture ran nothing
    # the oracle's coefficient from the device's own sum (the two sums agree to 1e-12, the
    # coefficient must not depend on which one is rounded)
    ps.ps_step_reduce_sumsq(spec, gl, 0.0, 0, ssd.data_ptr(), 0, ws.data_ptr(), ws.numel(), 0, n, valid,
                            stream_handle())
    coef = orc.clip_coef(float(ssd.item()), 0.0, max_norm)
    assert coef < 1.0
    s = orc.derive_scalars(t=t, n_devices=N, clip_coef=coef, **hpd)
    for k in range(3):
        red.fill_(float("nan")); ssd.fill_(-1.0); cdev.fill_(float("nan"))   # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        orc.step_f32(grads, s, *want, lo=0, hi=valid)
        got = [host(x) for x in (th, m, v, p)]
        assert assert_state_parity(got, want, "replay %d" % k) == 0
        assert abs(float(ssd.item()) - ss) <= 1e-12 * ss and host(cdev)[0] == np.float32(coef)
        for g_, a in zip(got, state):
            assert np.array_equal(g_[valid:].view(np.uint8), a[valid:].view(np.uint8))


def test_allocation_free_step_captured_in_a_hip_graph():
    """What a caller under stream capture can use: the reduce phase with the library's own
    partial-sum array (no workspace to allocate), the coefficient on the device, and the
    bucket loop reading the reduced gradient in place.  One warm-up call outside the capture
    (the first call per device looks the array up), then three replays against the oracle."""
    N, n, bucket = 4, 9 * TILE + 120, 2 * TILE
    _say("graph capture: static reduce + in-place bucket loop, n=%d N=%d" % (n, N))
    spec = ps.ps_spec_preset("zero3", N, 1, n * N)
    grads = [gen.gradient(n, 43, 0, r, "bf16", 1e-2) for r in range(N)]
    state = [gen.master(n, 43), *gen.moments(n, 43, True), np.zeros(n, np.uint16)]
    t, max_norm = 5, 0.05
    hpd, _ = hp_of(None, t)
    want = [a.copy() for a in state]
    cdev = torch.zeros(1, dtype=torch.float32, device="cuda")
    hp = ps.ps_adamw_t(hpd["lr"], hpd["beta1"], hpd["beta2"], hpd["eps"], hpd["weight_decay"], t,
                       1.0, 0.0, cdev.data_ptr())
    gd = [dev(g) for g in grads]
    th, m, v, p = [dev(a) for a in state]
    red = torch.zeros(-(-n // 512) * 512, dtype=torch.float32, device="cuda")
    ssd = torch.zeros(1, dtype=torch.float64, device="cuda")
    gl = grads_of(gd, "bf16")
    plan = ps.ps_bucket_plan_t()
    arr = (C.c_void_p * 1)(red.data_ptr())
    plan.source = C.cast(arr, C.POINTER(C.c_void_p))
    plan.n_contrib, plan.dtype, plan.bucket_elems, plan.source_elems = 1, ps.PS_F32, bucket, red.numel()
    plan.copy_engine = ps.PS_COPY_NONE
    shard = shard_of(th, m, v, p, n)
    ps.ps_step_reduce_sumsq_static(spec, gl, 0.0, 0, ssd.data_ptr(), 0, 0, n, n, stream_handle())   # warm-up
    torch.cuda.synchronize()
    coef = orc.clip_coef(float(ssd.item()), 0.0, max_norm)
    assert coef < 1.0
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        plan.compute_stream = stream_handle()
        ps.ps_step_reduce_sumsq_static(spec, gl, 0.0, red.data_ptr(), ssd.data_ptr(), 0, 0, n, n,
                                       stream_handle())
        ps.ps_step_clip_coef(ssd.data_ptr(), 0, max_norm, cdev.data_ptr(), stream_handle())
        ps.ps_step_update_bucketed(spec, hp, shard, plan)
    torch.cuda.synchronize()
    assert np.array_equal(host(th).view(np.uint32), state[0].view(np.uint32))   # capture ran nothing
    s = orc.derive_scalars(t=t, n_devices=N, clip_coef=coef, **hpd)
    for k in range(3):
        red.fill_(float("nan")); ssd.fill_(-1.0); cdev.fill_(float("nan"))      # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        orc.step_f32(grads, s, *want)
        got = [host(x) for x in (th, m, v, p)]
        assert assert_state_parity(got, want, "replay %d" % k) == 0
        assert host(cdev)[0] == np.float32(coef)


# ---- bucket pipeline ----

def _bucketed(spec, hp, state, src_np, dtype, n, valid, bucket, engine, timed=False,
              schedule=ps.PS_SCHED_AUTO):
    th, m, v, p = [dev(a) for a in state]
    esz = 2 if dtype == "bf16" else 4
    N = len(src_np)
    src = [dev(g) for g in src_np]
    staging = [torch.zeros(N * bucket * esz, dtype=torch.uint8, device="cuda") for _ in range(2)]
    copy, comp = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    plan = ps.ps_bucket_plan_t()
    arr = (C.c_void_p * N)(*[s.data_ptr() for s in src])
    plan.source = C.cast(arr, C.POINTER(C.c_void_p))
    plan.n_contrib, plan.dtype = N, (ps.PS_BF16 if dtype == "bf16" else ps.PS_F32)
    plan.bucket_elems, plan.source_elems = bucket, src_np[0].shape[0]
    plan.staging[0], plan.staging[1] = staging[0].data_ptr(), staging[1].data_ptr()
    plan.copy_stream, plan.compute_stream = copy.cuda_stream, comp.cuda_stream
    plan.copy_engine, plan.schedule = engine, schedule
    n_b = -(-n // bucket)
    ms = (C.c_float * n_b)()
    if timed:
        plan.kernel_ms, plan.kernel_ms_len = ms, n_b
    ps.ps_step_update_bucketed(spec, hp, shard_of(th, m, v, p, n, valid), plan)
    torch.cuda.synchronize()
    return [host(x) for x in (th, m, v, p)], list(ms)


def _periodic(src_np, n):
    """What the pipeline reads: element e of the shard comes from source[e % len(source)]."""
    reps = -(-n // src_np[0].shape[0])
    return [np.ascontiguousarray(np.tile(g, reps)[:n]) for g in src_np]


@pytest.mark.parametrize("engine,schedule", [(ps.PS_COPY_KERNEL, ps.PS_SCHED_AUTO),
                                             (ps.PS_COPY_KERNEL, ps.PS_SCHED_OVERLAP),
                                             (ps.PS_COPY_MEMCPY, ps.PS_SCHED_AUTO),
                                             (ps.PS_COPY_MEMCPY, ps.PS_SCHED_ALTERNATE),
                                             (ps.PS_COPY_NONE, ps.PS_SCHED_AUTO),
                                             (ps.PS_COPY_REDUCE, ps.PS_SCHED_AUTO),
                                             (ps.PS_COPY_REDUCE, ps.PS_SCHED_OVERLAP)])
@pytest.mark.parametrize("timed", [False, True])
def test_bucketed_step_matches_oracle(timed, engine, schedule):
    bucket, N = 2 * TILE + 512, 8          # 4608: a multiple of 512 so that both engines apply
    n = 4 * bucket + 1259                   # 5 buckets, the last one short and ragged
    valid = n - 3
    n_b = -(-n // bucket)
    _say("bucketed n=%d bucket=%d (%d buckets) timed=%s engine=%d schedule=%d" %
         (n, bucket, n_b, timed, engine, schedule))
    spec = ps.ps_spec_preset("zero3", N, 7, n * N)
    src = [gen.gradient(n_b * bucket, 41, 0, r, "bf16", 1e-4) for r in range(N)]   # every bucket resident
    state = [gen.master(n, 41), *gen.moments(n, 41, True), np.full(n, 0xABCD, np.uint16)]
    hpd, hp = hp_of(None, 1000)
    want = [a.copy() for a in state]
    orc.step_f32(_periodic(src, n), orc.derive_scalars(t=1000, n_devices=N, **hpd), *want, lo=0, hi=valid)
    got, ms = _bucketed(spec, hp, state, src, "bf16", n, valid, bucket, engine, timed, schedule)
    assert assert_state_parity(got, want, "bucketed") == 0
    for g, a in zip(got, state):
        assert np.array_equal(g[valid:].view(np.uint8), a[valid:].view(np.uint8))
    if timed:
        assert all(x > 0 for x in ms)


@pytest.mark.parametrize("dtype,engine,pool", [("f32", ps.PS_COPY_MEMCPY, 2 * TILE),    # pool of 2 buckets
                                               ("f32", ps.PS_COPY_KERNEL, 2 * TILE),
                                               ("bf16", ps.PS_COPY_KERNEL, 1536),        # shorter than a bucket,
                                               ("f32", ps.PS_COPY_KERNEL, 512),          # buckets straddle the wrap
                                               ("f32", ps.PS_COPY_NONE, 2 * TILE),       # read in place: whole
                                               ("bf16", ps.PS_COPY_NONE, 1536),          # buckets, pieces of a
                                               ("bf16", ps.PS_COPY_NONE, 512),           # bucket, many pieces
                                               ("f32", ps.PS_COPY_REDUCE, 2 * TILE),     # the reduce kernel as
                                               ("bf16", ps.PS_COPY_REDUCE, 1536),        # the staging engine,
                                               ("bf16", ps.PS_COPY_REDUCE, 512)])        # same source shapes
def test_bucketed_step_with_a_repeating_source_pool(dtype, engine, pool):
    """A source shorter than the shard repeats: element e reads source[e % source_elems]
    (how the benchmark feeds 33 buckets from a small resident pool)."""
    n, N, bucket = 6 * TILE + 40, 4, TILE
    _say("bucketed from a pool of %d elements, n=%d %s engine=%d" % (pool, n, dtype, engine))
    spec = ps.ps_spec_preset("zero3", N, 0, n * N)
    src = [gen.gradient(pool, 43, 0, r, dtype, 1e-3) for r in range(N)]
    state = [gen.master(n, 43), *gen.moments(n, 43, False), np.zeros(n, np.uint16)]
    hpd, hp = hp_of(None, 1)
    want = [a.copy() for a in state]
    orc.step_f32(_periodic(src, n), orc.derive_scalars(t=1, n_devices=N, **hpd), *want)
    got, _ = _bucketed(spec, hp, state, src, dtype, n, n, bucket, engine)
    assert assert_state_parity(got, want, "pool") == 0


def test_bucket_loop_geometry_at_random():
    """Forty seeded draws of shard length, valid length, bucket size, source length and
    contribution count for the loop that reads in place (the source wraps anywhere inside a
    bucket, buckets end anywhere) and for the staged pipeline; each compared with the oracle
    on every element, pads included."""
    rng = np.random.default_rng(20260102)
    for case in range(40):
        N = int(rng.integers(1, 9))
        dtype = "bf16" if N > 1 and rng.random() < 0.6 else "f32"
        if N == 1:
            dtype = "f32"                                           # one contribution: a pre-reduced gradient
        bucket = int(rng.integers(1, 40)) * 8 * int(rng.choice([1, 8, 64]))
        n = int(rng.integers(1, 9)) * bucket + int(rng.integers(0, bucket // 8 + 1)) * 8
        valid = n - int(rng.integers(0, min(n, 300)))
        pool = int(rng.integers(1, 2 + n // 512)) * 512
        engine = (ps.PS_COPY_NONE, ps.PS_COPY_KERNEL, ps.PS_COPY_NONE, ps.PS_COPY_REDUCE)[case % 4]
        _say("random bucket loop %d: n=%d valid=%d bucket=%d pool=%d N=%d %s engine=%d" %
             (case, n, valid, bucket, pool, N, dtype, engine))
        spec = ps.ps_spec_preset("zero3", max(N, 2), 0, n * max(N, 2))
        src = [gen.gradient(pool, 59, case, r, dtype, 1e-3) for r in range(N)]
        state = [gen.master(n, 59 + case), *gen.moments(n, 59 + case, True), np.full(n, 0x1234, np.uint16)]
        hpd, hp = hp_of(None, 3 + case, grad_scale=1.0 if N == 1 else 0.0)
        want = [a.copy() for a in state]
        orc.step_f32(_periodic(src, n), orc.derive_scalars(t=3 + case, n_devices=max(N, 2),
                                                             grad_scale=1.0 if N == 1 else 0.0, **hpd),
                     *want, lo=0, hi=valid)
        got, _ = _bucketed(spec, hp, state, src, dtype, n, valid, bucket, engine)
        assert assert_state_parity(got, want, "random case %d" % case) == 0
        for g, a in zip(got, state):
            assert np.array_equal(g[valid:].view(np.uint8), a[valid:].view(np.uint8))


def test_residency_override_changes_speed_never_results():
    """ps_probe_set_update_residency is a measurement aid: with any cap, or none, the update
    writes the same bits."""
    n, N = 70 * TILE + 9, 8
    spec = ps.ps_spec_preset("zero3", N, 0, n * N)
    grads = [gen.gradient(n, 61, 0, r, "bf16", 1e-3) for r in range(N)]
    state = [gen.master(n, 61), *gen.moments(n, 61, True), np.zeros(n, np.uint16)]
    hpd, hp = hp_of(None, 4)
    ref = None
    try:
        for cap in (0, 3, 8, 32, 40):
            ps.ps_probe_set_update_residency(cap)
            got = _run_gpu(spec, hp, state, grads, "bf16", n)
            if ref is None:
                ref = got
            for a, b in zip(got, ref):
                assert np.array_equal(a.view(np.uint8), b.view(np.uint8)), "cap %d changed the result" % cap
        with pytest.raises(ps.PsError) as e:
            ps.ps_probe_set_update_residency(2)
        assert e.value.status == ps.PS_ERANGE
    finally:
        ps.ps_probe_set_update_residency(0)
    want = [a.copy() for a in state]
    orc.step_f32(grads, orc.derive_scalars(t=4, n_devices=N, **hpd), *want)
    assert assert_state_parity(ref, want, "residency") == 0


def test_arena_that_cannot_be_had_fails_cleanly():
    """A piece larger than the device's memory: the call reports the runtime's error, leaves
    nothing mapped or reserved behind, and the next arena is created as usual."""
    free_before = torch.cuda.mem_get_info()[0]
    with pytest.raises(ps.PsError) as e:
        ps.ps_arena_create(1 << 38, 1 << 38, [4, 2])              # pieces of 1 TiB and 512 GiB
    assert e.value.status == ps.PS_EHIP and e.value.detail
    assert abs(torch.cuda.mem_get_info()[0] - free_before) < (64 << 20)
    levels = []
    for _ in range(3):                      # the runtime keeps some memory of its own after the first
        arena = ps.ps_arena_create(1 << 24, 1 << 20, [4, 2])      # mapping; after that nothing may grow
        assert ps.ps_arena_buffer(arena, 0) and ps.ps_arena_buffer(arena, 1)
        ps.ps_arena_destroy(arena)
        levels.append(torch.cuda.mem_get_info()[0])
    assert levels[1] - levels[2] < (8 << 20) and free_before - levels[2] < (512 << 20)


def test_step_on_arena_buffers_matches_oracle():
    """Flat buffers whose physical memory is created chunk by chunk (ps_arena_create): the
    bucket loop reads the contributions in place from them.  Chunks of 2^20 elements, a ragged
    last chunk, canaries past the valid range."""
    from synth import device as dgen
    chunk, N = 1 << 20, 4
    n = 2 * chunk + 12345 * 8
    valid = n - 5
    _say("arena: n=%d in chunks of %d, N=%d bf16, in-place bucket loop" % (n, chunk, N))
    spec = ps.ps_spec_preset("zero3", N, 1, n * N)
    arena = ps.ps_arena_create(n, chunk, [2] * N + [4, 4, 4, 2])
    try:
        ptrs = [ps.ps_arena_buffer(arena, k) for k in range(N + 4)]
        assert all(p and p % (2 << 20) == 0 for p in ptrs) and ps.ps_arena_buffer(arena, N + 4) == 0
        src_np = [gen.gradient(n, 47, 0, r, "bf16", 1e-3) for r in range(N)]
        state = [gen.master(n, 47), *gen.moments(n, 47, True), np.full(n, 0x5A5A, np.uint16)]
        views = [dgen.as_tensor(ptrs[r], n, torch.bfloat16) for r in range(N)]
        views += [dgen.as_tensor(ptrs[N + j], n, torch.float32) for j in range(3)]
        views.append(dgen.as_tensor(ptrs[N + 3], n, torch.bfloat16))
        for t_, a in zip(views, src_np + state):
            t_.copy_(dev(a).view(t_.dtype))
        hpd, hp = hp_of(None, 7)
        plan = ps.ps_bucket_plan_t()
        arr = (C.c_void_p * N)(*ptrs[:N])
        plan.source = C.cast(arr, C.POINTER(C.c_void_p))
        plan.n_contrib, plan.dtype, plan.bucket_elems, plan.source_elems = N, ps.PS_BF16, chunk, -(-n // 512) * 512
        plan.compute_stream, plan.copy_engine = stream_handle(), ps.PS_COPY_NONE
        sh = ps.ps_shard_t(ptrs[N], ptrs[N + 1], ptrs[N + 2], ptrs[N + 3], n, valid, ps.PS_BF16, 0)
        ps.ps_step_update_bucketed(spec, hp, sh, plan)
        torch.cuda.synchronize()
        want = [a.copy() for a in state]
        orc.step_f32(src_np, orc.derive_scalars(t=7, n_devices=N, **hpd), *want, lo=0, hi=valid)
        got = [host(t_) for t_ in views[N:]]
        assert assert_state_parity(got, want, "arena") == 0
        for g, a in zip(got, state):
            assert np.array_equal(g[valid:].view(np.uint8), a[valid:].view(np.uint8))
        del views, t_
    finally:
        torch.cuda.synchronize()
        ps.ps_arena_destroy(arena)


# ---- the other data-parallel rows: ZeRO-1 and gradient accumulation ----

@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_zero1_replicated_gradient_slice(dtype):
    """ZeRO-1: the gradient is one all-reduced, full-length replicated buffer; device i
    updates its Omega shard from slice i and writes slice i of the replicated parameters."""
    n, N, i = 4 * TILE + 264, 4, 2
    _say("zero1 n=%d shard %d of %d, %s" % (n, i, N, dtype))
    spec = ps.ps_spec_preset("zero1", N, i, n * N)
    c = ps.ps_cost_eval(spec)
    g_full = gen.gradient(n * N, 81, 0, 0, dtype, std=4e-3)          # stands for the all-reduced sum
    state = [gen.master(n, 81), *gen.moments(n, 81, True), np.zeros(n, np.uint16)]
    hpd, hp = hp_of(None, 9)
    want = [a.copy() for a in state]
    sl = slice(c.shard_offset, c.shard_offset + n)
    orc.step_f32([np.ascontiguousarray(g_full[sl])], orc.derive_scalars(t=9, n_devices=N, **hpd), *want)
    th, m, v = [dev(a) for a in state[:3]]
    full_p = dev(np.full(n * N, 0x7777, np.uint16))
    gd = dev(g_full)
    before = host(gd).copy()
    ps.ps_step_update(spec, hp, shard_of(th, m, v, full_p, n), grads_of([gd], dtype), 0, n,
                      stream_handle())
    torch.cuda.synchronize()
    p = host(full_p)
    got = [host(th), host(m), host(v), p[sl]]
    assert assert_state_parity(got, want, "zero1") == 0
    assert (p[:c.shard_offset] == 0x7777).all() and (p[c.shard_offset + n:] == 0x7777).all()
    assert np.array_equal(host(gd).view(np.uint8), before.view(np.uint8))


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_data_parallel_every_replica_updates_the_whole_tensor(dtype):
    """Data parallelism (all R): each of the N devices applies the all-reduced gradient
    to the whole state.  One call per device with its own copy of the state: all copies
    end up identical to the oracle's single unsharded update (state consistency for
    replicated state), in two ranges that split the tensor at an odd tile."""
    psi, N = 3 * TILE + 1000, 4
    _say("data parallel psi=%d N=%d %s" % (psi, N, dtype))
    g_sum = gen.gradient(psi, 19, 0, 0, dtype, std=4e-3)             # stands for the all-reduced sum
    state = [gen.master(psi, 19), *gen.moments(psi, 19, True), np.zeros(psi, np.uint16)]
    hpd, hp = hp_of(None, 4)
    want = [a.copy() for a in state]
    orc.step_f32([g_sum], orc.derive_scalars(t=4, n_devices=N, **hpd), *want)     # mean = sum / N
    gd = dev(g_sum)
    cut = TILE + 8
    for i in range(N):
        spec = ps.ps_spec_preset("dp", N, i, psi)
        t = [dev(a) for a in state]
        sh = shard_of(*t, psi)
        ps.ps_step_update(spec, hp, sh, grads_of([gd], dtype), 0, cut, stream_handle())
        ps.ps_step_update(spec, hp, sh, grads_of([gd], dtype), cut, psi - cut, stream_handle())
        torch.cuda.synchronize()
        got = [host(x) for x in t]
        assert assert_state_parity(got, want, "dp replica %d" % i) == 0
        assert np.array_equal(got[3], want[3])


@pytest.mark.parametrize("strategy", ["zero1", "dp"])
def test_clip_phases_on_a_replicated_gradient(strategy):
    """Clipping under pi_G = R: phase 1 reads this device's range of the all-reduced
    buffer (its slice under ZeRO-1, everything under data parallelism), phase 2 updates
    from the reduced mean with the coefficient."""
    N, i = 4, 3
    psi = N * (2 * TILE + 520)
    spec = ps.ps_spec_preset(strategy, N, i, psi)
    c = ps.ps_cost_eval(spec)
    off, n = (0, psi) if strategy == "dp" else (c.shard_offset, c.shard_len)
    _say("clip on a replicated gradient, %s: range [%d,+%d) of %d" % (strategy, off, n, psi))
    g_sum = gen.gradient(psi, 29, 0, 0, "f32", std=5e-2)
    mine = np.ascontiguousarray(g_sum[off:off + n])
    mean, ss = orc.mean_sumsq([mine], 1.0 / N)
    coef = orc.clip_coef(ss, 0.0 if strategy == "dp" else 3 * ss, 1.0)
    assert coef < 1.0
    state = [gen.master(n, 29), *gen.moments(n, 29, True), np.zeros(n, np.uint16)]
    hpd, _ = hp_of(None, 6)
    want = [a.copy() for a in state]
    orc.step_f32([mine], orc.derive_scalars(t=6, n_devices=N, clip_coef=coef, **hpd), *want)
    gd = dev(g_sum)
    red = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
    ssd = torch.zeros(1, dtype=torch.float64, device="cuda")
    ws = torch.empty(ps.ps_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    ps.ps_step_reduce_sumsq(spec, grads_of([gd], "f32"), 0.0, red.data_ptr(), ssd.data_ptr(), 0,
                            ws.data_ptr(), ws.numel(), 0, n, n, stream_handle())
    torch.cuda.synchronize()
    assert np.array_equal(host(red).view(np.uint32), mean.view(np.uint32))
    assert abs(float(ssd.item()) - ss) <= 1e-12 * ss
    th, m, v = [dev(a) for a in state[:3]]
    full_p = dev(np.full(psi, 0x6666, np.uint16))
    _, hp = hp_of(None, 6, grad_scale=1.0, clip_coef=coef)
    # Phase 1 leaves the mean in sharded form (element 0 = first element of this device's
    # range), so under ZeRO-1 phase 2 is a pi_G = S call on the same geometry (the ZeRO-2
    # row); under data parallelism the range is the whole tensor and the spec stays.
    spec2 = ps.ps_spec_preset("zero2", N, i, psi) if strategy == "zero1" else spec
    ps.ps_step_update(spec2, hp, shard_of(th, m, v, full_p, n), grads_of([red], "f32"), 0, n,
                      stream_handle())
    torch.cuda.synchronize()
    p = host(full_p)
    got = [host(th), host(m), host(v), p[off:off + n]]
    assert assert_state_parity(got, want, "clip %s" % strategy) == 0
    assert (p[:off] == 0x6666).all() and (p[off + n:] == 0x6666).all()


@pytest.mark.parametrize("dtype,N", [("bf16", 8), ("f32", 6), ("bf16", 3)])
def test_gradient_accumulation_then_update(dtype, N):
    """k micro-batches accumulate into the FP32 shard (fixed order inside a micro-batch,
    micro-batches in arrival order), then one update with grad_scale = 1/(N k)."""
    n, k = 6 * TILE + 250 + 5, 4
    valid = n - 3
    _say("accumulate k=%d n=%d valid=%d N=%d %s" % (k, n, valid, N, dtype))
    spec = ps.ps_spec_preset("zero3", N, 1, n * N)
    acc_want = np.full(n, np.float32(7.0))
    acc_dev = dev(acc_want.copy())
    for j in range(k):
        grads = [gen.gradient(n, 83, j, r, dtype, std=1e-3) for r in range(N)]
        orc.accumulate(grads, acc_want, overwrite=(j == 0), lo=0, hi=valid)
        gd = [dev(g) for g in grads]
        # two calls per micro-batch: the range may arrive in pieces
        cut = 3 * TILE + 8
        ps.ps_step_accumulate(spec, grads_of(gd, dtype), acc_dev.data_ptr(), j == 0, 0, cut, valid,
                              stream_handle())
        ps.ps_step_accumulate(spec, grads_of(gd, dtype, cut), acc_dev.data_ptr(), j == 0, cut,
                              n - cut, valid, stream_handle())
        torch.cuda.synchronize()
    assert np.array_equal(host(acc_dev).view(np.uint32), acc_want.view(np.uint32))   # pad (7.0) included
    state = [gen.master(n, 83), *gen.moments(n, 83, True), np.zeros(n, np.uint16)]
    scale = 1.0 / (N * k)
    hpd, hp = hp_of(None, 21, grad_scale=scale)
    want = [a.copy() for a in state]
    orc.step_f32([acc_want], orc.derive_scalars(t=21, n_devices=N, grad_scale=scale, **hpd), *want,
                 lo=0, hi=valid)
    th, m, v, p = [dev(a) for a in state]
    ps.ps_step_update(spec, hp, shard_of(th, m, v, p, n, valid), grads_of([acc_dev], "f32"), 0, n,
                      stream_handle())
    torch.cuda.synchronize()
    assert assert_state_parity([host(x) for x in (th, m, v, p)], want, "accumulated") == 0


@pytest.mark.parametrize("dtype,N", [("bf16", 8), ("f32", 6), ("bf16", 3), ("f16", 4), ("bf16", 12),
                                     ("f32", 1)])
def test_last_micro_batch_goes_straight_into_the_update(dtype, N):
    """The last of k micro-batches needs no accumulation pass: ps_step_update adds the
    accumulator of the k - 1 before it to the contributions' sum.  Bit for bit the oracle's
    accumulate-then-update; the accumulator is only read."""
    n, k = 5 * TILE + 250 + 5, 3
    valid = n - 3
    _say("fused last micro-batch k=%d n=%d valid=%d N=%d %s" % (k, n, valid, N, dtype))
    spec = ps.ps_spec_preset("zero3", max(N, 2), 1, n * max(N, 2))
    acc_want = np.full(n, np.float32(7.0))
    for j in range(k - 1):
        grads = [gen.gradient(n, 87, j, r, dtype, std=1e-3) for r in range(N)]
        orc.accumulate(grads, acc_want, overwrite=(j == 0), lo=0, hi=valid)
    acc_dev = dev(acc_want.copy())          # the first k - 1 passes are another test's business
    before = acc_want.copy()
    last = [gen.gradient(n, 87, k - 1, r, dtype, std=1e-3) for r in range(N)]
    orc.accumulate(last, acc_want, overwrite=False, lo=0, hi=valid)
    image = np.full(n, np.float16(-77.0), np.float16) if dtype == "f16" else np.zeros(n, np.uint16)
    state = [gen.master(n, 87), *gen.moments(n, 87, True), image]
    scale = 1.0 / (N * k)
    hpd, hp = hp_of(None, 9, grad_scale=scale)
    want = [a.copy() for a in state]
    orc.step_f32([acc_want], orc.derive_scalars(t=9, n_devices=max(N, 2), grad_scale=scale, **hpd),
                 *want, lo=0, hi=valid)
    th, m, v, p = [dev(a) for a in state]
    gd = [dev(g) for g in last]
    shard = shard_of(th, m, v, p, n, valid)
    cut = 2 * TILE + 8                      # two calls: the accumulator follows elem_offset
    ps.ps_step_update(spec, hp, shard, grads_of(gd, dtype, accum=acc_dev), 0, cut, stream_handle())
    ps.ps_step_update(spec, hp, shard, grads_of(gd, dtype, cut, accum=acc_dev), cut, n - cut,
                      stream_handle())
    torch.cuda.synchronize()
    assert assert_state_parity([host(x) for x in (th, m, v, p)], want, "fused last micro-batch") == 0
    assert np.array_equal(host(acc_dev).view(np.uint32), before.view(np.uint32))


# ---- offloaded optimizer state (ZeRO-Offload row) ----

def _pack_host(state, bucket):
    """Host image in the packed layout: per bucket master | m | v | parameters, each array's
    piece bucket elements long (the last bucket only partly meaningful, the rest canaries)."""
    n = state[0].shape[0]
    n_b = -(-n // bucket)
    buf = np.full(n_b * 14 * bucket, 0xEE, np.uint8)
    for b in range(n_b):
        lo, hi = b * bucket, min((b + 1) * bucket, n)
        base = b * 14 * bucket
        for j, off in enumerate((0, 4 * bucket, 8 * bucket)):
            buf[base + off:base + off + 4 * (hi - lo)] = state[j][lo:hi].view(np.uint8)
        buf[base + 12 * bucket:base + 12 * bucket + 2 * (hi - lo)] = state[3][lo:hi].view(np.uint8)
    return buf


def _unpack_host(buf, n, bucket):
    out = [np.empty(n, np.float32) for _ in range(3)] + [np.empty(n, np.uint16)]
    for b in range(-(-n // bucket)):
        lo, hi = b * bucket, min((b + 1) * bucket, n)
        base = b * 14 * bucket
        for j, off in enumerate((0, 4 * bucket, 8 * bucket)):
            out[j][lo:hi] = buf[base + off:base + off + 4 * (hi - lo)].view(np.float32)
        out[3][lo:hi] = buf[base + 12 * bucket:base + 12 * bucket + 2 * (hi - lo)].view(np.uint16)
    return out


@pytest.mark.parametrize("n_slots,dtype,N,packed", [(3, "bf16", 4, False), (2, "bf16", 4, False),
                                                    (3, "f32", 6, False), (3, "bf16", 4, True),
                                                    (2, "f32", 6, True)])
def test_offloaded_state_streams_through_the_device(n_slots, dtype, N, packed):
    n = 5 * TILE + 100
    valid = n - 3
    bucket = TILE + 8
    _say("offload n=%d bucket=%d slots=%d N=%d %s packed=%s" % (n, bucket, n_slots, N, dtype, packed))
    spec = ps.ps_spec_preset("zero_offload", N, 2, n * N)
    grads = [gen.gradient(n, 111, 0, r, dtype) for r in range(N)]
    state = [gen.master(n, 111), *gen.moments(n, 111, True), np.full(n, 0x5555, np.uint16)]
    hpd, hp = hp_of(None, 12)
    want = [a.copy() for a in state]
    orc.step_f32(grads, orc.derive_scalars(t=12, n_devices=N, **hpd), *want, lo=0, hi=valid)
    gd = [dev(g) for g in grads]
    slots = [torch.zeros(14 * bucket, dtype=torch.uint8, device="cuda") for _ in range(n_slots)]
    s1, s2, s3 = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    plan = ps.ps_offload_plan_t()
    if packed:
        image = _pack_host(state, bucket)
        pinned = torch.from_numpy(image.copy()).pin_memory()
        plan.host_layout, plan.host_packed = ps.PS_HOST_PACKED, pinned.data_ptr()
    else:
        pinned = [torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).pin_memory()
                  for a in state]
        plan.host_master, plan.host_m, plan.host_v, plan.host_param_out = [t.data_ptr() for t in pinned]
    plan.len, plan.valid_len, plan.bucket_elems, plan.n_slots = n, valid, bucket, n_slots
    for k, t in enumerate(slots):
        plan.slot[k] = t.data_ptr()
    plan.h2d_stream, plan.compute_stream, plan.d2h_stream = s1.cuda_stream, s2.cuda_stream, s3.cuda_stream
    ps.ps_step_update_offloaded(spec, hp, plan, grads_of(gd, dtype))
    torch.cuda.synchronize()
    if packed:
        got = _unpack_host(pinned.numpy(), n, bucket)
        # bytes of the image that belong to no element (the short last bucket's tail) keep their canary
        unused = _pack_host([np.zeros(n, np.float32)] * 3 + [np.zeros(n, np.uint16)], bucket) == 0xEE
        assert unused.any() and (pinned.numpy()[unused] == 0xEE).all()
    else:
        got = [t.numpy().copy() for t in pinned]
        got[3] = got[3].view(np.uint16)
    assert assert_state_parity(got, want, "offload") == 0
    for g, a in zip(got, state):                                   # pad untouched on the host
        assert np.array_equal(g[valid:].view(np.uint8), a[valid:].view(np.uint8))


def test_offloaded_steps_back_to_back_with_one_final_sync():
    """Three offloaded steps enqueued one after the other on the same streams and slots,
    the host waiting only once at the end: every step's uploads must see the previous
    step's downloads (state consistency across steps, Theorem 4)."""
    n, N, bucket, n_slots = 9 * TILE + 44, 4, 2 * TILE, 2
    _say("offload back to back: n=%d bucket=%d slots=%d, 3 steps, one sync" % (n, bucket, n_slots))
    spec = ps.ps_spec_preset("zero_offload", N, 0, n * N)
    state = [gen.master(n, 113), *gen.moments(n, 113, True), np.zeros(n, np.uint16)]
    want = [a.copy() for a in state]
    pinned = [torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a.copy()).pin_memory()
              for a in state]
    slots = [torch.zeros(14 * bucket, dtype=torch.uint8, device="cuda") for _ in range(n_slots)]
    s1, s2, s3 = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    plan = ps.ps_offload_plan_t()
    plan.host_master, plan.host_m, plan.host_v, plan.host_param_out = [t.data_ptr() for t in pinned]
    plan.len, plan.valid_len, plan.bucket_elems, plan.n_slots = n, n, bucket, n_slots
    for k, t in enumerate(slots):
        plan.slot[k] = t.data_ptr()
    plan.h2d_stream, plan.compute_stream, plan.d2h_stream = s1.cuda_stream, s2.cuda_stream, s3.cuda_stream
    all_g = [[gen.gradient(n, 113, t, r, "bf16") for r in range(N)] for t in (1, 2, 3)]
    all_gd = [[dev(g) for g in gs] for gs in all_g]
    torch.cuda.synchronize()
    for t, gd in zip((1, 2, 3), all_gd):
        _, hp = hp_of(None, t)
        ps.ps_step_update_offloaded(spec, hp, plan, grads_of(gd, "bf16"))      # no wait in between
    torch.cuda.synchronize()
    for t, gs in zip((1, 2, 3), all_g):
        hpd, _ = hp_of(None, t)
        orc.step_f32(gs, orc.derive_scalars(t=t, n_devices=N, **hpd), *want)
    got = [t.numpy().copy() for t in pinned]
    got[3] = got[3].view(np.uint16)
    assert assert_state_parity(got, want, "offload x3") == 0


# ---- verification protocol kernels ----

@pytest.mark.parametrize("dtype,n", [("f32", 9 * TILE + 777), ("bf16", 9 * TILE + 777),
                                     ("f32", 1200 * TILE + 131), ("bf16", 100)])
def test_verify_relative_difference(dtype, n):
    _say("verify diff n=%d %s" % (n, dtype))
    a = gen.gradient(n, 101, 0, 0, dtype, std=1e-2)
    b = gen.gradient(n, 101, 0, 1, dtype, std=1e-2)
    sd, sa = orc.diff_sumsq(a, b)
    ad, bd = dev(a), dev(b)
    esz = 2 if dtype == "bf16" else 4
    ws = torch.empty(ps.ps_verify_workspace_bytes(n * esz), dtype=torch.uint8, device="cuda")
    out = torch.zeros(2, dtype=torch.float64, device="cuda")
    dt = ps.PS_BF16 if dtype == "bf16" else ps.PS_F32

    def call(acc=0, lo=0, cnt=n):
        ps.ps_verify_diff_sumsq(ad.data_ptr() + lo * esz, bd.data_ptr() + lo * esz, dt, cnt,
                                out.data_ptr(), acc, ws.data_ptr(), ws.numel(), stream_handle())
        torch.cuda.synchronize()
        return out.cpu().numpy().copy()
    got = call()
    assert abs(got[0] - sd) <= 1e-12 * sd and abs(got[1] - sa) <= 1e-12 * sa
    assert np.array_equal(call(), got)                               # reproducible bit for bit
    if n > 64:                                                       # pieces accumulate
        cut = (n // 3) // 8 * 8
        call(0, 0, cut)
        two = call(1, cut, n - cut)
        assert abs(two[0] - sd) <= 1e-12 * sd and abs(two[1] - sa) <= 1e-12 * sa
    ps.ps_verify_diff_sumsq(ad.data_ptr(), ad.data_ptr(), dt, n, out.data_ptr(), 0, ws.data_ptr(),
                            ws.numel(), stream_handle())
    assert out.cpu().numpy()[0] == 0.0                               # identical buffers: exactly zero


@pytest.mark.parametrize("n_words", [1, 2, 127, 128, 129, 5 * 1024 + 77, 700 * 1024 + 3])
def test_verify_checksum_is_bit_exact(n_words):
    _say("verify checksum words=%d" % n_words)
    w = np.random.default_rng(n_words).integers(0, 2 ** 63, n_words, dtype=np.uint64)
    want = orc.checksum(w)
    wd = torch.from_numpy(w.view(np.int64)).cuda()
    ws = torch.empty(ps.ps_verify_workspace_bytes(n_words * 8), dtype=torch.uint8, device="cuda")
    out = torch.zeros(1, dtype=torch.int64, device="cuda")

    def call(ptr, nbytes, first=0, acc=0):
        ps.ps_verify_checksum(ptr, nbytes, first, out.data_ptr(), acc, ws.data_ptr(), ws.numel(),
                              stream_handle())
        torch.cuda.synchronize()
        return int(out.cpu().numpy().view(np.uint64)[0])
    assert call(wd.data_ptr(), n_words * 8) == want
    if n_words > 4:                                                  # pieces add up modulo 2^64
        cut = (n_words // 2) // 2 * 2                                # keeps 16-byte alignment
        call(wd.data_ptr(), cut * 8)
        assert call(wd.data_ptr() + cut * 8, (n_words - cut) * 8, first=cut, acc=1) == want
        sw = w.copy(); sw[[0, n_words - 1]] = sw[[n_words - 1, 0]]   # a swap shows
        assert call(torch.from_numpy(sw.view(np.int64)).cuda().data_ptr(), n_words * 8) == orc.checksum(sw) != want


def test_verify_checksum_of_updated_state_matches_oracle():
    """The protocol's use: after a step, the checksum of the device's shard equals the
    checksum of the oracle's shard (identical bits => identical checksums)."""
    n, N = 4 * TILE + 8, 4
    _say("checksum after a step n=%d" % n)
    spec = ps.ps_spec_preset("zero3", N, 0, n * N)
    grads = [gen.gradient(n, 103, 0, r, "bf16") for r in range(N)]
    state = [gen.master(n, 103), *gen.moments(n, 103, True), np.zeros(n, np.uint16)]
    hpd, hp = hp_of(None, 4)
    want = [a.copy() for a in state]
    orc.step_f32(grads, orc.derive_scalars(t=4, n_devices=N, **hpd), *want)
    th, m, v, p = [dev(a) for a in state]
    ps.ps_step_update(spec, hp, shard_of(th, m, v, p, n), grads_of([dev(g) for g in grads], "bf16"),
                      0, n, stream_handle())
    ws = torch.empty(ps.ps_verify_workspace_bytes(n * 4), dtype=torch.uint8, device="cuda")
    out = torch.zeros(1, dtype=torch.int64, device="cuda")
    for t_dev, w_host in zip((th, m, v, p), want):
        ps.ps_verify_checksum(t_dev.data_ptr(), w_host.nbytes, 0, out.data_ptr(), 0, ws.data_ptr(),
                              ws.numel(), stream_handle())
        torch.cuda.synchronize()
        assert int(out.cpu().numpy().view(np.uint64)[0]) == orc.checksum(w_host)


# ---- memory safety and statelessness ----

GUARD = 4096  # bytes of guard band on each side of every device buffer


def _guarded(a):
    """Upload `a` into the middle of a larger byte buffer filled with 0xA5; return
    (whole, view-of-payload)."""
    raw = np.full(a.nbytes + 2 * GUARD, 0xA5, np.uint8)
    raw[GUARD:GUARD + a.nbytes] = a.view(np.uint8)
    whole = torch.from_numpy(raw).cuda()
    return whole, whole[GUARD:GUARD + a.nbytes]


def _guards_intact(whole, nbytes):
    h = whole.cpu().numpy()
    return (h[:GUARD] == 0xA5).all() and (h[GUARD + nbytes:] == 0xA5).all()


@pytest.mark.parametrize("dtype,N", [("bf16", 8), ("f32", 6), ("bf16", 3)])
def test_no_write_outside_the_buffers(dtype, N):
    n = 5 * TILE + 250 + 3
    valid = n - 2
    _say("guard bands n=%d N=%d %s: update, reduce+sumsq, bucketed" % (n, N, dtype))
    spec = ps.ps_spec_preset("zero3", N, 0, n * N)
    grads = [gen.gradient(n, 61, 0, r, dtype) for r in range(N)]
    state = [gen.master(n, 61), *gen.moments(n, 61, True), np.zeros(n, np.uint16)]
    bufs = [_guarded(a) for a in state]
    gbufs = [_guarded(g) for g in grads]
    _, hp = hp_of(None, 3)
    shard = ps.ps_shard_t(*[v.data_ptr() for _, v in bufs], n, valid)
    g = ps.make_grads([v.data_ptr() for _, v in gbufs], ps.PS_BF16 if dtype == "bf16" else ps.PS_F32)
    ps.ps_step_update(spec, hp, shard, g, 0, n, stream_handle())
    red_w, red = _guarded(np.zeros(n, np.float32))
    ss_w, ss = _guarded(np.zeros(1, np.float64))
    ws_w, ws = _guarded(np.zeros(ps.ps_workspace_bytes(n), np.uint8))
    ps.ps_step_reduce_sumsq(spec, g, 0.0, red.data_ptr(), ss.data_ptr(), 0, ws.data_ptr(),
                            ws.numel(), 0, n, valid, stream_handle())
    bucket = TILE + 8
    esz = 2 if dtype == "bf16" else 4
    st = [_guarded(np.zeros(N * bucket * esz, np.uint8)) for _ in range(2)]
    plan = ps.ps_bucket_plan_t()
    src_np = [gen.gradient(1024, 62, 0, r, dtype) for r in range(N)]
    src = [_guarded(a) for a in src_np]
    arr = (C.c_void_p * N)(*[v.data_ptr() for _, v in src])
    plan.source = C.cast(arr, C.POINTER(C.c_void_p))
    plan.n_contrib, plan.dtype = N, (ps.PS_BF16 if dtype == "bf16" else ps.PS_F32)
    plan.bucket_elems, plan.source_elems = bucket, 1024
    plan.staging[0], plan.staging[1] = st[0][1].data_ptr(), st[1][1].data_ptr()
    c1, c2 = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    plan.copy_stream, plan.compute_stream = c1.cuda_stream, c2.cuda_stream
    ps.ps_step_update_bucketed(spec, hp, shard, plan)
    torch.cuda.synchronize()
    for (whole, _), a in zip(bufs + gbufs + src, state + grads + src_np):
        assert _guards_intact(whole, a.nbytes)
    assert _guards_intact(red_w, n * 4) and _guards_intact(ss_w, 8)
    assert _guards_intact(ws_w, ps.ps_workspace_bytes(n))
    assert all(_guards_intact(w_, N * bucket * esz) for w_, _ in st)
    for (_, v), a in zip(gbufs + src, grads + src_np):                    # inputs are read-only
        assert np.array_equal(v.cpu().numpy(), a.view(np.uint8))


def test_checkpoint_and_resume_is_bit_identical():
    """The library keeps no state: 10 steps equal 5 steps, a copy of the flat buffers to
    the host and into fresh device buffers, and 5 more steps."""
    n, N = 3 * TILE + 77, 4
    _say("checkpoint/resume n=%d" % n)
    spec = ps.ps_spec_preset("zero3", N, 1, n * N)
    state = [gen.master(n, 71), *gen.moments(n, 71, False), np.zeros(n, np.uint16)]

    def run(bufs, steps):
        for t in steps:
            gd = [dev(gen.gradient(n, 71, t, r, "bf16")) for r in range(N)]
            _, hp = hp_of(None, t)
            ps.ps_step_update(spec, hp, shard_of(*bufs, n), grads_of(gd, "bf16"), 0, n, stream_handle())
            torch.cuda.synchronize()
    a = [dev(x) for x in state]
    run(a, range(1, 11))
    b = [dev(x) for x in state]
    run(b, range(1, 6))
    saved = [host(x).copy() for x in b]
    del b
    c = [dev(x) for x in saved]
    run(c, range(6, 11))
    for x, y in zip(a, c):
        assert np.array_equal(host(x).view(np.uint8), host(y).view(np.uint8))


# ---- the paper's verification protocol, end to end on the device ----

def test_protocol_gradient_integrity_check_on_device():
    """Item 1 of the protocol: the reduced gradient from N contributions against a
    reference, ||G_1 - G_N|| / ||G_1|| < 1e-5.  Another summation order passes; a lost
    or duplicated contribution and a wrong normaliser fail."""
    n, N = 20 * TILE + 96, 8
    _say("protocol: gradient integrity on device n=%d" % n)
    spec = ps.ps_spec_preset("zero3", N, 0, n * N)
    grads = [gen.gradient(n, 121, 0, r, "f32", std=1e-3) for r in range(N)]
    gd = [dev(g) for g in grads]
    ws = torch.empty(max(ps.ps_workspace_bytes(n), ps.ps_verify_workspace_bytes(n * 4)),
                     dtype=torch.uint8, device="cuda")
    ss = torch.zeros(1, dtype=torch.float64, device="cuda")
    out2 = torch.zeros(2, dtype=torch.float64, device="cuda")

    def mean_of(tensors, scale=0.0, n_dev=N):
        sp = ps.ps_spec_preset("zero3", n_dev, 0, n * n_dev)
        red = torch.zeros(n, dtype=torch.float32, device="cuda")
        ps.ps_step_reduce_sumsq(sp, grads_of(tensors, "f32"), scale, red.data_ptr(), ss.data_ptr(), 0,
                                ws.data_ptr(), ws.numel(), 0, n, n, stream_handle())
        return red

    def rel(a, b):
        ps.ps_verify_diff_sumsq(a.data_ptr(), b.data_ptr(), ps.PS_F32, n, out2.data_ptr(), 0,
                                ws.data_ptr(), ws.numel(), stream_handle())
        torch.cuda.synchronize()
        sd, sa = out2.cpu().tolist()
        return (sd / sa) ** 0.5
    ref = mean_of(gd)
    tol = 1e-5
    assert rel(ref, mean_of(gd)) == 0.0
    assert 0.0 < rel(ref, mean_of(gd[::-1])) < tol                      # reduction order: allowed
    assert rel(ref, mean_of(gd[:-1], 1.0 / N, N - 1)) > tol             # a device failed to contribute
    assert rel(ref, mean_of(gd[:-1] + [gd[0]])) > tol                   # a contribution counted twice
    assert rel(ref, mean_of(gd, 1.0)) > tol                             # divided by the wrong count
    # and against the oracle's own numbers
    want, _ = orc.mean_sumsq(grads, 1.0 / N)
    assert np.array_equal(host(ref).view(np.uint32), want.view(np.uint32))


def test_protocol_trajectory_100_steps_sharded_equals_single_device():
    """Item 3 of the protocol: 100 steps on N devices (each its own shard) against the
    single-device run with the same seed.  There is no loss here; the parameters
    themselves are compared, and they agree bit for bit."""
    psi, N, steps = 4 * (2 * TILE + 72), 4, 100
    _say("protocol: 100-step trajectory psi=%d N=%d" % (psi, N))
    full = [gen.master(psi, 131), *gen.moments(psi, 131, False), np.zeros(psi, np.uint16)]
    shards = []
    for i in range(N):
        spec = ps.ps_spec_preset("zero3", N, i, psi)
        c = ps.ps_cost_eval(spec)
        sl = slice(c.shard_offset, c.shard_offset + c.shard_len)
        shards.append((spec, c, sl, [dev(np.ascontiguousarray(a[sl])) for a in full]))
    for t in range(1, steps + 1):
        grads = [gen.gradient(psi, 131, t, r, "bf16", 1e-3) for r in range(N)]
        hpd, hp = hp_of(None, t, lr=1e-3)
        orc.step_f32(grads, orc.derive_scalars(t=t, n_devices=N, **hpd), *full)
        for spec, c, sl, bufs in shards:
            gd = [dev(np.ascontiguousarray(g[sl])) for g in grads]
            ps.ps_step_update(spec, hp, shard_of(*bufs, c.shard_len), grads_of(gd, "bf16"), 0,
                              c.shard_len, stream_handle())
        torch.cuda.synchronize()
    ws = torch.empty(ps.ps_verify_workspace_bytes(psi), dtype=torch.uint8, device="cuda")
    out = torch.zeros(1, dtype=torch.int64, device="cuda")
    for k in range(4):
        cat = np.concatenate([host(bufs[k]) for _, _, _, bufs in shards])
        assert np.array_equal(cat.view(np.uint8), full[k].view(np.uint8))
    # item 2 of the protocol: checksums of each shard agree with the single-device state
    for spec, c, sl, bufs in shards:
        ps.ps_verify_checksum(bufs[0].data_ptr(), c.shard_len * 4, 0, out.data_ptr(), 0,
                              ws.data_ptr(), ws.numel(), stream_handle())
        torch.cuda.synchronize()
        assert int(out.cpu().numpy().view(np.uint64)[0]) == orc.checksum(np.ascontiguousarray(full[0][sl]))
    assert np.abs(full[0] - gen.master(psi, 131)).max() > 1e-3          # a hundred steps did move it


def test_c_abi_without_python():
    """The prebuilt native driver (built by build()): library and oracle meet in one C++
    program, no Python or torch in between."""
    import os
    import subprocess
    exe = os.path.join(os.path.dirname(os.path.abspath(__file__)), "native", "abi_parity")
    if not os.path.exists(exe):
        pytest.skip("tests/native/abi_parity has not been built (run build())")
    _say("native C ABI driver")
    p = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=100)
    assert p.returncode == 0 and "abi parity ok" in p.stdout, p.stdout


def test_two_host_threads_on_two_streams():
    """No shared state in the library: two host threads step two different shards on two
    streams at once; each result equals its own oracle run, and an error raised in one
    thread does not show up as the other's last error."""
    import threading
    n, N = 6 * TILE + 40, 4
    _say("two threads, two streams, n=%d" % n)
    results, errors = {}, {}

    def work(tag, seed, t):
        try:
            torch.cuda.set_device(0)
            spec = ps.ps_spec_preset("zero3", N, tag, n * N)
            grads = [gen.gradient(n, seed, 0, r, "bf16") for r in range(N)]
            state = [gen.master(n, seed), *gen.moments(n, seed, True), np.zeros(n, np.uint16)]
            hpd, hp = hp_of(None, t)
            want = [a.copy() for a in state]
            orc.step_f32(grads, orc.derive_scalars(t=t, n_devices=N, **hpd), *want)
            s = torch.cuda.Stream()
            with torch.cuda.stream(s):
                bufs = [dev(a) for a in state]
                gd = [dev(g) for g in grads]
                s.synchronize()
                for _ in range(3):      # idempotent inputs: restore and repeat to overlap in time
                    for b, a in zip(bufs, state):
                        b.copy_(dev(a))
                    ps.ps_step_update(spec, hp, shard_of(*bufs, n), grads_of(gd, "bf16"), 0, n, s.cuda_stream)
                if tag == 1:
                    try:
                        ps.ps_step_update(spec, hp, shard_of(*bufs, n), grads_of(gd[:2], "bf16"), 0, n, s.cuda_stream)
                    except ps.PsError as e:
                        errors[tag] = e.status
                s.synchronize()
            results[tag] = assert_state_parity([host(b) for b in bufs], want, "thread %d" % tag)
            errors.setdefault(tag, ps.ps_last_error())
        except Exception as e:      # surface assertion failures from the thread
            results[tag] = e
    th = [threading.Thread(target=work, args=(0, 141, 3)), threading.Thread(target=work, args=(1, 142, 9))]
    for t in th:
        t.start()
    for t in th:
        t.join()
    assert results == {0: 0, 1: 0}, results
    assert errors[1] == ps.PS_EINVAL and errors[0] == ""


@pytest.mark.parametrize("engine", [ps.PS_COPY_MEMCPY, ps.PS_COPY_KERNEL])
def test_bucketed_step_from_pinned_host_source(engine):
    """The bucket source may be pinned host memory (contributions arriving over the host
    link): DMA copies overlap the update; the copy kernel reads the mapped host pages."""
    bucket, N = 2 * TILE, 4
    n = 3 * bucket + 520
    n_b = -(-n // bucket)
    _say("bucketed from pinned host memory n=%d engine=%d" % (n, engine))
    spec = ps.ps_spec_preset("zero3", N, 3, n * N)
    src_np = [gen.gradient(n_b * bucket, 151, 0, r, "bf16", 1e-3) for r in range(N)]
    src = [torch.from_numpy(g.view(np.int16)).pin_memory() for g in src_np]
    state = [gen.master(n, 151), *gen.moments(n, 151, True), np.zeros(n, np.uint16)]
    hpd, hp = hp_of(None, 33)
    want = [a.copy() for a in state]
    orc.step_f32([np.ascontiguousarray(g[:n]) for g in src_np],
                 orc.derive_scalars(t=33, n_devices=N, **hpd), *want)
    th, m, v, p = [dev(a) for a in state]
    staging = [torch.zeros(N * bucket * 2, dtype=torch.uint8, device="cuda") for _ in range(2)]
    copy, comp = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    plan = ps.ps_bucket_plan_t()
    arr = (C.c_void_p * N)(*[s.data_ptr() for s in src])
    plan.source = C.cast(arr, C.POINTER(C.c_void_p))
    plan.n_contrib, plan.dtype, plan.bucket_elems, plan.source_elems = N, ps.PS_BF16, bucket, n_b * bucket
    plan.staging[0], plan.staging[1] = staging[0].data_ptr(), staging[1].data_ptr()
    plan.copy_stream, plan.compute_stream = copy.cuda_stream, comp.cuda_stream
    plan.copy_engine, plan.schedule = engine, ps.PS_SCHED_AUTO
    ps.ps_step_update_bucketed(spec, hp, shard_of(th, m, v, p, n), plan)
    torch.cuda.synchronize()
    assert assert_state_parity([host(x) for x in (th, m, v, p)], want, "pinned source") == 0


# ---- IEEE binary16 gradients and parameters (the FP16 of the paper's Table 1) ----

LOSS_SCALE = 1024.0


def _f16_case(n, N, seed, valid=None, std=1e-3):
    """Scaled FP16 contributions (a loss scale of 1024 rides on grad_scale), FP32 state,
    FP16 parameters; returns (grads, state, oracle scalars dict, hp)."""
    grads = [gen.gradient(n, seed, 0, r, "f16", std=std * LOSS_SCALE, outlier_frac=0.01, outlier_mult=30.0)
             for r in range(N)]
    state = [gen.master(n, seed), *gen.moments(n, seed, True), np.full(n, np.float16(-77.0), np.float16)]
    gs = 1.0 / (N * LOSS_SCALE)
    hpd, hp = hp_of(None, 5, grad_scale=gs)
    return grads, state, orc.derive_scalars(t=5, n_devices=N, grad_scale=gs, **hpd), hp


@pytest.mark.parametrize("N", [2, 3, 8, 16])
def test_f16_update_ragged(N):
    n = 3 * TILE + 1234 + 3
    valid = n - 5
    _say("binary16 update n=%d valid=%d N=%d" % (n, valid, N))
    spec = ps.ps_spec_preset("zero3", N, 0, n * N)
    grads, state, s, hp = _f16_case(n, N, 201)
    want = [a.copy() for a in state]
    orc.step_f32(grads, s, *want, lo=0, hi=valid)
    got = _run_gpu(spec, hp, state, grads, "f16", n, valid)
    assert assert_state_parity(got, want, "f16") == 0
    for g, a in zip(got, state):                                   # pads untouched, byte for byte
        assert np.array_equal(g[valid:].view(np.uint8), a[valid:].view(np.uint8))
    # a pre-reduced FP32 gradient with FP16 parameters (clip phase 2, accumulation)
    red = orc.reduce_sum(grads)
    want = [a.copy() for a in state]
    orc.step_f32([red], s, *want, lo=0, hi=valid)
    got = _run_gpu(spec, hp, state, [red], "f32", n, valid)
    assert assert_state_parity(got, want, "f32 gradient, f16 parameters") == 0


def test_f16_special_values():
    """Overflow of the parameter image to infinity, subnormal images, infinite and NaN
    gradients, the largest finite binary16 gradient summed N times."""
    n, N = TILE + 64, 2
    _say("binary16 special values n=%d" % n)
    spec = ps.ps_spec_preset("zero3", N, 0, n * N)
    grads, state, s, hp = _f16_case(n, N, 203)
    g0, g1 = grads
    g0[:6] = [np.inf, -np.inf, np.nan, 65504.0, 6e-8, -0.0]
    g1[:6] = [1.0, 1.0, 1.0, 65504.0, 6e-8, -0.0]
    g0[6:10] = np.inf
    g1[6:10] = -np.inf                                             # inf - inf
    th = state[0]
    th[16:26] = [65519.9, 65530.0, -7e4, 3e38, 6.0e-8, 2.98e-8, 2.99e-8, -1e-9, 6.1e-5, 0.0]
    for a in (g0, g1, state[1], state[2]):
        a[16:26] = 0                                               # there only the decay acts
    want = [a.copy() for a in state]
    orc.step_f32(grads, s, *want)
    got = _run_gpu(spec, hp, state, grads, "f16", n)
    assert_state_parity(got, want, "f16 specials")
    nan = np.isnan(want[0])
    assert nan[2] and nan[6:10].all()
    gp, wp = got[3].view(np.uint16), want[3].view(np.uint16)
    assert ((gp[nan] & 0x7fff) == 0x7e00).all()                    # canonical quiet NaN
    assert np.array_equal(gp[~nan], wp[~nan])
    assert got[3][16] == np.float16(65504.0) and np.isinf(got[3][17:20]).all()     # 65520 and up: infinity
    units = got[3][20:23].view(np.uint16)                    # subnormal images: units of 2^-24
    assert list(units) == [1, 0, 1]                          # 6.0e-8 -> 1; just under / over half a unit
    assert got[3][23].view(np.uint16) == 0x8000                                     # underflow keeps the sign


def test_f16_cast_exhaustive_over_all_binary32_patterns():
    """As for bf16: with lr = 0, zero moments and a zero gradient every finite master value
    but -0 passes unchanged, so the binary16 image covers the cast of all 2^32 patterns;
    compared bit for bit with the library's float32 -> float16 conversion."""
    chunk = 1 << 28
    _say("exhaustive binary16 cast: 2^32 master patterns in %d launches" % ((1 << 32) // chunk))
    spec = ps.ps_spec_preset("zero3", 4, 0, chunk * 4)
    _, hp = hp_of(None, 1, lr=0.0, weight_decay=0.0, grad_scale=1.0)
    bits = torch.empty(chunk, dtype=torch.int32, device="cuda")
    th = bits.view(torch.float32)
    m = torch.zeros(chunk, dtype=torch.float32, device="cuda")
    v = torch.zeros_like(m)
    g = torch.zeros_like(m)
    out = torch.empty(chunk, dtype=torch.float16, device="cuda")
    ramp = torch.arange(chunk, dtype=torch.int64, device="cuda")
    for lo in range(0, 1 << 32, chunk):
        before = ((ramp + lo) & 0xffffffff)
        bits.copy_(torch.where(before >= (1 << 31), before - (1 << 32), before).to(torch.int32))
        before = bits.clone()
        out.fill_(3.0)
        ps.ps_step_update(spec, hp, shard_of(th, m, v, out, chunk), grads_of([g], "f32"), 0, chunk,
                          stream_handle())
        torch.cuda.synchronize()
        finite = (before & 0x7fffffff) < 0x7f800000
        keep = finite & (before != -(1 << 31))
        assert torch.equal(bits[keep], before[keep]), hex(lo)
        nan = torch.isnan(th)
        lib = th.to(torch.float16).view(torch.int16)
        o16 = out.view(torch.int16)
        assert torch.equal(o16[~nan], lib[~nan]), hex(lo)
        assert bool(((o16[nan] & 0x7fff) == 0x7e00).all()), hex(lo)


def test_f16_reduce_accumulate_and_difference():
    """The other entry points that read gradients, with binary16 contributions: reduce +
    sum of squares, accumulation over micro-batches, and the relative-difference scan."""
    N, n = 4, 9 * TILE + 777
    valid = n - 11
    _say("binary16 reduce / accumulate / difference n=%d N=%d" % (n, N))
    spec = ps.ps_spec_preset("zero3", N, 0, n * N)
    grads, _, s, _ = _f16_case(n, N, 207)
    gs = 1.0 / (N * LOSS_SCALE)
    mean, ss = orc.mean_sumsq(grads, gs, 0, valid)
    red, ss_gpu = _reduce_gpu(spec, grads, "f16", n, valid, gs=gs)
    assert np.array_equal(red[:valid].view(np.uint32), mean[:valid].view(np.uint32))
    assert np.isnan(red[valid:]).all() and abs(ss_gpu - ss) <= 1e-12 * ss
    acc_want = np.full(n, np.float32(3.0))
    acc_dev = dev(acc_want.copy())
    for j in range(3):
        gj = [gen.gradient(n, 209, j, r, "f16", std=1.0) for r in range(N)]
        orc.accumulate(gj, acc_want, overwrite=(j == 0), lo=0, hi=valid)
        ps.ps_step_accumulate(spec, grads_of([dev(g) for g in gj], "f16"), acc_dev.data_ptr(), j == 0,
                              0, n, valid, stream_handle())
        torch.cuda.synchronize()
    assert np.array_equal(host(acc_dev).view(np.uint32), acc_want.view(np.uint32))
    a, b = grads[0], grads[1]
    want_d, want_a = orc.diff_sumsq(a, b)
    ws = torch.empty(ps.ps_verify_workspace_bytes(n * 2), dtype=torch.uint8, device="cuda")
    out2 = torch.zeros(2, dtype=torch.float64, device="cuda")
    da, db = dev(a), dev(b)
    ps.ps_verify_diff_sumsq(da.data_ptr(), db.data_ptr(), ps.PS_F16, n, out2.data_ptr(), 0,
                            ws.data_ptr(), ws.numel(), stream_handle())
    torch.cuda.synchronize()
    sd, sa = [float(x) for x in out2.tolist()]
    assert abs(sd - want_d) <= 1e-12 * want_d and abs(sa - want_a) <= 1e-12 * want_a


def test_f16_bucket_pipeline_and_offload():
    """The two pipelines with binary16 gradients and parameters."""
    N, bucket = 4, TILE
    n = 4 * bucket + 520
    valid = n - 7
    _say("binary16 through the bucket pipeline and the offload path n=%d" % n)
    spec = ps.ps_spec_preset("zero3", N, 3, n * N)
    grads, state, s, hp = _f16_case(n, N, 211)
    want = [a.copy() for a in state]
    orc.step_f32(grads, s, *want, lo=0, hi=valid)
    # bucket loop, every engine that runs on the device: the source holds every bucket
    src = [dev(g) for g in grads]
    n_src = -(-n // 512) * 512
    src = [torch.cat([x, torch.zeros(n_src - n, dtype=x.dtype, device="cuda")]) for x in src]
    for engine in (ps.PS_COPY_KERNEL, ps.PS_COPY_NONE, ps.PS_COPY_REDUCE):
        th, m, v, p = [dev(a) for a in state]
        staging = [torch.zeros(N * bucket * 2, dtype=torch.uint8, device="cuda") for _ in range(2)]
        copy, comp = torch.cuda.Stream(), torch.cuda.Stream()
        torch.cuda.synchronize()
        plan = ps.ps_bucket_plan_t()
        arr = (C.c_void_p * N)(*[x.data_ptr() for x in src])
        plan.source = C.cast(arr, C.POINTER(C.c_void_p))
        plan.n_contrib, plan.dtype, plan.bucket_elems, plan.source_elems = N, ps.PS_F16, bucket, n_src
        plan.staging[0], plan.staging[1] = staging[0].data_ptr(), staging[1].data_ptr()
        plan.copy_stream, plan.compute_stream = copy.cuda_stream, comp.cuda_stream
        plan.copy_engine, plan.schedule = engine, ps.PS_SCHED_AUTO
        ps.ps_step_update_bucketed(spec, hp, shard_of(th, m, v, p, n, valid), plan)
        torch.cuda.synchronize()
        assert assert_state_parity([host(x) for x in (th, m, v, p)], want, "f16 bucketed, engine %d" % engine) == 0
    # offload: state and FP16 parameters in pinned host memory
    spec_o = ps.ps_spec_preset("zero_offload", N, 3, n * N)
    pinned = [torch.from_numpy(a.copy()).pin_memory() for a in state]
    slots = [torch.zeros(14 * bucket, dtype=torch.uint8, device="cuda") for _ in range(3)]
    s1, s2, s3 = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    op = ps.ps_offload_plan_t()
    op.host_master, op.host_m, op.host_v, op.host_param_out = [t.data_ptr() for t in pinned]
    op.len, op.valid_len, op.bucket_elems, op.n_slots, op.param_dtype = n, valid, bucket, 3, ps.PS_F16
    for k, t in enumerate(slots):
        op.slot[k] = t.data_ptr()
    op.h2d_stream, op.compute_stream, op.d2h_stream = s1.cuda_stream, s2.cuda_stream, s3.cuda_stream
    ps.ps_step_update_offloaded(spec_o, hp, op, grads_of([dev(g) for g in grads], "f16"))
    torch.cuda.synchronize()
    assert assert_state_parity([t.numpy() for t in pinned], want, "f16 offload") == 0


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_widening_of_all_65536_patterns(dtype):
    """Every 16-bit pattern through the kernels' widening: one replicated contribution, scale
    1, so the reduced output is the widened value itself (subnormals kept, infinities kept)."""
    n = 65536
    _say("widening of all %d %s patterns" % (n, dtype))
    bits = np.arange(n, dtype=np.uint16)
    g = bits.view(np.float16).copy() if dtype == "f16" else bits
    want = g.astype(np.float32) if dtype == "f16" else (bits.astype(np.uint32) << 16).view(np.float32)
    spec = ps.ps_spec_preset("dp", 4, 0, n)
    red, _ = _reduce_gpu(spec, [g], dtype, n, n, gs=1.0)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(red), nan)
    assert np.array_equal(red[~nan].view(np.uint32), want[~nan].view(np.uint32))
    assert np.array_equal([orc.widen_f16(int(b)) if dtype == "f16" else orc.widen_bf16(int(b)) for b in bits[~nan][::97]],
                          want[~nan][::97])


def test_composed_tp_x_dp_step_equals_the_unsharded_update():
    """Composition (Definition 5, Theorem 6): tensor parallelism of degree T inside, ZeRO-2
    of degree D across.  Device d = (TP rank, DP rank) per ps_compose_index holds the
    1/T share of its TP rank and, of that share, the ZeRO shard of its DP rank; its step
    is the outer specification's step on the share (the convention of ps_compose_cost),
    reducing the D contributions of its data-parallel group.  All T*D device results put
    together are the unsharded update of the whole model with N = D."""
    T, D = 2, 3
    psi = T * D * (TILE + 264)
    share, n = psi // T, psi // (T * D)
    _say("TP(%d) x ZeRO-2(%d): psi=%d, share=%d, shard=%d" % (T, D, psi, share, n))
    grads = [gen.gradient(psi, 301, 0, d, "bf16") for d in range(D)]         # one per DP replica
    full = [gen.master(psi, 301), *gen.moments(psi, 301, True), np.zeros(psi, np.uint16)]
    hpd, hp = hp_of(None, 3)
    want = [a.copy() for a in full]
    orc.step_f32(grads, orc.derive_scalars(t=3, n_devices=D, **hpd), *want)
    got = [np.zeros_like(a) for a in full]
    cost = None
    for dev_id in range(T * D):
        tp_group, tp_rank, dp_group, dp_rank = ps.ps_compose_index(T, D, dev_id)
        assert dp_group == tp_rank and dp_rank == tp_group
        spec = ps.ps_spec_preset("zero2", D, dp_rank, share)                 # outer spec on the share
        c = ps.ps_cost_eval(spec)
        cc = ps.ps_compose_cost(ps.ps_spec_preset("zero2", D, dp_rank, psi), T)
        assert (c.shard_len, c.shard_offset, c.peak_total) == (cc.shard_len, cc.shard_offset, cc.peak_total)
        lo = tp_rank * share + c.shard_offset                                # where this shard sits in the model
        sl = slice(lo, lo + n)
        th, m, v = [dev(np.ascontiguousarray(a[sl])) for a in full[:3]]
        p_share = dev(np.zeros(share, np.uint16))                            # pi_Theta = R inside the DP group
        gd = [dev(np.ascontiguousarray(g[sl])) for g in grads]
        ps.ps_step_update(spec, hp, shard_of(th, m, v, p_share, n), grads_of(gd, "bf16"), 0, n,
                          stream_handle())
        torch.cuda.synchronize()
        for k, t_ in enumerate((th, m, v)):
            got[k][sl] = host(t_)
        got[3][sl] = host(p_share)[c.shard_offset:c.shard_offset + n]
    assert assert_state_parity(got, want, "TP x DP") == 0
    assert np.array_equal(got[3], want[3])

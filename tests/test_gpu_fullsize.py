"""Full-size GPU parity in the launch configurations bench.py times: the 7B ZeRO-2
shard (one launch), the 70B ZeRO-3 shard (33 buckets through the two-stream
pipeline) and the ragged 13B shard with clipping (two phases).  Inputs are
generated on the device; sampled slices are copied to the host *before* the step
and the oracle is run on exactly those slices.  Whole-shard properties that hold
at any size are checked on the device with library primitives."""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_2601_02311_amd as ps
from oracle import step as orc
from synth import WORKLOADS
from synth import device as dgen

from gpu_util import assert_state_parity, host, shard_of, stream_handle

pytestmark = pytest.mark.gpu

SLICE = 1 << 20


def _say(msg):
    print("[case] " + msg, flush=True)


def _need(gb):
    free, _ = torch.cuda.mem_get_info()
    if free < gb * 1e9:
        pytest.skip("needs %.0f GB of free device memory" % gb)


def _slices(n, extra=()):
    """Head, an odd-offset middle, the tail, plus any extra (lo, hi) ranges."""
    mid = (n // 2) // 8 * 8 + 8
    out = [(0, SLICE), (mid, mid + SLICE + 24), (n - SLICE - 8, n)]
    out += [(max(0, lo), min(n, hi)) for lo, hi in extra]
    return out


def _take(t, lo, hi):
    return host(t[lo:hi].clone())


def _hp(w, t, **kw):
    d = dict(lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, weight_decay=w.weight_decay)
    return d, ps.ps_adamw_t(w.lr, w.beta1, w.beta2, w.eps, w.weight_decay, t,
                            kw.get("grad_scale", 0.0), kw.get("clip_coef", 0.0))


def _whole_shard_properties(master, m, v, out_slice, valid):
    """bf16 image == RNE cast of the new master weight (library conversion), v' >= 0,
    everything finite -- over every element, on the device."""
    step = 1 << 28
    for lo in range(0, valid, step):
        hi = min(lo + step, valid)
        assert torch.equal(master[lo:hi].to(torch.bfloat16).view(torch.int16),
                           out_slice[lo:hi].view(torch.int16))
        assert bool((v[lo:hi] >= 0).all())
        assert bool(torch.isfinite(master[lo:hi]).all()) and bool(torch.isfinite(m[lo:hi]).all())


def test_7b_zero2_full_shard_sampled():
    w = WORKLOADS["7b_zero2"]
    _need(45)
    n, N, t = w.shard_len, w.n_devices, w.first_step
    _say("7b_zero2 full shard n=%d, one launch, sampled slices" % n)
    spec = ps.ps_spec_preset(w.strategy, N, w.shard_index, w.psi)
    cost = ps.ps_cost_eval(spec)
    master, m, v = dgen.workload_state(w)
    grads = dgen.workload_gradients(w, t)
    out = torch.zeros(cost.psi_padded, dtype=torch.bfloat16, device="cuda")   # replicated Theta
    sl = _slices(n)
    before = [([_take(x, lo, hi) for x in (master, m, v)], [_take(g, lo, hi) for g in grads])
              for lo, hi in sl]
    hpd, hp = _hp(w, t)
    ps.ps_step_update(spec, hp, shard_of(master, m, v, out, n), ps.make_grads(
        [g.data_ptr() for g in grads], ps.PS_BF16), 0, n, stream_handle())
    torch.cuda.synchronize()
    s = orc.derive_scalars(t=t, n_devices=N, **hpd)
    off = cost.shard_offset
    for (lo, hi), (st, gr) in zip(sl, before):
        want = [a.copy() for a in st] + [np.zeros(hi - lo, np.uint16)]
        orc.step_f32(gr, s, *want)
        got = [_take(x, lo, hi) for x in (master, m, v)] + [_take(out, off + lo, off + hi)]
        assert assert_state_parity(got, want, "7b [%d,%d)" % (lo, hi)) == 0
    _whole_shard_properties(master, m, v, out[off:off + n], n)
    assert not bool(out[off + n:off + n + SLICE].view(torch.int16).any())   # next shard's slice untouched
    del master, m, v, grads, out
    torch.cuda.empty_cache()


def test_70b_zero3_bucketed_full_shard_sampled():
    w = WORKLOADS["70b_zero3"]
    _need(140)
    n, N, t, B = w.shard_len, w.n_devices, w.first_step, w.bucket_elems
    pool_elems = 1 << 21
    n_b = -(-n // B)
    _say("70b_zero3 full shard n=%d, %d buckets of %d, pool %d, sampled slices" % (n, n_b, B, pool_elems))
    spec = ps.ps_spec_preset(w.strategy, N, w.shard_index, w.psi)
    master, m, v = dgen.workload_state(w)
    out = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    pool = [dgen.fill_gradient_(torch.empty(pool_elems, dtype=torch.bfloat16, device="cuda"),
                                w.seed, t, r, w.grad_std) for r in range(N)]
    pool_np = [host(p) for p in pool]
    staging = [torch.empty(N * B, dtype=torch.bfloat16, device="cuda") for _ in range(2)]
    copy, comp = torch.cuda.Stream(), torch.cuda.Stream()
    # buckets 0, 16 and the short last one, plus ranges that straddle bucket edges
    sl = _slices(n, extra=[(16 * B - 4096, 16 * B + 4096), ((n_b - 1) * B - 4096, (n_b - 1) * B + 4096),
                           (16 * B + 12345 * 8, 16 * B + 12345 * 8 + SLICE)])
    before = [[_take(x, lo, hi) for x in (master, m, v)] for lo, hi in sl]
    torch.cuda.synchronize()
    plan = ps.ps_bucket_plan_t()
    arr = (C.c_void_p * N)(*[p.data_ptr() for p in pool])
    plan.source = C.cast(arr, C.POINTER(C.c_void_p))
    plan.n_contrib, plan.dtype, plan.bucket_elems, plan.source_elems = N, ps.PS_BF16, B, pool_elems
    plan.staging[0], plan.staging[1] = staging[0].data_ptr(), staging[1].data_ptr()
    plan.copy_stream, plan.compute_stream = copy.cuda_stream, comp.cuda_stream
    plan.copy_engine, plan.schedule = ps.PS_COPY_KERNEL, ps.PS_SCHED_AUTO
    hpd, hp = _hp(w, t)
    ps.ps_step_update_bucketed(spec, hp, shard_of(master, m, v, out, n), plan)
    torch.cuda.synchronize()
    s = orc.derive_scalars(t=t, n_devices=N, **hpd)
    for (lo, hi), st in zip(sl, before):
        idx = np.arange(lo, hi) % pool_elems             # element e reads source[e % source_elems]
        gr = [np.ascontiguousarray(p[idx]) for p in pool_np]
        want = [a.copy() for a in st] + [np.zeros(hi - lo, np.uint16)]
        orc.step_f32(gr, s, *want)
        got = [_take(x, lo, hi) for x in (master, m, v, out)]
        assert assert_state_parity(got, want, "70b [%d,%d)" % (lo, hi)) == 0
    _whole_shard_properties(master, m, v, out, n)
    del master, m, v, out, pool, staging
    torch.cuda.empty_cache()


def test_13b_clip_ragged_full_shard_sampled():
    w = WORKLOADS["13b_clip"]
    _need(100)
    N, t = w.n_devices, w.first_step
    psi = w.extra["psi_ragged"]                          # same buffers, last shard owns a pad of 1001
    spec = ps.ps_spec_preset(w.strategy, N, w.shard_index, psi, align_elems=w.align_elems)
    cost = ps.ps_cost_eval(spec)
    n, valid = cost.shard_len, cost.valid_len
    assert n == w.shard_len and valid == n - 1001
    _say("13b_clip ragged full shard n=%d valid=%d N=%d fp32, two phases" % (n, valid, N))
    master, m, v = dgen.workload_state(w)
    grads = dgen.workload_gradients(w, t)
    out = torch.full((n,), -1.0, dtype=torch.bfloat16, device="cuda")
    red = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
    ssd = torch.zeros(1, dtype=torch.float64, device="cuda")
    ws = torch.empty(ps.ps_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    sl = _slices(valid, extra=[(n - SLICE, n)])          # the last range includes the pad
    before = [([_take(x, lo, hi) for x in (master, m, v, out)], [_take(g, lo, hi) for g in grads])
              for lo, hi in sl]
    g = ps.make_grads([x.data_ptr() for x in grads], ps.PS_F32)
    ps.ps_step_reduce_sumsq(spec, g, 0.0, red.data_ptr(), ssd.data_ptr(), 0, ws.data_ptr(),
                            ws.numel(), 0, n, valid, stream_handle())
    ss_gpu = float(ssd.item())
    # the same sum with library primitives in binary64 on the device (a definition, not the HIP path)
    gs = np.float32(1.0 / N)
    ss_ref = 0.0
    step = 1 << 27
    for lo in range(0, valid, step):
        hi = min(lo + step, valid)
        acc = grads[0][lo:hi].clone()
        for r in range(1, N):
            acc += grads[r][lo:hi]
        acc *= float(gs)
        assert torch.equal(acc, red[lo:hi])                                  # bit-exact mean, every element
        ss_ref += float(acc.double().square_().sum().item())
    assert abs(ss_gpu - ss_ref) <= 1e-9 * ss_ref
    assert bool(torch.isnan(red[valid:]).all())                               # pad never written
    again = torch.zeros(1, dtype=torch.float64, device="cuda")
    ps.ps_step_reduce_sumsq(spec, g, 0.0, 0, again.data_ptr(), 0, ws.data_ptr(), ws.numel(), 0, n,
                            valid, stream_handle())
    assert float(again.item()) == ss_gpu                                      # run-to-run identical
    # the oracle's coefficient from the independent sum; both sides use this one value
    coef = orc.clip_coef(ss_ref, 5 * ss_ref, w.max_grad_norm)
    assert ps.ps_clip_coef(ss_ref, 5 * ss_ref, w.max_grad_norm) == coef
    hpd, hp = _hp(w, t, grad_scale=1.0, clip_coef=coef)
    ps.ps_step_update(spec, hp, shard_of(master, m, v, out, n, valid),
                      ps.make_grads([red.data_ptr()], ps.PS_F32), 0, n, stream_handle())
    torch.cuda.synchronize()
    s = orc.derive_scalars(t=t, n_devices=N, clip_coef=coef, **hpd)
    for (lo, hi), (st, gr) in zip(sl, before):
        want = [a.copy() for a in st]
        orc.step_f32(gr, s, *want, lo=0, hi=min(hi, valid) - lo)              # oracle stops at valid
        got = [_take(x, lo, hi) for x in (master, m, v, out)]
        assert assert_state_parity(got, want, "13b [%d,%d)" % (lo, hi)) == 0
        assert np.array_equal(got[3], want[3])
        if hi > valid:                                                        # pad bytes untouched
            for a, b in zip(got, st):
                assert np.array_equal(a[valid - lo:].view(np.uint8), b[valid - lo:].view(np.uint8))
    _whole_shard_properties(master, m, v, out, valid)
    del master, m, v, out, red, grads, ws
    torch.cuda.empty_cache()


def test_single_launch_beyond_2_32_elements():
    """Maximum size in one launch: the whole 70B shard (8.75e9 elements, 34 million
    workgroups) updated from one pre-reduced fp32 gradient; element indices pass 2^32
    and byte offsets pass 2^35.  Sampled slices straddle 2^31, 2^32 and 2^33."""
    w = WORKLOADS["70b_zero3"]
    _need(165)
    n, N, t = w.shard_len, w.n_devices, w.first_step
    _say("single launch over n=%d elements (fp32 pre-reduced gradient)" % n)
    spec = ps.ps_spec_preset(w.strategy, N, w.shard_index, w.psi)
    master, m, v = dgen.workload_state(w)
    g = dgen.fill_normal_(torch.empty(n, dtype=torch.float32, device="cuda"), 1e-4, w.seed, 9)
    out = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    sl = _slices(n, extra=[((1 << 31) - 4096, (1 << 31) + 4096), ((1 << 32) - 4096, (1 << 32) + 4096),
                           ((1 << 33) - 4096, (1 << 33) + 4096)])
    before = [([_take(x, lo, hi) for x in (master, m, v)], [_take(g, lo, hi)]) for lo, hi in sl]
    hpd, hp = _hp(w, t, grad_scale=1.0)
    ps.ps_step_update(spec, hp, shard_of(master, m, v, out, n),
                      ps.make_grads([g.data_ptr()], ps.PS_F32), 0, n, stream_handle())
    torch.cuda.synchronize()
    s = orc.derive_scalars(t=t, n_devices=N, grad_scale=1.0, **hpd)
    for (lo, hi), (st, gr) in zip(sl, before):
        want = [a.copy() for a in st] + [np.zeros(hi - lo, np.uint16)]
        orc.step_f32(gr, s, *want)
        got = [_take(x, lo, hi) for x in (master, m, v, out)]
        assert assert_state_parity(got, want, "big [%d,%d)" % (lo, hi)) == 0
    _whole_shard_properties(master, m, v, out, n)
    del master, m, v, g, out
    torch.cuda.empty_cache()

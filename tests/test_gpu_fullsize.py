"""Full-size GPU parity in the launch configurations bench.py times: the 7B ZeRO-2
shard (one launch), the 70B ZeRO-3 shard (33 buckets through the two-stream
pipeline), the ragged 13B shard with clipping (two phases), and the ZeRO-1,
accumulation, verification and offload rows on the 7B shard.  Inputs are
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
    """16-bit image == RNE cast of the new master weight (library conversion), v' >= 0,
    everything finite -- over every element, on the device."""
    step = 1 << 28
    for lo in range(0, valid, step):
        hi = min(lo + step, valid)
        assert torch.equal(master[lo:hi].to(out_slice.dtype).view(torch.int16),
                           out_slice[lo:hi].view(torch.int16))
        assert bool((v[lo:hi] >= 0).all())
        assert bool(torch.isfinite(master[lo:hi]).all()) and bool(torch.isfinite(m[lo:hi]).all())


@pytest.mark.parametrize("name", ["7b_zero2", "7b_zero2_f16"])
def test_7b_zero2_full_shard_sampled(name):
    """bf16 gradients and parameters, and the same shard in binary16 with a loss scale."""
    w = WORKLOADS[name]
    _need(45)
    n, N, t = w.shard_len, w.n_devices, w.first_step
    f16 = w.param_dtype == "f16"
    _say("%s full shard n=%d, one launch, sampled slices" % (name, n))
    spec = ps.ps_spec_preset(w.strategy, N, w.shard_index, w.psi)
    cost = ps.ps_cost_eval(spec)
    master, m, v = dgen.workload_state(w)
    grads = dgen.workload_gradients(w, t)
    out = torch.zeros(cost.psi_padded, dtype=torch.float16 if f16 else torch.bfloat16,
                      device="cuda")                                            # replicated Theta
    sl = _slices(n)
    before = [([_take(x, lo, hi) for x in (master, m, v)], [_take(g, lo, hi) for g in grads])
              for lo, hi in sl]
    gs = 1.0 / (N * w.loss_scale) if w.loss_scale != 1.0 else 0.0
    hpd, hp = _hp(w, t, grad_scale=gs)
    ps.ps_step_update(spec, hp, shard_of(master, m, v, out, n), ps.make_grads(
        [g.data_ptr() for g in grads], ps.PS_F16 if f16 else ps.PS_BF16), 0, n, stream_handle())
    torch.cuda.synchronize()
    s = orc.derive_scalars(t=t, n_devices=N, grad_scale=gs, **hpd)
    off = cost.shard_offset
    for (lo, hi), (st, gr) in zip(sl, before):
        want = [a.copy() for a in st] + [np.zeros(hi - lo, np.float16 if f16 else np.uint16)]
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


# ---- rows beyond the base path, at the sizes bench.py times them ----

def test_7b_zero1_full_shard_sampled():
    """ZeRO-1 row: one all-reduced, replicated bf16 gradient of psi elements; the library
    reads and writes slice i.  Run for the shard bench.py uses and for one with a large
    offset, on the same buffers."""
    w = WORKLOADS["7b_zero1"]
    _need(45)
    N, t = w.n_devices, w.first_step
    master, m, v = dgen.workload_state(w)
    n = w.shard_len
    grad = dgen.fill_gradient_(torch.empty(w.psi, dtype=torch.bfloat16, device="cuda"),
                               w.seed, t, 0, w.grad_std)
    out = torch.zeros(w.psi, dtype=torch.bfloat16, device="cuda")
    for i in (w.shard_index, 5):
        spec = ps.ps_spec_preset(w.strategy, N, i, w.psi)
        cost = ps.ps_cost_eval(spec)
        assert cost.shard_len == n and cost.psi_padded == w.psi
        off = cost.shard_offset
        _say("7b_zero1 shard %d: n=%d at offset %d of the replicated gradient" % (i, n, off))
        sl = _slices(n)
        before = [([_take(x, lo, hi) for x in (master, m, v)], [_take(grad, off + lo, off + hi)])
                  for lo, hi in sl]
        out.zero_()
        hpd, hp = _hp(w, t)
        ps.ps_step_update(spec, hp, shard_of(master, m, v, out, n),
                          ps.make_grads([grad.data_ptr()], ps.PS_BF16), 0, n, stream_handle())
        torch.cuda.synchronize()
        s = orc.derive_scalars(t=t, n_devices=N, **hpd)          # grad_scale 0: 1/N, the all-reduce sums
        for (lo, hi), (st, gr) in zip(sl, before):
            want = [a.copy() for a in st] + [np.zeros(hi - lo, np.uint16)]
            orc.step_f32(gr, s, *want)
            got = [_take(x, lo, hi) for x in (master, m, v)] + [_take(out, off + lo, off + hi)]
            assert assert_state_parity(got, want, "zero1 shard %d [%d,%d)" % (i, lo, hi)) == 0
        _whole_shard_properties(master, m, v, out[off:off + n], n)
        if off:                                                    # neighbours' slices untouched
            assert not bool(out[off - SLICE:off].view(torch.int16).any())
        if off + n < w.psi:
            assert not bool(out[off + n:off + n + SLICE].view(torch.int16).any())
    del master, m, v, grad, out
    torch.cuda.empty_cache()


def test_7b_accum4_full_shard_sampled():
    """Gradient accumulation row: four micro-batches (fresh contributions each) into the
    FP32 accumulator, then one update with grad_scale = 1/(N k)."""
    w = WORKLOADS["7b_accum4"]
    _need(45)
    n, N, t, k = w.shard_len, w.n_devices, w.first_step, w.micro_batches
    _say("7b_accum4 full shard n=%d, %d micro-batches, sampled slices" % (n, k))
    spec = ps.ps_spec_preset(w.strategy, N, w.shard_index, w.psi)
    cost = ps.ps_cost_eval(spec)
    master, m, v = dgen.workload_state(w)
    out = torch.zeros(n, dtype=torch.bfloat16, device="cuda")      # this shard's slice only
    accum = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
    sl = _slices(n)
    acc_want = [np.full(hi - lo, np.float32(np.nan)) for lo, hi in sl]
    grads = None
    for j in range(k):
        del grads
        grads = dgen.workload_gradients(w, t * 16 + j)             # a different stream per micro-batch
        for (lo, hi), a in zip(sl, acc_want):
            orc.accumulate([_take(g, lo, hi) for g in grads], a, overwrite=(j == 0))
        ps.ps_step_accumulate(spec, ps.make_grads([g.data_ptr() for g in grads], ps.PS_BF16),
                              accum.data_ptr(), j == 0, 0, n, n, stream_handle())
        torch.cuda.synchronize()
    for (lo, hi), a in zip(sl, acc_want):
        assert np.array_equal(_take(accum, lo, hi).view(np.uint32), a.view(np.uint32))
    assert bool(torch.isfinite(accum).all())                       # every element was overwritten first
    before = [[_take(x, lo, hi) for x in (master, m, v)] for lo, hi in sl]
    scale = 1.0 / (N * k)
    hpd, hp = _hp(w, t, grad_scale=scale)
    assert cost.shard_offset == 0          # shard 0: its slice of the replicated parameters starts the buffer
    ps.ps_step_update(spec, hp, shard_of(master, m, v, out, n),
                      ps.make_grads([accum.data_ptr()], ps.PS_F32), 0, n, stream_handle())
    torch.cuda.synchronize()
    s = orc.derive_scalars(t=t, n_devices=N, grad_scale=scale, **hpd)
    for (lo, hi), st, a in zip(sl, before, acc_want):
        want = [x.copy() for x in st] + [np.zeros(hi - lo, np.uint16)]
        orc.step_f32([a], s, *want)
        got = [_take(x, lo, hi) for x in (master, m, v, out)]
        assert assert_state_parity(got, want, "accum [%d,%d)" % (lo, hi)) == 0
    _whole_shard_properties(master, m, v, out, n)
    del master, m, v, out, accum, grads
    torch.cuda.empty_cache()


def test_7b_verify_scans_whole_buffers_against_the_oracle():
    """Verification row at the size bench.py times: the relative-difference scan over two
    bf16 gradient copies of the 7B shard and the checksum of its FP32 master shard, each
    against the oracle run over the WHOLE buffer on the host; pieces add up."""
    w = WORKLOADS["7b_zero2"]
    _need(12)
    n = w.shard_len
    _say("7b verify: diff scan over 2 x %d bf16, checksum over %d fp32, whole-buffer oracle" % (n, n))
    a = dgen.fill_gradient_(torch.empty(n, dtype=torch.bfloat16, device="cuda"), w.seed, 1, 0, w.grad_std)
    b = a.clone()
    b[12345] += 1.0
    b[n - 7] -= 0.5
    master, _, _ = dgen.workload_state(w)
    ws = torch.empty(ps.ps_verify_workspace_bytes(n * 4), dtype=torch.uint8, device="cuda")
    out2 = torch.zeros(2, dtype=torch.float64, device="cuda")
    outc = torch.zeros(1, dtype=torch.int64, device="cuda")
    st = stream_handle()
    ps.ps_verify_diff_sumsq(a.data_ptr(), b.data_ptr(), ps.PS_BF16, n, out2.data_ptr(), 0,
                            ws.data_ptr(), ws.numel(), st)
    ps.ps_verify_checksum(master.data_ptr(), n * 4, 0, outc.data_ptr(), 0, ws.data_ptr(), ws.numel(), st)
    torch.cuda.synchronize()
    sd, sa = [float(x) for x in out2.tolist()]
    whole = int(outc.item()) & 0xffffffffffffffff
    # in three pieces with running totals: same checksum exactly, same sums to rounding
    cuts = [0, (n // 3) // 8 * 8, (2 * n // 3) // 8 * 8 + 8, n]
    for j in range(3):
        lo, hi = cuts[j], cuts[j + 1]
        ps.ps_verify_diff_sumsq(a.data_ptr() + 2 * lo, b.data_ptr() + 2 * lo, ps.PS_BF16, hi - lo,
                                out2.data_ptr(), j > 0, ws.data_ptr(), ws.numel(), st)
        ps.ps_verify_checksum(master.data_ptr() + 4 * lo, (hi - lo) * 4, lo // 2, outc.data_ptr(),
                              j > 0, ws.data_ptr(), ws.numel(), st)
    torch.cuda.synchronize()
    assert int(outc.item()) & 0xffffffffffffffff == whole
    pd, pa = [float(x) for x in out2.tolist()]
    assert abs(pd - sd) <= 1e-12 * sd and abs(pa - sa) <= 1e-12 * sa
    # the oracle adds its 8.4e8 exact products one after another: its own rounding error is
    # bounded by n * 2^-53 relative (all terms >= 0), and that is the bar against it
    want_d, want_a = orc.diff_sumsq(host(a), host(b))
    bound = n * 2.0 ** -53
    assert abs(sd - want_d) <= bound * want_d and abs(sa - want_a) <= bound * want_a
    # against a pairwise binary64 reduction with library primitives the trees agree far closer
    lib_d = lib_a = 0.0
    step = 1 << 27
    for lo in range(0, n, step):
        x, y = a[lo:lo + step].double(), b[lo:lo + step].double()
        lib_a += float(x.square().sum().item())
        lib_d += float((x - y).square_().sum().item())
    assert abs(sd - lib_d) <= 1e-12 * lib_d and abs(sa - lib_a) <= 1e-12 * lib_a
    assert orc.checksum(host(master)) == whole
    del a, b, master, ws
    torch.cuda.empty_cache()


def test_7b_offload_full_shard_sampled():
    """ZeRO-Offload row at bench.py's shape: master/m/v and the bf16 parameters of the 7B
    shard in pinned host memory, streamed through three device slots of 2^24 elements."""
    w = WORKLOADS["7b_offload"]
    _need(20)
    n, N, t, B = w.shard_len, w.n_devices, w.first_step, w.bucket_elems
    _say("7b_offload full shard n=%d, buckets of %d through 3 slots, sampled slices" % (n, B))
    spec = ps.ps_spec_preset(w.strategy, N, w.shard_index, w.psi)
    pinned = [x.cpu().pin_memory() for x in dgen.workload_state(w)]
    pinned.append(torch.zeros(n, dtype=torch.bfloat16).pin_memory())
    torch.cuda.empty_cache()
    grads = dgen.workload_gradients(w, t)
    n_b = -(-n // B)
    sl = _slices(n, extra=[(B - 4096, B + 4096), ((n_b - 1) * B - 4096, (n_b - 1) * B + 4096)])
    before = [([host(x[lo:hi].clone()) for x in pinned[:3]], [_take(g, lo, hi) for g in grads])
              for lo, hi in sl]
    slots = [torch.empty(14 * B, dtype=torch.uint8, device="cuda") for _ in range(3)]
    s1, s2, s3 = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    plan = ps.ps_offload_plan_t()
    plan.host_master, plan.host_m, plan.host_v, plan.host_param_out = [x.data_ptr() for x in pinned]
    plan.len, plan.valid_len, plan.bucket_elems, plan.n_slots = n, n, B, 3
    for j, x in enumerate(slots):
        plan.slot[j] = x.data_ptr()
    plan.h2d_stream, plan.compute_stream, plan.d2h_stream = s1.cuda_stream, s2.cuda_stream, s3.cuda_stream
    hpd, hp = _hp(w, t)
    ps.ps_step_update_offloaded(spec, hp, plan, ps.make_grads([g.data_ptr() for g in grads], ps.PS_BF16))
    torch.cuda.synchronize()
    s = orc.derive_scalars(t=t, n_devices=N, **hpd)
    for (lo, hi), (st, gr) in zip(sl, before):
        want = [x.copy() for x in st] + [np.zeros(hi - lo, np.uint16)]
        orc.step_f32(gr, s, *want)
        got = [host(x[lo:hi].clone()) for x in pinned]
        assert assert_state_parity(got, want, "offload [%d,%d)" % (lo, hi)) == 0
    # whole shard, on the host: the bf16 image is the cast of the new master weight
    step = 1 << 26
    for lo in range(0, n, step):
        hi = min(lo + step, n)
        assert torch.equal(pinned[0][lo:hi].to(torch.bfloat16).view(torch.int16),
                           pinned[3][lo:hi].view(torch.int16))
    del pinned, grads, slots
    torch.cuda.empty_cache()

"""Full-size GPU parity in the launch configurations bench.py times.  The 7B ZeRO-2
shard (one launch), the 70B ZeRO-3 shard (33 buckets read in place from arena
buffers) and the ragged 13B shard with clipping (two phases) are compared with the
oracle on EVERY element: inputs are generated on the device from seeded generators,
the state before the step is regenerated chunk by chunk afterwards, and chunks of
2^27 elements travel to the host where the oracle runs on all cores.  The staged
two-stream pipeline is checked on whole buckets at full size, the ZeRO-1,
accumulation and offload rows on sampled slices, the verification scans on whole
buffers.  Whole-shard properties that hold at any size are checked on the device
with library primitives."""
import ctypes as C
import time

import numpy as np
import pytest
import torch

import paper_2601_02311_amd as ps
from oracle import step as orc
from synth import WORKLOADS
from synth import device as dgen

from gpu_util import (HostChunks, assert_state_parity, host, oracle_mismatches, shard_of,
                      stream_handle)

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


CHUNK = dgen.CHUNK            # elements per host round trip of the every-element checks


def _progress(capsys, msg):
    """A line that reaches the terminal while the test runs (long tests must not look hung)."""
    with capsys.disabled():
        print("[full-size] " + msg, flush=True)


def _pinned(n_contrib, grad_torch_dtype, param_torch_dtype, extra=()):
    spec = {"g%d" % r: (CHUNK, grad_torch_dtype) for r in range(n_contrib)}
    for k in ("th0", "m0", "v0", "th1", "m1", "v1"):
        spec[k] = (CHUNK, torch.float32)
    spec["p1"] = (CHUNK, param_torch_dtype)
    for name, dt in extra:
        spec[name] = (CHUNK, dt)
    return HostChunks(**spec)


class _Arena:
    """Flat buffers as bench.py allocates them for the large workloads: one arena, physical
    memory created in chunks of 2^28 elements; views for torch, released on exit."""

    def __init__(self, n, elem_bytes, chunk=1 << 28):
        self.n = n
        self.handle = ps.ps_arena_create(n, chunk, elem_bytes)
        self.ptr = [ps.ps_arena_buffer(self.handle, k) for k in range(len(elem_bytes))]

    def view(self, k, dtype):
        return dgen.as_tensor(self.ptr[k], self.n, dtype)

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        torch.cuda.synchronize()
        ps.ps_arena_destroy(self.handle)
        return False


def _check_every_element(capsys, what, w, s, pin, grads_of_chunk, master, m, v, out_slice, valid,
                         saved_head=None):
    """Every element of [0, valid) against the oracle: the state before the step is regenerated
    chunk by chunk from the seeded generator (same values the buffers were filled with), the
    contributions and the state after the step come from the device; the oracle runs on all
    host threads.  Asserts zero differing elements in master, m, v and the 16-bit image."""
    bad = [0, 0, 0, 0]
    done = 0
    t0 = time.time()
    for lo, hi, th0, m0, v0 in dgen.state_chunks(w):
        if lo >= valid:
            break
        k = min(hi, valid) - lo
        pre = [pin.fetch("th0", th0), pin.fetch("m0", m0), pin.fetch("v0", v0)]
        if lo == 0 and saved_head is not None:      # the regenerated stream is the one the buffers held
            for a, b in zip(pre, saved_head):
                assert np.array_equal(a[:b.shape[0]].view(np.uint32), b.view(np.uint32))
        grads = grads_of_chunk(lo, hi)
        post = [pin.fetch("th1", master[lo:hi]), pin.fetch("m1", m[lo:hi]), pin.fetch("v1", v[lo:hi]),
                pin.fetch("p1", out_slice[lo:hi])]
        if hi > valid:                               # pad: untouched, byte for byte
            for a, b in zip(post[:3], pre):
                assert np.array_equal(a[k:].view(np.uint32), b[k:].view(np.uint32)), what + ": pad touched"
        for j, x in enumerate(oracle_mismatches(orc.step_f32, s, grads, pre, post, k)):
            bad[j] += x
        done += k
        if (lo // CHUNK) % 8 == 7 or hi >= valid:
            _progress(capsys, "%s: %d of %d elements checked against the oracle, %.0f s, mismatches %s"
                      % (what, done, valid, time.time() - t0, bad))
        assert bad == [0, 0, 0, 0], "%s: elements differing from the oracle in [%d,%d): %s" % (what, lo, hi, bad)
    assert done == valid
    return bad


@pytest.mark.parametrize("name", ["7b_zero2", "7b_zero2_f16"])
def test_7b_zero2_full_shard_every_element(name, capsys):
    """bf16 gradients and parameters, and the same shard in binary16 with a loss scale: one
    launch over the whole shard, every element compared with the oracle."""
    w = WORKLOADS[name]
    _need(45)
    n, N, t = w.shard_len, w.n_devices, w.first_step
    f16 = w.param_dtype == "f16"
    tdt = torch.float16 if f16 else torch.bfloat16
    _say("%s full shard n=%d, one launch, every element" % (name, n))
    spec = ps.ps_spec_preset(w.strategy, N, w.shard_index, w.psi)
    cost = ps.ps_cost_eval(spec)
    with _Arena(n, [2] * N + [4, 4, 4]) as ar:                                # contributions, master, m, v
        master, m, v = dgen.workload_state(w, into=[ar.view(N + j, torch.float32) for j in range(3)])
        head = [_take(x, 0, 4096) for x in (master, m, v)]
        grads = [dgen.fill_gradient_(ar.view(r, tdt), w.seed, t, r, w.grad_std * w.loss_scale,
                                     w.outlier_frac, w.outlier_mult, w.student_t_dof) for r in range(N)]
        out = torch.zeros(cost.psi_padded, dtype=tdt, device="cuda")           # replicated Theta
        gs = 1.0 / (N * w.loss_scale) if w.loss_scale != 1.0 else 0.0
        hpd, hp = _hp(w, t, grad_scale=gs)
        ps.ps_step_update(spec, hp, shard_of(master, m, v, out, n), ps.make_grads(
            [g.data_ptr() for g in grads], ps.PS_F16 if f16 else ps.PS_BF16), 0, n, stream_handle())
        torch.cuda.synchronize()
        s = orc.derive_scalars(t=t, n_devices=N, grad_scale=gs, **hpd)
        off = cost.shard_offset
        pin = _pinned(N, tdt, tdt)
        _check_every_element(capsys, name, w, s, pin,
                             lambda lo, hi: [pin.fetch("g%d" % r, grads[r][lo:hi]) for r in range(N)],
                             master, m, v, out[off:off + n], n, saved_head=head)
        assert not bool(out[off + n:].view(torch.int16).any())                 # the other shards' slices untouched
        del master, m, v, grads, out, pin
    torch.cuda.empty_cache()


def test_70b_zero3_in_place_every_element(capsys):
    """The configuration bench.py times: the whole 70B shard, its 140 GB of contributions
    resident and distinct in flat arena buffers, 33 buckets read in place; every one of the
    8.75e9 elements compared with the oracle."""
    w = WORKLOADS["70b_zero3"]
    _need(280)
    n, N, t, B = w.shard_len, w.n_devices, w.first_step, w.bucket_elems
    n_b = -(-n // B)
    _say("70b_zero3 full shard n=%d, %d buckets of %d read in place from arena buffers, every element" % (n, n_b, B))
    spec = ps.ps_spec_preset(w.strategy, N, w.shard_index, w.psi)
    arena = ps.ps_arena_create(n, B, [2] * N + [4, 4, 4, 2])
    try:
        buf = [ps.ps_arena_buffer(arena, k) for k in range(N + 4)]
        master, m, v = dgen.workload_state(w, into=[dgen.as_tensor(buf[N + j], n, torch.float32) for j in range(3)])
        out = dgen.as_tensor(buf[N + 3], n, torch.bfloat16).zero_()
        grads = [dgen.fill_gradient_(dgen.as_tensor(buf[r], n, torch.bfloat16), w.seed, t, r, w.grad_std)
                 for r in range(N)]
        head = [_take(x, 0, 4096) for x in (master, m, v)]
        comp = torch.cuda.Stream()
        torch.cuda.synchronize()
        plan = ps.ps_bucket_plan_t()
        arr = (C.c_void_p * N)(*buf[:N])
        plan.source = C.cast(arr, C.POINTER(C.c_void_p))
        plan.n_contrib, plan.dtype, plan.bucket_elems = N, ps.PS_BF16, B
        plan.source_elems = -(-n // 512) * 512          # as long as the shard: never wraps
        plan.compute_stream, plan.copy_engine = comp.cuda_stream, ps.PS_COPY_NONE
        hpd, hp = _hp(w, t)
        ps.ps_step_update_bucketed(spec, hp, shard_of(master, m, v, out, n), plan)
        torch.cuda.synchronize()
        s = orc.derive_scalars(t=t, n_devices=N, **hpd)
        pin = _pinned(N, torch.bfloat16, torch.bfloat16)
        _check_every_element(capsys, "70b in place", w, s, pin,
                             lambda lo, hi: [pin.fetch("g%d" % r, grads[r][lo:hi]) for r in range(N)],
                             master, m, v, out, n, saved_head=head)
        del master, m, v, out, grads, pin
    finally:
        torch.cuda.synchronize()
        ps.ps_arena_destroy(arena)
    torch.cuda.empty_cache()


@pytest.mark.parametrize("engine", ["copy", "reduce"])
def test_70b_zero3_staged_pipeline_whole_buckets(engine, capsys):
    """The two-stream pipeline that stages each bucket first (the copy kernel, or the reduce
    kernel staging the FP32 sum), at full size, from a pool whose length does not divide the
    bucket size (every bucket starts somewhere else in the pool and wraps inside it).  Whole
    buckets 0, 15 (the other staging slot), 16 and the short last one are compared element by
    element with the oracle; the rest of the shard by properties."""
    w = WORKLOADS["70b_zero3"]
    _need(150)
    n, N, t, B = w.shard_len, w.n_devices, w.first_step, w.bucket_elems
    pool_elems = 5 * (1 << 25) + 3 * 512
    n_b = -(-n // B)
    check = (0, 15, 16, n_b - 1)
    _say("70b_zero3 staged (%s): n=%d, %d buckets of %d, pool %d, whole buckets %s" % (engine, n, n_b, B, pool_elems, check))
    spec = ps.ps_spec_preset(w.strategy, N, w.shard_index, w.psi)
    master, m, v = dgen.workload_state(w)
    out = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    pool = [dgen.fill_gradient_(torch.empty(pool_elems, dtype=torch.bfloat16, device="cuda"),
                                w.seed, t, r, w.grad_std) for r in range(N)]
    pool_np = [host(p) for p in pool]
    if engine == "reduce":          # the slots hold one FP32 sum per element
        staging = [torch.empty(B, dtype=torch.float32, device="cuda") for _ in range(2)]
    else:
        staging = [torch.empty(N * B, dtype=torch.bfloat16, device="cuda") for _ in range(2)]
    copy, comp = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    plan = ps.ps_bucket_plan_t()
    arr = (C.c_void_p * N)(*[p.data_ptr() for p in pool])
    plan.source = C.cast(arr, C.POINTER(C.c_void_p))
    plan.n_contrib, plan.dtype, plan.bucket_elems, plan.source_elems = N, ps.PS_BF16, B, pool_elems
    plan.staging[0], plan.staging[1] = staging[0].data_ptr(), staging[1].data_ptr()
    plan.copy_stream, plan.compute_stream = copy.cuda_stream, comp.cuda_stream
    plan.copy_engine = ps.PS_COPY_REDUCE if engine == "reduce" else ps.PS_COPY_KERNEL
    plan.schedule = ps.PS_SCHED_AUTO
    hpd, hp = _hp(w, t)
    ps.ps_step_update_bucketed(spec, hp, shard_of(master, m, v, out, n), plan)
    torch.cuda.synchronize()
    s = orc.derive_scalars(t=t, n_devices=N, **hpd)
    pin = _pinned(0, torch.bfloat16, torch.bfloat16)

    def wrapped(lo, hi):
        """Contributions of elements [lo, hi): element e reads source[e % source_elems]."""
        outs = []
        for p_ in pool_np:
            parts, cur = [], lo
            while cur < hi:
                pos = cur % pool_elems
                take = min(hi - cur, pool_elems - pos)
                parts.append(p_[pos:pos + take])
                cur += take
            outs.append(np.ascontiguousarray(np.concatenate(parts)))
        return outs
    bad, t0 = [0, 0, 0, 0], time.time()
    for lo, hi, th0, m0, v0 in dgen.state_chunks(w):
        if lo // B not in check and (hi - 1) // B not in check:
            continue                                   # the generators still advanced past this chunk
        pre = [pin.fetch("th0", th0), pin.fetch("m0", m0), pin.fetch("v0", v0)]
        post = [pin.fetch("th1", master[lo:hi]), pin.fetch("m1", m[lo:hi]), pin.fetch("v1", v[lo:hi]),
                pin.fetch("p1", out[lo:hi])]
        for j, x in enumerate(oracle_mismatches(orc.step_f32, s, wrapped(lo, hi), pre, post, hi - lo)):
            bad[j] += x
        _progress(capsys, "70b staged: [%d,%d) (bucket %d) checked, %.0f s, mismatches %s"
                  % (lo, hi, lo // B, time.time() - t0, bad))
        assert bad == [0, 0, 0, 0]
    _whole_shard_properties(master, m, v, out, n)
    del master, m, v, out, pool, staging, pin
    torch.cuda.empty_cache()


def test_13b_clip_ragged_full_shard_every_element(capsys):
    """Ragged 13B shard, six fp32 contributions, global-norm clipping in two phases.  The mean
    gradient of every valid element and the sum of its squares come from the oracle
    (sequential binary64), the coefficient both sides use is formed from THAT sum, and every
    element of the updated state is compared with the oracle; the pad stays untouched."""
    w = WORKLOADS["13b_clip"]
    _need(100)
    N, t = w.n_devices, w.first_step
    psi = w.extra["psi_ragged"]                          # same buffers, last shard owns a pad of 1001
    spec = ps.ps_spec_preset(w.strategy, N, w.shard_index, psi, align_elems=w.align_elems)
    cost = ps.ps_cost_eval(spec)
    n, valid = cost.shard_len, cost.valid_len
    assert n == w.shard_len and valid == n - 1001
    _say("13b_clip ragged full shard n=%d valid=%d N=%d fp32, two phases, every element" % (n, valid, N))
    # contributions, master, m, v, parameters, reduced gradient: the buffers bench.py allocates
    with _Arena(n, [4] * N + [4, 4, 4, 2, 4]) as ar:
        master, m, v = dgen.workload_state(w, into=[ar.view(N + j, torch.float32) for j in range(3)])
        head = [_take(x, 0, 4096) for x in (master, m, v)]
        grads = [dgen.fill_gradient_(ar.view(r, torch.float32), w.seed, t, r, w.grad_std * w.loss_scale,
                                     w.outlier_frac, w.outlier_mult, w.student_t_dof) for r in range(N)]
        out = ar.view(N + 3, torch.bfloat16).fill_(-1.0)
        red = ar.view(N + 4, torch.float32).fill_(float("nan"))
        ssd = torch.zeros(1, dtype=torch.float64, device="cuda")
        ws = torch.empty(ps.ps_workspace_bytes(n), dtype=torch.uint8, device="cuda")
        g = ps.make_grads([x.data_ptr() for x in grads], ps.PS_F32)
        ps.ps_step_reduce_sumsq(spec, g, 0.0, red.data_ptr(), ssd.data_ptr(), 0, ws.data_ptr(),
                                ws.numel(), 0, n, valid, stream_handle())
        ss_gpu = float(ssd.item())
        again = torch.zeros(1, dtype=torch.float64, device="cuda")
        ps.ps_step_reduce_sumsq(spec, g, 0.0, 0, again.data_ptr(), 0, ws.data_ptr(), ws.numel(), 0, n,
                                valid, stream_handle())
        assert float(again.item()) == ss_gpu                                  # run-to-run identical
        # phase 1 against the oracle: the mean bit for bit on every element, the sum within the
        # sequential sum's own rounding bound (valid * 2^-53 relative, all terms >= 0)
        pin = _pinned(N, torch.float32, torch.bfloat16, extra=[("red", torch.float32)])
        gs = np.float32(1.0 / N)
        ss_oracle, t0 = 0.0, time.time()
        for lo in range(0, valid, CHUNK):
            hi = min(lo + CHUNK, valid)
            gr = [pin.fetch("g%d" % r, grads[r][lo:hi]) for r in range(N)]
            gm, ss_c = orc.mean_sumsq(gr, gs, 0, hi - lo)
            ss_oracle += ss_c
            assert np.array_equal(gm.view(np.uint32), pin.fetch("red", red[lo:hi]).view(np.uint32))
            if (lo // CHUNK) % 8 == 7 or hi == valid:
                _progress(capsys, "13b phase 1: mean of %d of %d elements equals the oracle's, %.0f s"
                          % (hi, valid, time.time() - t0))
        assert abs(ss_gpu - ss_oracle) <= valid * 2.0 ** -53 * ss_oracle
        assert bool(torch.isnan(red[valid:]).all())                           # pad never written
        coef = orc.clip_coef(ss_oracle, 5 * ss_oracle, w.max_grad_norm)       # five iid peer shards
        assert ps.ps_clip_coef(ss_oracle, 5 * ss_oracle, w.max_grad_norm) == coef
        hpd, hp = _hp(w, t, grad_scale=1.0, clip_coef=coef)
        ps.ps_step_update(spec, hp, shard_of(master, m, v, out, n, valid),
                          ps.make_grads([red.data_ptr()], ps.PS_F32), 0, n, stream_handle())
        torch.cuda.synchronize()
        s = orc.derive_scalars(t=t, n_devices=N, clip_coef=coef, **hpd)       # the unsharded definition:
        _check_every_element(capsys, "13b phase 2", w, s, pin,                # six contributions, mean 1/N
                             lambda lo, hi: [pin.fetch("g%d" % r, grads[r][lo:hi]) for r in range(N)],
                             master, m, v, out, valid, saved_head=head)
        assert bool((out[valid:].view(torch.int16) == out.new_full((1,), -1.0).view(torch.int16)).all())
        del master, m, v, out, red, grads, ws, pin
    torch.cuda.empty_cache()


def test_single_launch_beyond_2_32_elements(capsys):
    """Maximum size in one launch: the whole 70B shard (8.75e9 elements, 34 million
    workgroups) updated from one pre-reduced fp32 gradient; element indices pass 2^32
    and byte offsets pass 2^35.  Every element is compared with the oracle."""
    w = WORKLOADS["70b_zero3"]
    _need(165)
    n, N, t = w.shard_len, w.n_devices, w.first_step
    _say("single launch over n=%d elements (fp32 pre-reduced gradient), every element" % n)
    spec = ps.ps_spec_preset(w.strategy, N, w.shard_index, w.psi)
    master, m, v = dgen.workload_state(w)
    head = [_take(x, 0, 4096) for x in (master, m, v)]
    g = dgen.fill_normal_(torch.empty(n, dtype=torch.float32, device="cuda"), 1e-4, w.seed, 9)
    out = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    hpd, hp = _hp(w, t, grad_scale=1.0)
    ps.ps_step_update(spec, hp, shard_of(master, m, v, out, n),
                      ps.make_grads([g.data_ptr()], ps.PS_F32), 0, n, stream_handle())
    torch.cuda.synchronize()
    s = orc.derive_scalars(t=t, n_devices=N, grad_scale=1.0, **hpd)
    pin = _pinned(1, torch.float32, torch.bfloat16)
    _check_every_element(capsys, "one launch, 8.75e9 elements", w, s, pin,
                         lambda lo, hi: [pin.fetch("g0", g[lo:hi])], master, m, v, out, n, saved_head=head)
    del master, m, v, g, out, pin
    torch.cuda.empty_cache()


# ---- rows beyond the base path, at the sizes bench.py times them ----

def test_7b_zero1_full_shard_every_element(capsys):
    """ZeRO-1 row: one all-reduced, replicated bf16 gradient of psi elements; the library
    reads and writes slice i.  Run for the shard bench.py uses and for one with a large
    offset; every element of each is compared with the oracle."""
    w = WORKLOADS["7b_zero1"]
    _need(45)
    N, t = w.n_devices, w.first_step
    n = w.shard_len
    grad = dgen.fill_gradient_(torch.empty(w.psi, dtype=torch.bfloat16, device="cuda"),
                               w.seed, t, 0, w.grad_std)
    out = torch.zeros(w.psi, dtype=torch.bfloat16, device="cuda")
    pin = _pinned(1, torch.bfloat16, torch.bfloat16)
    for i in (w.shard_index, 5):
        master, m, v = dgen.workload_state(w)                     # the same state for either shard index
        head = [_take(x, 0, 4096) for x in (master, m, v)]
        spec = ps.ps_spec_preset(w.strategy, N, i, w.psi)
        cost = ps.ps_cost_eval(spec)
        assert cost.shard_len == n and cost.psi_padded == w.psi
        off = cost.shard_offset
        _say("7b_zero1 shard %d: n=%d at offset %d of the replicated gradient, every element" % (i, n, off))
        out.zero_()
        hpd, hp = _hp(w, t)
        ps.ps_step_update(spec, hp, shard_of(master, m, v, out, n),
                          ps.make_grads([grad.data_ptr()], ps.PS_BF16), 0, n, stream_handle())
        torch.cuda.synchronize()
        s = orc.derive_scalars(t=t, n_devices=N, **hpd)          # grad_scale 0: 1/N, the all-reduce sums
        _check_every_element(capsys, "zero1 shard %d" % i, w, s, pin,
                             lambda lo, hi: [pin.fetch("g0", grad[off + lo:off + hi])],
                             master, m, v, out[off:off + n], n, saved_head=head)
        assert not bool(out[:off].view(torch.int16).any())        # the other shards' slices untouched
        assert not bool(out[off + n:].view(torch.int16).any())
        del master, m, v
    del grad, out, pin
    torch.cuda.empty_cache()


def test_7b_accum4_full_shard_every_element(capsys):
    """Gradient accumulation row: four micro-batches (fresh contributions each), the first
    three into the FP32 accumulator, the last straight into the update beside the
    accumulator, grad_scale = 1/(N k).  The accumulator after three micro-batches (oracle:
    accumulate over the whole shard, on all host threads) and the updated state (oracle:
    the fourth accumulation, then the update from the accumulator alone) are compared on
    every element."""
    import threading
    w = WORKLOADS["7b_accum4"]
    _need(45)
    n, N, t, k = w.shard_len, w.n_devices, w.first_step, w.micro_batches
    _say("7b_accum4 full shard n=%d, %d micro-batches, every element" % (n, k))
    spec = ps.ps_spec_preset(w.strategy, N, w.shard_index, w.psi)
    cost = ps.ps_cost_eval(spec)
    master, m, v = dgen.workload_state(w)
    head = [_take(x, 0, 4096) for x in (master, m, v)]
    out = torch.zeros(n, dtype=torch.bfloat16, device="cuda")      # this shard's slice only
    accum = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
    acc_want = np.full(n, np.float32(np.nan))                       # the oracle's accumulator, whole shard
    pin = _pinned(N, torch.bfloat16, torch.bfloat16, extra=[("acc", torch.float32)])
    threads = 16
    grads = None
    for j in range(k):
        del grads
        grads = dgen.workload_gradients(w, t * 16 + j)             # a different stream per micro-batch
        if j < k - 1:
            ps.ps_step_accumulate(spec, ps.make_grads([g.data_ptr() for g in grads], ps.PS_BF16),
                                  accum.data_ptr(), j == 0, 0, n, n, stream_handle())
        else:       # what the device's accumulator holds when the last micro-batch arrives
            for lo in range(0, n, CHUNK):
                hi = min(lo + CHUNK, n)
                assert np.array_equal(pin.fetch("acc", accum[lo:hi]).view(np.uint32),
                                      acc_want[lo:hi].view(np.uint32))
        for lo in range(0, n, CHUNK):
            hi = min(lo + CHUNK, n)
            gr = [pin.fetch("g%d" % r, grads[r][lo:hi]) for r in range(N)]
            part = acc_want[lo:hi]
            bounds = [(hi - lo) * q // threads for q in range(threads + 1)]
            ts = [threading.Thread(target=orc.accumulate, args=(gr, part, j == 0, bounds[q], bounds[q + 1]))
                  for q in range(threads)]
            for x in ts:
                x.start()
            for x in ts:
                x.join()
        torch.cuda.synchronize()
        _progress(capsys, "accumulation: micro-batch %d of %d %s" %
                  (j + 1, k, "added on both sides" if j < k - 1 else "added by the oracle"))
    scale = 1.0 / (N * k)
    hpd, hp = _hp(w, t, grad_scale=scale)
    assert cost.shard_offset == 0          # shard 0: its slice of the replicated parameters starts the buffer
    ws = torch.empty(ps.ps_verify_workspace_bytes(n * 4), dtype=torch.uint8, device="cuda")
    sums = torch.zeros(2, dtype=torch.int64, device="cuda")
    ps.ps_verify_checksum(accum.data_ptr(), n * 4, 0, sums[0:].data_ptr(), 0, ws.data_ptr(), ws.numel(),
                          stream_handle())
    ps.ps_step_update(spec, hp, shard_of(master, m, v, out, n),
                      ps.make_grads([g.data_ptr() for g in grads], ps.PS_BF16, accum=accum.data_ptr()),
                      0, n, stream_handle())
    ps.ps_verify_checksum(accum.data_ptr(), n * 4, 0, sums[1:].data_ptr(), 0, ws.data_ptr(), ws.numel(),
                          stream_handle())
    torch.cuda.synchronize()
    assert sums[0].item() == sums[1].item()                        # the accumulator is only read
    s = orc.derive_scalars(t=t, n_devices=N, grad_scale=scale, **hpd)
    _check_every_element(capsys, "update from the accumulator", w, s, pin,
                         lambda lo, hi: [np.ascontiguousarray(acc_want[lo:hi])],
                         master, m, v, out, n, saved_head=head)
    del master, m, v, out, accum, grads, pin
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


@pytest.mark.parametrize("packed", [True, False])
def test_7b_offload_full_shard_every_element(packed, capsys):
    """ZeRO-Offload row at bench.py's shape: master/m/v and the bf16 parameters of the 7B
    shard in pinned host memory (one image packed bucket by bucket, or four flat arrays),
    streamed through three device slots of 2^25 elements; every element compared."""
    w = WORKLOADS["7b_offload"]
    _need(20)
    n, N, t, B = w.shard_len, w.n_devices, w.first_step, w.bucket_elems
    n_b = -(-n // B)
    _say("7b_offload full shard n=%d, buckets of %d through 3 slots, packed=%s, every element" % (n, B, packed))
    spec = ps.ps_spec_preset(w.strategy, N, w.shard_index, w.psi)
    state = [x.cpu().numpy() for x in dgen.workload_state(w)]        # the state before the step, on the host
    torch.cuda.empty_cache()
    plan = ps.ps_offload_plan_t()
    if packed:
        image = torch.full((n_b * 14 * B,), 0xEE, dtype=torch.uint8).pin_memory()
        img = image.numpy()
        for b in range(n_b):
            lo, hi = b * B, min((b + 1) * B, n)
            for j in range(3):
                img[b * 14 * B + 4 * B * j:b * 14 * B + 4 * B * j + 4 * (hi - lo)] = state[j][lo:hi].view(np.uint8)
        plan.host_layout, plan.host_packed = ps.PS_HOST_PACKED, image.data_ptr()
    else:
        pinned = [torch.from_numpy(a.copy()).pin_memory() for a in state]
        pinned.append(torch.zeros(n, dtype=torch.bfloat16).pin_memory())
        plan.host_master, plan.host_m, plan.host_v, plan.host_param_out = [x.data_ptr() for x in pinned]
    grads = dgen.workload_gradients(w, t)
    slots = [torch.empty(14 * B, dtype=torch.uint8, device="cuda") for _ in range(3)]
    s1, s2, s3 = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    plan.len, plan.valid_len, plan.bucket_elems, plan.n_slots = n, n, B, 3
    for j, x in enumerate(slots):
        plan.slot[j] = x.data_ptr()
    plan.h2d_stream, plan.compute_stream, plan.d2h_stream = s1.cuda_stream, s2.cuda_stream, s3.cuda_stream
    hpd, hp = _hp(w, t)
    ps.ps_step_update_offloaded(spec, hp, plan, ps.make_grads([g.data_ptr() for g in grads], ps.PS_BF16))
    torch.cuda.synchronize()
    s = orc.derive_scalars(t=t, n_devices=N, **hpd)
    pin = _pinned(N, torch.bfloat16, torch.bfloat16)
    bad, t0 = [0, 0, 0, 0], time.time()
    for b in range(n_b):                                             # one bucket at a time
        lo, hi = b * B, min((b + 1) * B, n)
        gr = [pin.fetch("g%d" % r, grads[r][lo:hi]) for r in range(N)]
        pre = [np.ascontiguousarray(a[lo:hi]) for a in state]
        if packed:
            base = b * 14 * B
            post = [img[base + 4 * B * j:base + 4 * B * j + 4 * (hi - lo)].view(np.float32) for j in range(3)]
            post.append(img[base + 12 * B:base + 12 * B + 2 * (hi - lo)].view(np.uint16))
        else:
            post = [x[lo:hi].numpy() for x in pinned[:3]] + [pinned[3][lo:hi].view(torch.int16).numpy().view(np.uint16)]
        for j, x in enumerate(oracle_mismatches(orc.step_f32, s, gr, pre, post, hi - lo)):
            bad[j] += x
        assert bad == [0, 0, 0, 0], "offload bucket %d: %s" % (b, bad)
    _progress(capsys, "offload packed=%s: %d elements checked against the oracle, %.0f s, mismatches %s"
              % (packed, n, time.time() - t0, bad))
    if packed:                                                       # bytes that belong to no element keep their canary
        tail = n - (n_b - 1) * B
        base = (n_b - 1) * 14 * B
        for j in range(3):
            assert (img[base + 4 * B * j + 4 * tail:base + 4 * B * (j + 1)] == 0xEE).all()
        assert (img[base + 12 * B + 2 * tail:base + 14 * B] == 0xEE).all()
    del grads, slots, pin
    torch.cuda.empty_cache()

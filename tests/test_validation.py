"""Argument validation of the device entry points.  Every case here is rejected
before the first HIP call, so fake (never dereferenced) addresses are safe and
the results are the same with or without a GPU."""
import ctypes as C

import pytest
import torch

import paper_2601_02311_amd as ps

FAKE = 0x10000  # 16-byte aligned, never dereferenced


def _valid(n=1024, N=4, theta="zero3"):
    spec = ps.ps_spec_preset(theta, N, 1, n * N)
    hp = ps.ps_adamw_t(1e-4, 0.9, 0.999, 1e-8, 0.01, 1, 0.0, 0.0)
    shard = ps.ps_shard_t(FAKE, FAKE * 2, FAKE * 3, FAKE * 4, n, n)
    grads = ps.make_grads([FAKE * (5 + r) for r in range(N)], ps.PS_BF16)
    return spec, hp, shard, grads


def _status(fn):
    with pytest.raises(ps.PsError) as e:
        fn()
    assert e.value.detail
    return e.value.status


def test_update_rejects_bad_arguments():
    spec, hp, shard, grads = _valid()
    upd = ps.ps_step_update
    assert _status(lambda: upd(None, hp, shard, grads, 0, 8)) == ps.PS_EINVAL
    assert _status(lambda: upd(spec, None, shard, grads, 0, 8)) == ps.PS_EINVAL
    assert _status(lambda: upd(spec, hp, None, grads, 0, 8)) == ps.PS_EINVAL
    assert _status(lambda: upd(spec, hp, shard, None, 0, 8)) == ps.PS_EINVAL
    # placements this path does not execute
    for name in ("zero_offload", "tp", "pp"):
        other = ps.ps_spec_preset(name, 4, 1, 4096)
        assert _status(lambda: upd(other, hp, shard, grads, 0, 8)) == ps.PS_EUNSUPPORTED
    # step count, betas
    bad = ps.ps_adamw_t(1e-4, 0.9, 0.999, 1e-8, 0.01, 0, 0.0, 0.0)
    assert _status(lambda: upd(spec, bad, shard, grads, 0, 8)) == ps.PS_ERANGE
    bad = ps.ps_adamw_t(1e-4, 1.0, 0.999, 1e-8, 0.01, 1, 0.0, 0.0)
    assert _status(lambda: upd(spec, bad, shard, grads, 0, 8)) == ps.PS_ERANGE
    bad = ps.ps_adamw_t(float("nan"), 0.9, 0.999, 1e-8, 0.01, 1, 0.0, 0.0)
    assert _status(lambda: upd(spec, bad, shard, grads, 0, 8)) == ps.PS_ERANGE
    # shard buffers
    s2 = ps.ps_shard_t(0, FAKE, FAKE, FAKE, 1024, 1024)
    assert _status(lambda: upd(spec, hp, s2, grads, 0, 8)) == ps.PS_EINVAL
    s2 = ps.ps_shard_t(FAKE + 4, FAKE, FAKE, FAKE, 1024, 1024)
    assert _status(lambda: upd(spec, hp, s2, grads, 0, 8)) == ps.PS_EALIGN
    s2 = ps.ps_shard_t(FAKE, FAKE, FAKE, FAKE, 1000, 1000)
    assert _status(lambda: upd(spec, hp, s2, grads, 0, 8)) == ps.PS_ERANGE
    s2 = ps.ps_shard_t(FAKE, FAKE, FAKE, FAKE, 1024, 1025)
    assert _status(lambda: upd(spec, hp, s2, grads, 0, 8)) == ps.PS_ERANGE
    # ranges
    assert _status(lambda: upd(spec, hp, shard, grads, 4, 8)) == ps.PS_EALIGN
    assert _status(lambda: upd(spec, hp, shard, grads, 1024, 8)) == ps.PS_ERANGE
    assert _status(lambda: upd(spec, hp, shard, grads, 8, 1024)) == ps.PS_ERANGE
    assert _status(lambda: upd(spec, hp, shard, grads, 2 ** 63, 2 ** 63)) == ps.PS_ERANGE


def test_update_rejects_integrity_violations():
    """A missing or surplus contribution, a NULL one, or mixed element types are
    refused: they are the paper's gradient-integrity / type-mismatch violations."""
    spec, hp, shard, _ = _valid()
    upd = ps.ps_step_update
    missing = ps.make_grads([FAKE] * 3, ps.PS_BF16)
    assert _status(lambda: upd(spec, hp, shard, missing, 0, 8)) == ps.PS_EINVAL
    extra = ps.make_grads([FAKE] * 5, ps.PS_BF16)
    assert _status(lambda: upd(spec, hp, shard, extra, 0, 8)) == ps.PS_EINVAL
    null = ps.make_grads([FAKE, 0, FAKE, FAKE], ps.PS_BF16)
    assert _status(lambda: upd(spec, hp, shard, null, 0, 8)) == ps.PS_EINVAL
    odd = ps.make_grads([FAKE, FAKE + 2, FAKE, FAKE], ps.PS_BF16)
    assert _status(lambda: upd(spec, hp, shard, odd, 0, 8)) == ps.PS_EALIGN
    badtype = ps.make_grads([FAKE] * 4, 3)
    assert _status(lambda: upd(spec, hp, shard, badtype, 0, 8)) == ps.PS_EINVAL
    one_bf16 = ps.make_grads([FAKE], ps.PS_BF16)       # a single pre-reduced gradient is fp32 only
    assert _status(lambda: upd(spec, hp, shard, one_bf16, 0, 8)) == ps.PS_EINVAL
    none = ps.make_grads([], ps.PS_BF16)
    assert _status(lambda: upd(spec, hp, shard, none, 0, 8)) == ps.PS_ERANGE
    spec17 = ps.ps_spec_preset("zero3", 17, 0, 17 * 1024)
    many = ps.make_grads([FAKE] * 17, ps.PS_BF16)
    assert _status(lambda: upd(spec17, hp, shard, many, 0, 8)) == ps.PS_ERANGE


def test_zero1_takes_one_replicated_gradient():
    spec = ps.ps_spec_preset("zero1", 4, 1, 4096)
    _, hp, shard, grads4 = _valid()
    upd = ps.ps_step_update
    assert _status(lambda: upd(spec, hp, shard, grads4, 0, 8)) == ps.PS_EINVAL      # N buffers: no
    two = ps.make_grads([FAKE, FAKE], ps.PS_BF16)
    assert _status(lambda: upd(spec, hp, shard, two, 0, 8)) == ps.PS_EINVAL
    one = ps.make_grads([FAKE], ps.PS_BF16)
    upd(spec, hp, shard, one, 0, 0)                                                  # valid, empty
    assert _status(lambda: ps.ps_step_accumulate(spec, one, FAKE, 1, 0, 8, 1024)) == ps.PS_EUNSUPPORTED
    plan = ps.ps_bucket_plan_t()
    assert _status(lambda: ps.ps_step_update_bucketed(spec, hp, shard, plan)) == ps.PS_EUNSUPPORTED


def test_data_parallel_updates_the_whole_tensor():
    """All four states R: the "shard" is everything, the gradient one all-reduced buffer."""
    spec = ps.ps_spec_preset("dp", 4, 1, 4096)
    _, hp, shard, grads4 = _valid()
    upd = ps.ps_step_update
    one = ps.make_grads([FAKE], ps.PS_BF16)
    assert _status(lambda: upd(spec, hp, shard, one, 0, 8)) == ps.PS_ERANGE         # a quarter is not the whole
    whole = ps.ps_shard_t(FAKE, FAKE * 2, FAKE * 3, FAKE * 4, 4096, 4096)
    assert _status(lambda: upd(spec, hp, whole, grads4, 0, 8)) == ps.PS_EINVAL       # N buffers: no
    upd(spec, hp, whole, one, 0, 0)                                                  # valid, empty
    assert _status(lambda: upd(spec, hp, whole, one, 4096, 8)) == ps.PS_ERANGE
    assert _status(lambda: ps.ps_step_accumulate(spec, one, FAKE, 1, 0, 8, 4096)) == ps.PS_EUNSUPPORTED
    plan = ps.ps_bucket_plan_t()
    assert _status(lambda: ps.ps_step_update_bucketed(spec, hp, whole, plan)) == ps.PS_EUNSUPPORTED


def test_accumulate_rejects_bad_arguments():
    spec, _, _, grads = _valid()
    acc = ps.ps_step_accumulate
    assert _status(lambda: acc(None, grads, FAKE, 1, 0, 8, 1024)) == ps.PS_EINVAL
    assert _status(lambda: acc(spec, None, FAKE, 1, 0, 8, 1024)) == ps.PS_EINVAL
    assert _status(lambda: acc(spec, grads, 0, 1, 0, 8, 1024)) == ps.PS_EINVAL
    assert _status(lambda: acc(spec, grads, FAKE + 4, 1, 0, 8, 1024)) == ps.PS_EALIGN
    assert _status(lambda: acc(spec, grads, FAKE, 1, 4, 8, 1024)) == ps.PS_EALIGN
    assert _status(lambda: acc(spec, grads, FAKE, 1, 1024, 8, 1024)) == ps.PS_ERANGE
    assert _status(lambda: acc(spec, grads, FAKE, 1, 0, 8, 1025)) == ps.PS_ERANGE
    missing = ps.make_grads([FAKE] * 3, ps.PS_BF16)
    assert _status(lambda: acc(spec, missing, FAKE, 1, 0, 8, 1024)) == ps.PS_EINVAL
    acc(spec, grads, FAKE, 1, 0, 0, 1024)                                            # empty range
    acc(spec, grads, FAKE, 1, 512, 512, 512)                                         # all padding


def test_accumulator_beside_the_contributions_is_for_the_update_only():
    """grads.accum: the sum of earlier micro-batches, taken by ps_step_update under pi_G = S."""
    spec, hp, shard, _ = _valid()
    upd = ps.ps_step_update
    with_acc = ps.make_grads([FAKE] * 4, ps.PS_BF16, accum=FAKE * 5)
    upd(spec, hp, shard, with_acc, 0, 0)                                             # valid, empty
    crooked = ps.make_grads([FAKE] * 4, ps.PS_BF16, accum=FAKE * 5 + 4)
    assert _status(lambda: upd(spec, hp, shard, crooked, 0, 8)) == ps.PS_EALIGN
    z1 = ps.ps_spec_preset("zero1", 4, 1, 4096)
    one = ps.make_grads([FAKE], ps.PS_BF16, accum=FAKE * 5)
    assert _status(lambda: upd(z1, hp, shard, one, 0, 8)) == ps.PS_EUNSUPPORTED
    assert "pi_G = R" in ps.ps_last_error()
    # nobody else takes it
    assert _status(lambda: ps.ps_step_accumulate(spec, with_acc, FAKE, 1, 0, 8, 1024)) == ps.PS_EUNSUPPORTED
    ws = ps.ps_workspace_bytes(8)
    assert _status(lambda: ps.ps_step_reduce_sumsq(spec, with_acc, 0.0, FAKE, FAKE, 0, FAKE, ws, 0, 8,
                                                   1024, 0)) == ps.PS_EUNSUPPORTED
    assert _status(lambda: ps.ps_step_reduce_sumsq_static(spec, with_acc, 0.0, FAKE, FAKE, 0, 0, 8,
                                                          1024, 0)) == ps.PS_EUNSUPPORTED
    off = ps.ps_spec_preset("zero_offload", 4, 0, 4096)
    assert _status(lambda: ps.ps_step_update_offloaded(off, hp, ps.ps_offload_plan_t(), with_acc)) \
        == ps.PS_EUNSUPPORTED


def test_zero2_output_offset_must_keep_alignment():
    spec = ps.ps_spec_preset("zero2", 4, 1, 4 * 1028)     # shard offset 1028, not a multiple of 8
    _, hp, _, grads = _valid()
    shard = ps.ps_shard_t(FAKE, FAKE, FAKE, FAKE, 1028, 1028)
    assert _status(lambda: ps.ps_step_update(spec, hp, shard, grads, 0, 8)) == ps.PS_EALIGN


def test_empty_ranges_are_ok_without_a_device():
    spec, hp, shard, grads = _valid()
    ps.ps_step_update(spec, hp, shard, grads, 0, 0)
    ps.ps_step_update(spec, hp, shard, grads, 1024, 0)
    pad_only = ps.ps_shard_t(FAKE, FAKE, FAKE, FAKE, 1024, 512)
    ps.ps_step_update(spec, hp, pad_only, grads, 512, 512)      # range lies entirely in the pad
    ps.ps_probe_copy(FAKE, FAKE * 2, 0)


def test_reduce_sumsq_rejects_bad_arguments():
    spec, _, _, grads = _valid()
    ws = ps.ps_workspace_bytes(8)
    assert ws >= 8 * 1024 and ps.ps_workspace_bytes(1 << 30) >= (1 << 30) // 128
    red = ps.ps_step_reduce_sumsq
    ok = dict(spec=spec, grads=grads, grad_scale=0.0, reduced_out=FAKE, sumsq_out=FAKE,
              accumulate=0, workspace=FAKE, workspace_bytes=ws, elem_offset=0, elem_count=8,
              valid_len=1024)
    assert _status(lambda: red(**dict(ok, spec=None))) == ps.PS_EINVAL
    assert _status(lambda: red(**dict(ok, grads=None))) == ps.PS_EINVAL
    assert _status(lambda: red(**dict(ok, sumsq_out=0))) == ps.PS_EINVAL
    assert _status(lambda: red(**dict(ok, workspace=0))) == ps.PS_EINVAL
    assert _status(lambda: red(**dict(ok, workspace_bytes=ws - 1))) == ps.PS_ERANGE
    assert _status(lambda: red(**dict(ok, sumsq_out=FAKE + 4))) == ps.PS_EALIGN
    assert _status(lambda: red(**dict(ok, reduced_out=FAKE + 8))) == ps.PS_EALIGN
    assert _status(lambda: red(**dict(ok, elem_offset=4))) == ps.PS_EALIGN
    assert _status(lambda: red(**dict(ok, elem_offset=1024, elem_count=8))) == ps.PS_ERANGE
    assert _status(lambda: red(**dict(ok, valid_len=1025))) == ps.PS_ERANGE
    assert _status(lambda: red(**dict(ok, grad_scale=float("nan")))) == ps.PS_ERANGE


def test_bucketed_rejects_bad_arguments():
    spec, hp, shard, _ = _valid()
    src = (C.c_void_p * 4)(*[FAKE] * 4)

    def plan(**kw):
        p = ps.ps_bucket_plan_t()
        p.source = C.cast(src, C.POINTER(C.c_void_p))
        p.n_contrib, p.dtype, p.bucket_elems, p.source_elems = 4, ps.PS_BF16, 256, 1024
        p.staging[0], p.staging[1] = FAKE * 2, FAKE * 3
        p.copy_stream, p.compute_stream = 0x100, 0x200
        for k, v in kw.items():
            if k == "staging":
                p.staging[0], p.staging[1] = v
            else:
                setattr(p, k, v)
        return p
    run = ps.ps_step_update_bucketed
    assert _status(lambda: run(spec, hp, shard, None)) == ps.PS_EINVAL
    assert _status(lambda: run(spec, hp, shard, plan(bucket_elems=0))) == ps.PS_EALIGN
    assert _status(lambda: run(spec, hp, shard, plan(bucket_elems=100))) == ps.PS_EALIGN
    assert _status(lambda: run(spec, hp, shard, plan(source_elems=0))) == ps.PS_ERANGE
    assert _status(lambda: run(spec, hp, shard, plan(source_elems=1000))) == ps.PS_EALIGN
    assert _status(lambda: run(spec, hp, shard, plan(copy_engine=4))) == ps.PS_EINVAL
    assert _status(lambda: run(spec, hp, shard, plan(copy_engine=ps.PS_COPY_NONE,
                                                       source_elems=1000))) == ps.PS_EALIGN
    assert _status(lambda: run(spec, hp, shard, plan(schedule=3))) == ps.PS_EINVAL
    assert _status(lambda: run(spec, hp, shard, plan(copy_engine=ps.PS_COPY_MEMCPY, bucket_elems=384,
                                                       source_elems=1024))) == ps.PS_EUNSUPPORTED
    assert _status(lambda: run(spec, hp, shard, plan(staging=(FAKE, FAKE)))) == ps.PS_EINVAL
    assert _status(lambda: run(spec, hp, shard, plan(staging=(FAKE, 0)))) == ps.PS_EINVAL
    assert _status(lambda: run(spec, hp, shard, plan(compute_stream=0x100))) == ps.PS_EINVAL
    assert _status(lambda: run(spec, hp, shard, plan(n_contrib=3))) == ps.PS_EINVAL
    ms = (C.c_float * 2)()
    assert _status(lambda: run(spec, hp, shard, plan(kernel_ms=ms, kernel_ms_len=2))) == ps.PS_ERANGE


def test_arena_rejects_bad_arguments():
    L = ps.library()
    out = C.c_void_p(1)
    eb = (C.c_uint32 * 3)(2, 4, 4)
    bad = (C.c_uint32 * 3)(2, 0, 4)
    run = lambda *a: L.ps_arena_create(*a)
    assert run(1 << 20, 1 << 20, None, 3, C.byref(out)) == ps.PS_EINVAL
    assert run(1 << 20, 1 << 20, eb, 3, None) == ps.PS_EINVAL
    assert run(1 << 20, 1 << 20, eb, 0, C.byref(out)) == ps.PS_ERANGE
    assert run(0, 1 << 20, eb, 3, C.byref(out)) == ps.PS_ERANGE
    assert run(1 << 20, 0, eb, 3, C.byref(out)) == ps.PS_ERANGE
    assert run(1 << 20, 1 << 20, bad, 3, C.byref(out)) == ps.PS_ERANGE
    assert run(1 << 20, (1 << 20) + 8, eb, 3, C.byref(out)) == ps.PS_EALIGN       # pieces not whole 2 MiB pages
    assert out.value is None                                                       # cleared on every refusal
    assert "2 MiB" in ps.ps_last_error()
    assert L.ps_arena_buffer(None, 0) is None and L.ps_arena_destroy(None) == ps.PS_OK


def test_offloaded_rejects_bad_arguments():
    spec = ps.ps_spec_preset("zero_offload", 4, 1, 4096)
    _, hp, _, grads = _valid()

    def plan(**kw):
        p = ps.ps_offload_plan_t()
        p.host_master, p.host_m, p.host_v, p.host_param_out = FAKE, FAKE * 2, FAKE * 3, FAKE * 4
        p.len, p.valid_len, p.bucket_elems, p.n_slots = 1024, 1024, 256, 3
        p.slot[0], p.slot[1], p.slot[2] = FAKE * 5, FAKE * 6, FAKE * 7
        p.h2d_stream, p.compute_stream, p.d2h_stream = 0x100, 0x200, 0x300
        for k, v in kw.items():
            if k.startswith("slot"):
                p.slot[int(k[4])] = v
            else:
                setattr(p, k, v)
        return p
    run = ps.ps_step_update_offloaded
    assert _status(lambda: run(spec, hp, None, grads)) == ps.PS_EINVAL
    assert _status(lambda: run(spec, hp, plan(), None)) == ps.PS_EINVAL
    z3 = ps.ps_spec_preset("zero3", 4, 1, 4096)
    assert _status(lambda: run(z3, hp, plan(), grads)) == ps.PS_EUNSUPPORTED
    assert _status(lambda: run(spec, hp, plan(host_m=0), grads)) == ps.PS_EINVAL
    assert _status(lambda: run(spec, hp, plan(n_slots=1), grads)) == ps.PS_EINVAL
    assert _status(lambda: run(spec, hp, plan(n_slots=4), grads)) == ps.PS_EINVAL
    assert _status(lambda: run(spec, hp, plan(slot1=0), grads)) == ps.PS_EINVAL
    assert _status(lambda: run(spec, hp, plan(slot1=FAKE * 5), grads)) == ps.PS_EINVAL
    assert _status(lambda: run(spec, hp, plan(slot2=FAKE * 7 + 8), grads)) == ps.PS_EALIGN
    assert _status(lambda: run(spec, hp, plan(bucket_elems=100), grads)) == ps.PS_EALIGN
    assert _status(lambda: run(spec, hp, plan(d2h_stream=0x100), grads)) == ps.PS_EINVAL
    assert _status(lambda: run(spec, hp, plan(len=1000), grads)) == ps.PS_ERANGE
    assert _status(lambda: run(spec, hp, plan(valid_len=1025), grads)) == ps.PS_ERANGE
    missing = ps.make_grads([FAKE] * 3, ps.PS_BF16)
    assert _status(lambda: run(spec, hp, plan(), missing)) == ps.PS_EINVAL
    run(spec, hp, plan(valid_len=0), grads)                       # nothing valid: no work, no device needed
    # the resident-state entry point refuses the offloaded placement
    shard = ps.ps_shard_t(FAKE, FAKE, FAKE, FAKE, 1024, 1024)
    assert _status(lambda: ps.ps_step_update(spec, hp, shard, grads, 0, 8)) == ps.PS_EUNSUPPORTED


def test_verification_calls_validation():
    ws = ps.ps_verify_workspace_bytes(4096)
    assert ws >= 2 * 1024 * 8
    d = ps.ps_verify_diff_sumsq
    assert _status(lambda: d(0, FAKE, ps.PS_F32, 8, FAKE, 0, FAKE, ws)) == ps.PS_EINVAL
    assert _status(lambda: d(FAKE, FAKE, 5, 8, FAKE, 0, FAKE, ws)) == ps.PS_EINVAL
    assert _status(lambda: d(FAKE, FAKE + 4, ps.PS_F32, 8, FAKE, 0, FAKE, ws)) == ps.PS_EALIGN
    assert _status(lambda: d(FAKE, FAKE, ps.PS_F32, 8, FAKE + 4, 0, FAKE, ws)) == ps.PS_EALIGN
    assert _status(lambda: d(FAKE, FAKE, ps.PS_F32, 1 << 30, FAKE, 0, FAKE, ws)) == ps.PS_ERANGE
    c = ps.ps_verify_checksum
    assert _status(lambda: c(0, 64, 0, FAKE, 0, FAKE, ws)) == ps.PS_EINVAL
    assert _status(lambda: c(FAKE, 60, 0, FAKE, 0, FAKE, ws)) == ps.PS_EALIGN
    assert _status(lambda: c(FAKE, 64, 0, FAKE + 2, 0, FAKE, ws)) == ps.PS_EALIGN
    assert _status(lambda: c(FAKE, 1 << 32, 0, FAKE, 0, FAKE, ws)) == ps.PS_ERANGE


def test_copy_probe_validation():
    assert _status(lambda: ps.ps_probe_copy(0, FAKE, 16)) == ps.PS_EINVAL
    assert _status(lambda: ps.ps_probe_copy(FAKE, FAKE + 8, 16)) == ps.PS_EALIGN
    assert _status(lambda: ps.ps_probe_copy(FAKE, FAKE, 24)) == ps.PS_EALIGN


@pytest.mark.skipif(torch.cuda.device_count() > 0, reason="a device is present")
def test_valid_calls_report_no_device():
    spec, hp, shard, grads = _valid()
    assert _status(lambda: ps.ps_step_update(spec, hp, shard, grads, 0, 1024)) == ps.PS_ENODEVICE
    assert _status(lambda: ps.ps_device_info()) == ps.PS_ENODEVICE
    assert _status(lambda: ps.ps_probe_copy(FAKE, FAKE * 2, 4096)) == ps.PS_ENODEVICE
    assert _status(lambda: ps.ps_step_reduce_sumsq(
        spec, grads, 0.0, FAKE, FAKE, 0, FAKE, ps.ps_workspace_bytes(8), 0, 8, 1024)) == ps.PS_ENODEVICE
    assert _status(lambda: ps.ps_step_reduce_sumsq_static(
        spec, grads, 0.0, FAKE, FAKE, 0, 0, 8, 1024)) == ps.PS_ENODEVICE
    # the bucket loop that reads in place needs no staging slots and no second stream, so
    # neither is checked: the otherwise valid call gets as far as looking for a device
    src = (C.c_void_p * 4)(*[FAKE] * 4)
    p = ps.ps_bucket_plan_t()
    p.source = C.cast(src, C.POINTER(C.c_void_p))
    p.n_contrib, p.dtype, p.bucket_elems, p.source_elems = 4, ps.PS_BF16, 256, 1024
    p.compute_stream, p.copy_engine = 0x200, ps.PS_COPY_NONE
    assert _status(lambda: ps.ps_step_update_bucketed(spec, hp, shard, p)) == ps.PS_ENODEVICE
    out = C.c_void_p()
    assert ps.library().ps_arena_create(1 << 20, 1 << 20, (C.c_uint32 * 2)(2, 4), 2,
                                        C.byref(out)) == ps.PS_ENODEVICE


def test_device_clip_coefficient_arguments():
    spec, _, shard, grads = _valid()
    upd = ps.ps_step_update
    hp = ps.ps_adamw_t(1e-4, 0.9, 0.999, 1e-8, 0.01, 1, 0.0, 0.0, FAKE + 2)
    assert _status(lambda: upd(spec, hp, shard, grads, 0, 8)) == ps.PS_EALIGN
    hp = ps.ps_adamw_t(1e-4, 0.9, 0.999, 1e-8, 0.01, 1, 0.0, 0.5, FAKE)
    assert _status(lambda: upd(spec, hp, shard, grads, 0, 8)) == ps.PS_EINVAL         # both given
    hp = ps.ps_adamw_t(1e-4, 0.9, 0.999, 1e-8, 0.01, 1, 0.0, 0.0, FAKE)
    upd(spec, hp, shard, grads, 0, 0)                                                 # valid, empty
    cc = ps.ps_step_clip_coef
    assert _status(lambda: cc(0, 0, 1.0, FAKE)) == ps.PS_EINVAL
    assert _status(lambda: cc(FAKE, 0, 1.0, 0)) == ps.PS_EINVAL
    assert _status(lambda: cc(FAKE + 4, 0, 1.0, FAKE)) == ps.PS_EALIGN
    assert _status(lambda: cc(FAKE, FAKE + 4, 1.0, FAKE)) == ps.PS_EALIGN
    assert _status(lambda: cc(FAKE, 0, 1.0, FAKE + 2)) == ps.PS_EALIGN


def test_parameter_format_must_match_16_bit_gradients():
    spec, hp, _, grads_bf16 = _valid()
    upd = ps.ps_step_update
    half = ps.ps_shard_t(FAKE, FAKE * 2, FAKE * 3, FAKE * 4, 1024, 1024, ps.PS_F16, 0)
    assert _status(lambda: upd(spec, hp, half, grads_bf16, 0, 8)) == ps.PS_EUNSUPPORTED   # bf16 grads, FP16 params
    g16 = ps.make_grads([FAKE * (5 + r) for r in range(4)], ps.PS_F16)
    upd(spec, hp, half, g16, 0, 0)                                                        # FP16 both: valid, empty
    bf = ps.ps_shard_t(FAKE, FAKE * 2, FAKE * 3, FAKE * 4, 1024, 1024)
    assert _status(lambda: upd(spec, hp, bf, g16, 0, 8)) == ps.PS_EUNSUPPORTED            # FP16 grads, bf16 params
    one32 = ps.make_grads([FAKE], ps.PS_F32)
    upd(spec, hp, half, one32, 0, 0)                                                      # FP32 gradient: either format
    upd(spec, hp, bf, one32, 0, 0)
    bad = ps.ps_shard_t(FAKE, FAKE * 2, FAKE * 3, FAKE * 4, 1024, 1024, ps.PS_F32, 0)
    assert _status(lambda: upd(spec, hp, bad, one32, 0, 8)) == ps.PS_EINVAL               # parameters are 16-bit
    bad = ps.ps_shard_t(FAKE, FAKE * 2, FAKE * 3, FAKE * 4, 1024, 1024, ps.PS_F16, 7)
    assert _status(lambda: upd(spec, hp, bad, one32, 0, 8)) == ps.PS_EINVAL               # reserved
    g_bad = ps.make_grads([FAKE * (5 + r) for r in range(4)], 3)
    assert _status(lambda: upd(spec, hp, bf, g_bad, 0, 8)) == ps.PS_EINVAL                # no such type

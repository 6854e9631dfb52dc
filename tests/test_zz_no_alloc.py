"""The reduce entry point that allocates nothing (partial sums in the library's static
device array) against the entry point that takes a caller workspace: same kernels, so
the mean is bit-identical and the sum of squares is the same double.  Two calls in a row
on one stream, the second over a smaller input, then a range in two pieces with the
accumulate flag, an empty valid range, and the size limit."""
import numpy as np
import pytest
import torch

import paper_2601_02311_amd as ps
from synth import host as gen

from gpu_util import dev, grads_of, host, stream_handle

pytestmark = pytest.mark.gpu

TILE = 256


def _both(spec, grads_np, dtype, n, valid, accumulate=False, pieces=None):
    """Returns ((mean, sumsq) of the workspace call, (mean, sumsq) of the static call)."""
    g_dev = [dev(g) for g in grads_np]
    out = []
    for static in (False, True):
        red = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
        ss = torch.full((1,), 3.0 if accumulate else -1.0, dtype=torch.float64, device="cuda")
        ws = torch.empty(ps.ps_workspace_bytes(n), dtype=torch.uint8, device="cuda")
        for j, (lo, cnt) in enumerate(pieces or [(0, n)]):
            acc = accumulate or j > 0
            g = grads_of(g_dev, dtype, lo)
            if static:
                ps.ps_step_reduce_sumsq_static(spec, g, 0.0, red.data_ptr(), ss.data_ptr(), acc,
                                               lo, cnt, valid, stream_handle())
            else:
                ps.ps_step_reduce_sumsq(spec, g, 0.0, red.data_ptr(), ss.data_ptr(), acc,
                                        ws.data_ptr(), ws.numel(), lo, cnt, valid, stream_handle())
        torch.cuda.synchronize()
        out.append((host(red), float(ss.item())))
    return out


def _same(a, b, valid):
    assert np.array_equal(a[0][:valid].view(np.uint32), b[0][:valid].view(np.uint32))
    assert np.isnan(a[0][valid:]).all() and np.isnan(b[0][valid:]).all()     # pad never written
    assert a[1] == b[1], "sum of squares differs: %r vs %r" % (a[1], b[1])


def test_static_reduce_equals_the_workspace_call_twice_in_a_row():
    N = 6
    big, small = 1500 * TILE + 1255, 37 * TILE + 13          # two-level sum, then a one-level one
    print("[case] no-alloc reduce: n=%d then n=%d, N=%d f32" % (big, small, N), flush=True)
    for n in (big, small):                                   # the second call is the smaller one
        valid = n - 101
        spec = ps.ps_spec_preset("zero3", N, N - 1, n * N)
        grads = [gen.gradient(n, 77, n & 7, r, "f32", std=1e-4, student_t_dof=3) for r in range(N)]
        ws_call, static_call = _both(spec, grads, "f32", n, valid)
        _same(ws_call, static_call, valid)
        assert static_call[1] > 0.0
    # bf16 contributions, the range in three pieces adding into a total that starts at 3.0
    n, N = 700 * TILE + 8, 8
    valid = n
    spec = ps.ps_spec_preset("zero3", N, 2, n * N)
    grads = [gen.gradient(n, 78, 0, r, "bf16", std=1e-3) for r in range(N)]
    b = (n // 3) // 8 * 8 + 8
    pieces = [(lo, min(b, n - lo)) for lo in range(0, n, b)]
    ws_call, static_call = _both(spec, grads, "bf16", n, valid, accumulate=True, pieces=pieces)
    _same(ws_call, static_call, valid)
    # nothing valid: the sum is exactly zero and nothing is written
    ws_call, static_call = _both(spec, grads, "bf16", n, 0)
    assert ws_call[1] == 0.0 and static_call[1] == 0.0 and np.isnan(static_call[0]).all()


def test_static_reduce_rejects_more_than_its_maximum():
    N = 2
    n = ps.PS_STATIC_MAX_ELEMS + 8
    spec = ps.ps_spec_preset("zero3", N, 0, n * N)
    ss = torch.zeros(1, dtype=torch.float64, device="cuda")
    one = torch.zeros(8, dtype=torch.float32, device="cuda")      # never read: the call is refused
    g = ps.make_grads([one.data_ptr(), one.data_ptr()], ps.PS_F32)
    with pytest.raises(ps.PsError) as e:
        ps.ps_step_reduce_sumsq_static(spec, g, 0.0, 0, ss.data_ptr(), 0, 0, n, n, stream_handle())
    assert e.value.status == ps.PS_ERANGE and "PS_STATIC_MAX_ELEMS" in e.value.detail
    torch.cuda.synchronize()
    assert float(ss.item()) == 0.0

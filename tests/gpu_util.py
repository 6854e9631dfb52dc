"""Helpers for the GPU tests: upload/download and thin call wrappers.  Imports the
GPU binding only; the oracle is imported by the tests themselves."""
import ctypes as C

import numpy as np
import torch

import paper_2601_02311_amd as ps

DT = {"bf16": ps.PS_BF16, "f32": ps.PS_F32, "f16": ps.PS_F16}


def dev(a):
    """numpy -> device tensor carrying the same bytes (uint16 travels as int16)."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda()
    return torch.from_numpy(a).cuda()


def host(t):
    """device tensor -> numpy with the original byte meaning (2-byte types -> uint16)."""
    t = t.detach()
    if t.dtype == torch.bfloat16:
        t = t.view(torch.int16)
    a = t.cpu().numpy()                      # float16 tensors come back as numpy float16
    return a.view(np.uint16) if a.dtype == np.int16 else a


def stream_handle(s=None):
    return (s or torch.cuda.current_stream()).cuda_stream


def hp_of(w=None, t=1, **kw):
    d = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)
    if w is not None:
        d = dict(lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, weight_decay=w.weight_decay)
    d.update({k: v for k, v in kw.items() if k in d})
    return d, ps.ps_adamw_t(d["lr"], d["beta1"], d["beta2"], d["eps"], d["weight_decay"], t,
                            kw.get("grad_scale", 0.0), kw.get("clip_coef", 0.0))


def shard_of(master, m, v, out, length, valid=None):
    """The parameter format follows the output tensor: float16 -> PS_F16, else bf16."""
    fmt = ps.PS_F16 if out.dtype == torch.float16 else ps.PS_BF16
    return ps.ps_shard_t(master.data_ptr(), m.data_ptr(), v.data_ptr(), out.data_ptr(), length,
                         length if valid is None else valid, fmt, 0)


def grads_of(tensors, dtype, elem_offset=0, accum=None):
    """accum: the FP32 accumulator tensor of earlier micro-batches (shard-based, no offset)."""
    esz = 4 if dtype == "f32" else 2
    return ps.make_grads([t.data_ptr() + elem_offset * esz for t in tensors], DT[dtype],
                         accum=None if accum is None else accum.data_ptr())


def ulp_diff(a, b):
    def key(x):
        i = np.ascontiguousarray(x, dtype=np.float32).view(np.int32).astype(np.int64)
        return np.where(i < 0, -(i & 0x7fffffff), i)
    return np.abs(key(a) - key(b))


def assert_state_parity(got, want, what=""):
    """got/want: (theta, m, v, p) numpy arrays.  master/m/v within 2 binary32 ulp of the
    oracle (NaNs must coincide); the 16-bit image bit-exact wherever theta' agrees."""
    for name, g, w in zip(("theta", "m", "v"), got[:3], want[:3]):
        gn, wn = np.isnan(g), np.isnan(w)
        assert np.array_equal(gn, wn), "%s %s: NaN pattern differs" % (what, name)
        d = ulp_diff(g[~gn], w[~wn])
        assert d.size == 0 or d.max() <= 2, "%s %s: max ulp %d" % (what, name, d.max())
    same = got[0].view(np.uint32) == want[0].view(np.uint32)
    gp, wp = got[3].view(np.uint16), want[3].view(np.uint16)         # bf16 bits or binary16, as bits
    assert np.array_equal(gp[same], wp[same]), "%s 16-bit image differs" % what
    return int((~same).sum())


class HostChunks:
    """Pinned host buffers, one per named array, reused from chunk to chunk."""

    def __init__(self, **specs):
        self.buf = {}
        for name, (numel, dtype) in specs.items():
            carrier = torch.int16 if dtype == torch.bfloat16 else dtype
            self.buf[name] = torch.empty(numel, dtype=carrier, pin_memory=True)

    def fetch(self, name, t):
        """Copy the device tensor t (at most the buffer's length) to the host; returns a numpy
        view of the pinned buffer with the original byte meaning (2-byte bit patterns as
        uint16, float16 as float16)."""
        k = t.numel()
        t = t.detach()
        if t.dtype == torch.bfloat16:
            t = t.view(torch.int16)
        dst = self.buf[name][:k]
        dst.copy_(t)                     # synchronous for pinned destinations on this stream
        torch.cuda.current_stream().synchronize()
        a = dst.numpy()
        return a.view(np.uint16) if a.dtype == np.int16 else a


def oracle_mismatches(step_f32, scalars, grads, pre, post, count, threads=16):
    """Runs the oracle's step over [0, count) of one chunk on `threads` host threads that
    share nothing (contiguous ranges; the update is elementwise) and counts, per array, the
    elements whose bits differ from what the device produced.  grads: contributions (host);
    pre: [theta, m, v] before the step, overwritten with the oracle's result; post: [theta,
    m, v, p] from the device.  Returns [bad_theta, bad_m, bad_v, bad_p]."""
    import threading
    p_want = np.zeros(pre[0].shape[0], post[3].dtype)
    bounds = [count * k // threads for k in range(threads + 1)]
    bad = [[0, 0, 0, 0] for _ in range(threads)]

    def work(k):
        lo, hi = bounds[k], bounds[k + 1]
        if hi <= lo:
            return
        step_f32(grads, scalars, pre[0], pre[1], pre[2], p_want, lo, hi)
        for j in range(3):
            bad[k][j] = int(np.count_nonzero(pre[j][lo:hi].view(np.uint32) != post[j][lo:hi].view(np.uint32)))
        bad[k][3] = int(np.count_nonzero(p_want[lo:hi].view(np.uint16) != post[3][lo:hi].view(np.uint16)))
    ts = [threading.Thread(target=work, args=(k,)) for k in range(threads)]
    for t in ts:
        t.start()
    for t in ts:
        t.join()
    return [sum(b[j] for b in bad) for j in range(4)]

"""Device-side (torch, ROCm) generators for the large workloads.

Buffers are filled in place, chunk by chunk, from a seeded ``torch.Generator``
so that no temporary larger than a chunk is ever alive.  bf16 data is stored
in ``torch.bfloat16`` tensors, binary16 in ``torch.float16``; the step library and the
oracle only ever see the raw bytes.
"""
import torch

CHUNK = 1 << 27

_TYPESTR = {torch.float32: "<f4", torch.int16: "<i2", torch.uint8: "|u1", torch.float16: "<f2",
            torch.float64: "<f8", torch.int64: "<i8"}


class _Foreign:
    """Device memory that torch did not allocate, described the way array libraries expect."""

    def __init__(self, ptr, numel, typestr):
        self.__cuda_array_interface__ = {"shape": (numel,), "typestr": typestr,
                                         "data": (int(ptr), False), "version": 2, "strides": None}


def as_tensor(ptr, numel, dtype):
    """A torch view (no copy) of `numel` elements of device memory at `ptr` that someone else
    owns and keeps alive (an arena of the step library).  bfloat16 travels as int16."""
    carrier = torch.int16 if dtype == torch.bfloat16 else dtype
    t = torch.as_tensor(_Foreign(ptr, numel, _TYPESTR[carrier]), device="cuda")
    return t.view(dtype)


def _gen(seed, *stream):
    g = torch.Generator(device="cuda")
    s = seed
    for x in stream:
        s = (s * 1_000_003 + int(x) + 1) % (2 ** 63 - 1)
    g.manual_seed(s)
    return g


def _normal_into_(c, std, g, absolute, square):
    """One chunk: c <- std * N(0,1) from generator g, optionally |.| or (.)^2."""
    c.normal_(0.0, std, generator=g)
    if absolute:
        c.abs_()
    if square:
        c.mul_(c)
    return c


def fill_normal_(t, std, seed, *stream, absolute=False, square=False):
    """t <- std * N(0,1), optionally |.| or (.)^2, chunked."""
    g = _gen(seed, *stream)
    n = t.numel()
    for lo in range(0, n, CHUNK):
        _normal_into_(t[lo:min(lo + CHUNK, n)], std, g, absolute, square)
    return t


def fill_gradient_(t, seed, step, replica, std=1e-3, outlier_frac=0.0, outlier_mult=1.0,
                   student_t_dof=0):
    """One device's gradient contribution (bf16 or fp32 tensor), in place."""
    g = _gen(seed, 4, step, replica)
    n = t.numel()
    for lo in range(0, n, CHUNK):
        c = t[lo:min(lo + CHUNK, n)]
        if student_t_dof > 0:
            z = torch.empty(c.numel(), dtype=torch.float32, device=t.device).normal_(generator=g)
            chi = torch.zeros_like(z)
            for _ in range(student_t_dof):
                w = torch.empty_like(z).normal_(generator=g)
                chi.addcmul_(w, w)
            z.div_(chi.div_(student_t_dof).sqrt_()).mul_(std)
            c.copy_(z)
            del z, chi, w
        else:
            c.normal_(0.0, std, generator=g)
        if outlier_frac > 0.0:
            mask = torch.empty(c.numel(), dtype=torch.float32, device=t.device).uniform_(generator=g)
            c.mul_(torch.where(mask < outlier_frac, outlier_mult, 1.0).to(c.dtype))
            del mask
    return t


def workload_state(w, n=None, into=None):
    """(master, m, v) fp32 device tensors of the workload's shard length; `into`: three
    tensors to fill instead of new ones."""
    n = w.shard_len if n is None else n
    master, m, v = into if into is not None else [torch.empty(n, dtype=torch.float32, device="cuda")
                                                  for _ in range(3)]
    fill_normal_(master, w.theta_std, w.seed, 1)
    if w.warm_moments:
        fill_normal_(m, 1e-3, w.seed, 2, absolute=True)
        fill_normal_(v, 1e-3, w.seed, 3, square=True)
    else:
        m.zero_()
        v.zero_()
    return master, m, v


def state_chunks(w, n=None):
    """The same values workload_state() writes, regenerated chunk by chunk: yields
    (lo, hi, master, m, v) with temporaries of at most CHUNK elements.  The generators are
    advanced exactly as fill_normal_ advances them, so the streams are identical."""
    n = w.shard_len if n is None else n
    gens = [_gen(w.seed, k) for k in (1, 2, 3)]
    for lo in range(0, n, CHUNK):
        hi = min(lo + CHUNK, n)
        th, m, v = [torch.empty(hi - lo, dtype=torch.float32, device="cuda") for _ in range(3)]
        _normal_into_(th, w.theta_std, gens[0], False, False)
        if w.warm_moments:
            _normal_into_(m, 1e-3, gens[1], True, False)
            _normal_into_(v, 1e-3, gens[2], False, True)
        else:
            m.zero_()
            v.zero_()
        yield lo, hi, th, m, v


def workload_gradients(w, step, n=None):
    n = w.shard_len if n is None else n
    dt = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}[w.grad_dtype]
    return [fill_gradient_(torch.empty(n, dtype=dt, device="cuda"), w.seed, step, r,
                           w.grad_std * w.loss_scale, w.outlier_frac, w.outlier_mult, w.student_t_dof)
            for r in range(w.n_devices)]

"""ctypes mirror of ``include/ps_step.h``.  Argument marshalling only.

Every function has the name and meaning of the C entry point it calls and
raises :class:`PsError` on a non-zero status.  There is no CPU fallback: if the
shared library is missing and cannot be built, importing fails.
"""
import ctypes as C
import os

# The caller's device buffers and streams come from PyTorch, so the library must
# bind to the HIP runtime instance PyTorch has loaded (same SONAME; whichever is
# loaded first serves both).  Importing torch first guarantees that order.
import torch  # noqa: F401

from . import build as _build

__all__ = [
    "PS_R", "PS_S", "PS_SG", "PS_M", "PS_O", "PS_BF16", "PS_F32", "PS_F16", "PS_MAX_CONTRIB", "PS_COPY_KERNEL", "PS_COPY_MEMCPY", "PS_COPY_NONE", "PS_COPY_REDUCE", "PS_SCHED_AUTO", "PS_SCHED_OVERLAP", "PS_SCHED_ALTERNATE", "PS_HOST_FLAT", "PS_HOST_PACKED",
    "PS_OK", "PS_EINVAL", "PS_EUNSUPPORTED", "PS_EALIGN", "PS_ERANGE", "PS_ENODEVICE", "PS_EHIP",
    "PsError", "ps_spec_t", "ps_cost_t", "ps_adamw_t", "ps_shard_t", "ps_grads_t",
    "ps_bucket_plan_t", "ps_offload_plan_t", "ps_device_info_t", "library", "library_path",
    "ps_abi_version", "ps_status_string", "ps_last_error", "ps_spec_preset", "ps_cost_eval",
    "ps_device_info", "ps_step_update", "ps_step_update_bucketed", "ps_workspace_bytes",
    "ps_step_reduce_sumsq", "ps_step_accumulate", "ps_probe_copy", "ps_clip_coef",
    "ps_verify_workspace_bytes", "ps_verify_diff_sumsq", "ps_verify_checksum",
    "ps_select_strategy", "ps_compose_index", "ps_compose_cost", "ps_step_update_offloaded",
    "ps_step_clip_coef", "ps_step_reduce_sumsq_static", "PS_STATIC_MAX_ELEMS",
    "ps_probe_set_update_residency", "ps_arena_create", "ps_arena_buffer", "ps_arena_destroy",
    "EXPORTED_SYMBOLS", "ABI_VERSION",
]

ABI_VERSION = 5   # PS_ABI_VERSION of include/ps_step.h this binding mirrors
PS_R, PS_S, PS_SG, PS_M, PS_O = range(5)
PS_BF16, PS_F32, PS_F16 = 0, 1, 2
PS_COPY_KERNEL, PS_COPY_MEMCPY, PS_COPY_NONE, PS_COPY_REDUCE = 0, 1, 2, 3
PS_SCHED_AUTO, PS_SCHED_OVERLAP, PS_SCHED_ALTERNATE = 0, 1, 2
PS_HOST_FLAT, PS_HOST_PACKED = 0, 1
PS_MAX_CONTRIB = 16
PS_STATIC_MAX_ELEMS = 1 << 30
(PS_OK, PS_EINVAL, PS_EUNSUPPORTED, PS_EALIGN, PS_ERANGE, PS_ENODEVICE, PS_EHIP) = range(7)

EXPORTED_SYMBOLS = (
    "ps_abi_version", "ps_status_string", "ps_last_error", "ps_spec_preset", "ps_cost_eval",
    "ps_device_info", "ps_step_update", "ps_step_update_bucketed", "ps_workspace_bytes",
    "ps_step_reduce_sumsq", "ps_step_accumulate", "ps_probe_copy", "ps_clip_coef",
    "ps_verify_workspace_bytes", "ps_verify_diff_sumsq", "ps_verify_checksum",
    "ps_select_strategy", "ps_compose_index", "ps_compose_cost", "ps_step_update_offloaded",
    "ps_step_clip_coef", "ps_step_reduce_sumsq_static", "ps_probe_set_update_residency",
    "ps_arena_create", "ps_arena_buffer", "ps_arena_destroy",
)


class PsError(RuntimeError):
    def __init__(self, status, text, detail):
        super().__init__("ps status %d (%s): %s" % (status, text, detail))
        self.status = status
        self.detail = detail


class ps_spec_t(C.Structure):
    _fields_ = [("theta", C.c_int32), ("omega", C.c_int32), ("grad", C.c_int32),
                ("act", C.c_int32), ("n_devices", C.c_uint32), ("shard_index", C.c_uint32),
                ("psi", C.c_uint64), ("align_elems", C.c_uint32), ("reserved", C.c_uint32),
                ("s_unit_bytes", C.c_uint64), ("act_bytes", C.c_uint64)]


class ps_cost_t(C.Structure):
    _fields_ = [("theta_bytes", C.c_uint64), ("omega_bytes", C.c_uint64),
                ("grad_bytes", C.c_uint64), ("act_bytes", C.c_uint64),
                ("transient_bytes", C.c_uint64), ("persistent_total", C.c_uint64),
                ("peak_total", C.c_uint64), ("comm_grad_sync_xN", C.c_uint64),
                ("comm_param_gather_xN", C.c_uint64), ("comm_total_bytes", C.c_double),
                ("implied_update_gather_xN", C.c_uint64), ("psi_padded", C.c_uint64),
                ("shard_offset", C.c_uint64), ("shard_len", C.c_uint64),
                ("valid_len", C.c_uint64)]


class ps_adamw_t(C.Structure):
    _fields_ = [("lr", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double),
                ("eps", C.c_double), ("weight_decay", C.c_double), ("step", C.c_uint64),
                ("grad_scale", C.c_double), ("clip_coef", C.c_double),
                ("clip_coef_device", C.c_void_p)]


class ps_shard_t(C.Structure):
    _fields_ = [("master", C.c_void_p), ("m", C.c_void_p), ("v", C.c_void_p),
                ("gather_out", C.c_void_p), ("len", C.c_uint64), ("valid_len", C.c_uint64),
                ("param_dtype", C.c_int32), ("reserved", C.c_int32)]


class ps_grads_t(C.Structure):
    _fields_ = [("contrib", C.POINTER(C.c_void_p)), ("n_contrib", C.c_uint32),
                ("dtype", C.c_int32), ("accum", C.c_void_p)]


class ps_bucket_plan_t(C.Structure):
    _fields_ = [("source", C.POINTER(C.c_void_p)), ("n_contrib", C.c_uint32),
                ("dtype", C.c_int32), ("bucket_elems", C.c_uint64),
                ("source_elems", C.c_uint64), ("staging", C.c_void_p * 2),
                ("copy_stream", C.c_void_p), ("compute_stream", C.c_void_p),
                ("copy_engine", C.c_int32), ("schedule", C.c_int32),
                ("kernel_ms", C.POINTER(C.c_float)), ("kernel_ms_len", C.c_uint64)]


class ps_offload_plan_t(C.Structure):
    _fields_ = [("host_master", C.c_void_p), ("host_m", C.c_void_p), ("host_v", C.c_void_p),
                ("host_param_out", C.c_void_p), ("len", C.c_uint64), ("valid_len", C.c_uint64),
                ("bucket_elems", C.c_uint64), ("n_slots", C.c_uint32), ("param_dtype", C.c_int32),
                ("slot", C.c_void_p * 3), ("h2d_stream", C.c_void_p),
                ("compute_stream", C.c_void_p), ("d2h_stream", C.c_void_p),
                ("host_layout", C.c_int32), ("reserved", C.c_int32), ("host_packed", C.c_void_p)]


class ps_device_info_t(C.Structure):
    _fields_ = [("name", C.c_char * 128), ("arch", C.c_char * 64),
                ("compute_units", C.c_int32), ("wavefront_size", C.c_int32),
                ("clock_khz", C.c_int32), ("memory_clock_khz", C.c_int32),
                ("memory_bus_bits", C.c_int32), ("l2_bytes", C.c_int32),
                ("total_bytes", C.c_uint64), ("free_bytes", C.c_uint64)]


_lib = None


def library_path():
    return _build.LIB


def library():
    """The loaded shared library.  A library that is missing, or that was built from other
    sources than the ones on disk (content hash recorded at build time), is rebuilt first;
    where that is impossible the import fails: a stale binary is never loaded silently."""
    global _lib
    if _lib is None:
        if _build.stale():
            if not os.path.exists(_build.HIPCC):
                raise ImportError("%s is missing or was built from other sources, and there is "
                                  "no %s to rebuild it" % (_build.LIB, _build.HIPCC))
            _build.build()
        L = C.CDLL(_build.LIB)
        L.ps_abi_version.restype = C.c_uint32
        L.ps_status_string.restype = C.c_char_p
        L.ps_status_string.argtypes = [C.c_int]
        L.ps_last_error.restype = C.c_char_p
        L.ps_spec_preset.restype = C.c_int
        L.ps_spec_preset.argtypes = [C.c_char_p, C.c_uint32, C.c_uint32, C.c_uint64,
                                     C.POINTER(ps_spec_t)]
        L.ps_cost_eval.restype = C.c_int
        L.ps_cost_eval.argtypes = [C.POINTER(ps_spec_t), C.POINTER(ps_cost_t)]
        L.ps_clip_coef.restype = C.c_double
        L.ps_clip_coef.argtypes = [C.c_double] * 3
        L.ps_select_strategy.restype = C.c_int
        L.ps_select_strategy.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint64, C.c_int32,
                                         C.POINTER(ps_spec_t), C.POINTER(C.c_int32),
                                         C.POINTER(C.c_int32)]
        L.ps_compose_index.restype = C.c_int
        L.ps_compose_index.argtypes = [C.c_uint32] * 3 + [C.POINTER(C.c_uint32)] * 4
        L.ps_step_clip_coef.restype = C.c_int
        L.ps_step_clip_coef.argtypes = [C.c_void_p, C.c_void_p, C.c_double, C.c_void_p, C.c_void_p]
        L.ps_compose_cost.restype = C.c_int
        L.ps_compose_cost.argtypes = [C.POINTER(ps_spec_t), C.c_uint32, C.POINTER(ps_cost_t)]
        L.ps_device_info.restype = C.c_int
        L.ps_device_info.argtypes = [C.POINTER(ps_device_info_t)]
        L.ps_step_update.restype = C.c_int
        L.ps_step_update.argtypes = [C.POINTER(ps_spec_t), C.POINTER(ps_adamw_t),
                                     C.POINTER(ps_shard_t), C.POINTER(ps_grads_t),
                                     C.c_uint64, C.c_uint64, C.c_void_p]
        L.ps_step_update_bucketed.restype = C.c_int
        L.ps_step_update_bucketed.argtypes = [C.POINTER(ps_spec_t), C.POINTER(ps_adamw_t),
                                              C.POINTER(ps_shard_t),
                                              C.POINTER(ps_bucket_plan_t)]
        L.ps_step_update_offloaded.restype = C.c_int
        L.ps_step_update_offloaded.argtypes = [C.POINTER(ps_spec_t), C.POINTER(ps_adamw_t),
                                               C.POINTER(ps_offload_plan_t),
                                               C.POINTER(ps_grads_t)]
        L.ps_workspace_bytes.restype = C.c_uint64
        L.ps_workspace_bytes.argtypes = [C.c_uint64]
        L.ps_step_reduce_sumsq.restype = C.c_int
        L.ps_step_reduce_sumsq.argtypes = [C.POINTER(ps_spec_t), C.POINTER(ps_grads_t),
                                           C.c_double, C.c_void_p, C.c_void_p, C.c_int32,
                                           C.c_void_p, C.c_uint64, C.c_uint64, C.c_uint64,
                                           C.c_uint64, C.c_void_p]
        L.ps_step_reduce_sumsq_static.restype = C.c_int
        L.ps_step_reduce_sumsq_static.argtypes = [C.POINTER(ps_spec_t), C.POINTER(ps_grads_t),
                                                  C.c_double, C.c_void_p, C.c_void_p, C.c_int32,
                                                  C.c_uint64, C.c_uint64, C.c_uint64, C.c_void_p]
        L.ps_step_accumulate.restype = C.c_int
        L.ps_step_accumulate.argtypes = [C.POINTER(ps_spec_t), C.POINTER(ps_grads_t), C.c_void_p,
                                         C.c_int32, C.c_uint64, C.c_uint64, C.c_uint64,
                                         C.c_void_p]
        L.ps_verify_workspace_bytes.restype = C.c_uint64
        L.ps_verify_workspace_bytes.argtypes = [C.c_uint64]
        L.ps_verify_diff_sumsq.restype = C.c_int
        L.ps_verify_diff_sumsq.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_uint64,
                                           C.c_void_p, C.c_int32, C.c_void_p, C.c_uint64,
                                           C.c_void_p]
        L.ps_verify_checksum.restype = C.c_int
        L.ps_verify_checksum.argtypes = [C.c_void_p, C.c_uint64, C.c_uint64, C.c_void_p, C.c_int32,
                                         C.c_void_p, C.c_uint64, C.c_void_p]
        L.ps_arena_create.restype = C.c_int
        L.ps_arena_create.argtypes = [C.c_uint64, C.c_uint64, C.POINTER(C.c_uint32), C.c_uint32,
                                      C.POINTER(C.c_void_p)]
        L.ps_arena_buffer.restype = C.c_void_p
        L.ps_arena_buffer.argtypes = [C.c_void_p, C.c_uint32]
        L.ps_arena_destroy.restype = C.c_int
        L.ps_arena_destroy.argtypes = [C.c_void_p]
        L.ps_probe_set_update_residency.restype = C.c_int
        L.ps_probe_set_update_residency.argtypes = [C.c_uint32]
        L.ps_probe_copy.restype = C.c_int
        L.ps_probe_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p]
        if L.ps_abi_version() != ABI_VERSION:
            raise ImportError("libps_step.so has ABI %d, binding wants %d" %
                              (L.ps_abi_version(), ABI_VERSION))
        _lib = L
    return _lib


def _check(status):
    if status != PS_OK:
        L = library()
        raise PsError(status, L.ps_status_string(status).decode(), L.ps_last_error().decode())


def _ptr_array(ptrs):
    return (C.c_void_p * len(ptrs))(*[int(p) for p in ptrs])


def _ref(x):
    return C.byref(x) if x is not None else None


def ps_abi_version():
    return library().ps_abi_version()


def ps_status_string(status):
    return library().ps_status_string(int(status)).decode()


def ps_last_error():
    return library().ps_last_error().decode()


def ps_spec_preset(name, n_devices, shard_index, psi, align_elems=0):
    spec = ps_spec_t()
    _check(library().ps_spec_preset(name.encode(), n_devices, shard_index, psi, C.byref(spec)))
    spec.align_elems = align_elems
    return spec


def ps_cost_eval(spec):
    cost = ps_cost_t()
    _check(library().ps_cost_eval(_ref(spec), C.byref(cost)))
    return cost


def ps_clip_coef(sumsq_local, sumsq_others, max_norm):
    return library().ps_clip_coef(sumsq_local, sumsq_others, max_norm)


def ps_select_strategy(psi, device_mem_bytes, n_devices, layer_bytes=0, fast_interconnect=False):
    """Returns (spec, fits, add_tp)."""
    spec, fits, tp = ps_spec_t(), C.c_int32(), C.c_int32()
    _check(library().ps_select_strategy(psi, device_mem_bytes, n_devices, layer_bytes,
                                        int(bool(fast_interconnect)), C.byref(spec),
                                        C.byref(fits), C.byref(tp)))
    return spec, bool(fits.value), bool(tp.value)


def ps_compose_index(inner, outer, device):
    """Returns (inner_group, inner_rank, outer_group, outer_rank)."""
    out = [C.c_uint32() for _ in range(4)]
    _check(library().ps_compose_index(inner, outer, device, *[C.byref(x) for x in out]))
    return tuple(x.value for x in out)


def ps_compose_cost(outer, inner):
    cost = ps_cost_t()
    _check(library().ps_compose_cost(_ref(outer), inner, C.byref(cost)))
    return cost


def ps_device_info():
    info = ps_device_info_t()
    _check(library().ps_device_info(C.byref(info)))
    return info


def make_grads(contrib_ptrs, dtype, accum=None):
    """Build a ps_grads_t; the pointer array is kept alive on the returned object.  accum:
    device address of the FP32 accumulator of earlier micro-batches (ps_step_update only)."""
    g = ps_grads_t()
    arr = _ptr_array(contrib_ptrs) if contrib_ptrs is not None else None
    g._keep = arr
    g.contrib = C.cast(arr, C.POINTER(C.c_void_p)) if arr is not None else None
    g.n_contrib = len(contrib_ptrs) if contrib_ptrs is not None else 0
    g.dtype = dtype
    g.accum = accum or None
    return g


def ps_step_update(spec, hp, shard, grads, elem_offset, elem_count, stream=0):
    _check(library().ps_step_update(_ref(spec), _ref(hp), _ref(shard), _ref(grads),
                                    elem_offset, elem_count, stream or None))


def ps_step_update_bucketed(spec, hp, shard, plan):
    _check(library().ps_step_update_bucketed(_ref(spec), _ref(hp), _ref(shard), _ref(plan)))


def ps_step_update_offloaded(spec, hp, plan, grads):
    _check(library().ps_step_update_offloaded(_ref(spec), _ref(hp), _ref(plan), _ref(grads)))


def ps_step_clip_coef(sumsq_local, sumsq_others, max_norm, coef_out, stream=0):
    _check(library().ps_step_clip_coef(sumsq_local or None, sumsq_others or None, max_norm,
                                       coef_out or None, stream or None))


def ps_workspace_bytes(elem_count):
    return library().ps_workspace_bytes(elem_count)


def ps_step_reduce_sumsq(spec, grads, grad_scale, reduced_out, sumsq_out, accumulate,
                         workspace, workspace_bytes, elem_offset, elem_count, valid_len,
                         stream=0):
    _check(library().ps_step_reduce_sumsq(_ref(spec), _ref(grads), grad_scale,
                                          reduced_out or None, sumsq_out or None,
                                          int(accumulate), workspace or None, workspace_bytes,
                                          elem_offset, elem_count, valid_len, stream or None))


def ps_step_reduce_sumsq_static(spec, grads, grad_scale, reduced_out, sumsq_out, accumulate,
                                elem_offset, elem_count, valid_len, stream=0):
    _check(library().ps_step_reduce_sumsq_static(_ref(spec), _ref(grads), grad_scale,
                                                 reduced_out or None, sumsq_out or None,
                                                 int(accumulate), elem_offset, elem_count,
                                                 valid_len, stream or None))


def ps_step_accumulate(spec, grads, accum, overwrite, elem_offset, elem_count, valid_len,
                       stream=0):
    _check(library().ps_step_accumulate(_ref(spec), _ref(grads), accum or None, int(overwrite),
                                        elem_offset, elem_count, valid_len, stream or None))


def ps_verify_workspace_bytes(buffer_bytes):
    return library().ps_verify_workspace_bytes(buffer_bytes)


def ps_verify_diff_sumsq(a, b, dtype, elem_count, out2, accumulate, workspace, workspace_bytes,
                         stream=0):
    _check(library().ps_verify_diff_sumsq(a or None, b or None, dtype, elem_count, out2 or None,
                                          int(accumulate), workspace or None, workspace_bytes,
                                          stream or None))


def ps_verify_checksum(buf, nbytes, first_word_index, out, accumulate, workspace, workspace_bytes,
                       stream=0):
    _check(library().ps_verify_checksum(buf or None, nbytes, first_word_index, out or None,
                                        int(accumulate), workspace or None, workspace_bytes,
                                        stream or None))


def ps_arena_create(length, chunk_elems, elem_bytes):
    """Returns the arena handle (an integer); buffers via ps_arena_buffer(handle, k)."""
    n = len(elem_bytes)
    arr = (C.c_uint32 * n)(*elem_bytes) if n else None
    out = C.c_void_p()
    _check(library().ps_arena_create(length, chunk_elems, arr, n, C.byref(out)))
    return out.value


def ps_arena_buffer(arena, k):
    return library().ps_arena_buffer(arena, k) or 0


def ps_arena_destroy(arena):
    _check(library().ps_arena_destroy(arena))


def ps_probe_set_update_residency(waves_per_cu):
    _check(library().ps_probe_set_update_residency(waves_per_cu))


def ps_probe_copy(dst, src, nbytes, stream=0):
    _check(library().ps_probe_copy(dst or None, src or None, nbytes, stream or None))


__all__ += ["make_grads"]

"""Host-side (numpy) generators for the small workloads and for test cases."""
import numpy as np
import torch


def _bf16_bits(x32: np.ndarray) -> np.ndarray:
    """Round float32 samples to bf16 with the library's own conversion and return
    the 16-bit patterns as uint16."""
    t = torch.from_numpy(np.ascontiguousarray(x32, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def rng_for(seed: int, *stream) -> np.random.Generator:
    return np.random.default_rng([seed, *stream])


def master(n, seed, std=0.02):
    return (rng_for(seed, 1).standard_normal(n, dtype=np.float32) * np.float32(std)).astype(np.float32)


def moments(n, seed, warm):
    if not warm:
        return np.zeros(n, np.float32), np.zeros(n, np.float32)
    m = np.abs(rng_for(seed, 2).standard_normal(n, dtype=np.float32) * np.float32(1e-3))
    v = (rng_for(seed, 3).standard_normal(n, dtype=np.float32) * np.float32(1e-3)) ** 2
    return m.astype(np.float32), v.astype(np.float32)


def gradient(n, seed, step, replica, dtype="bf16", std=1e-3, outlier_frac=0.0,
             outlier_mult=1.0, student_t_dof=0):
    """One device's gradient contribution for one step, as uint16 bf16 bits, float32, or
    float16 (dtype "f16": rounded to nearest, values past 65504 saturate to infinity as
    they would in an unscaled FP16 backward pass)."""
    r = rng_for(seed, 4, step, replica)
    if student_t_dof > 0:
        z = r.standard_normal(n)
        chi = r.chisquare(student_t_dof, n)
        x = (z / np.sqrt(chi / student_t_dof) * std).astype(np.float32)
    else:
        x = r.standard_normal(n, dtype=np.float32) * np.float32(std)
    if outlier_frac > 0.0:
        mask = r.random(n, dtype=np.float32) < outlier_frac
        x = np.where(mask, x * np.float32(outlier_mult), x).astype(np.float32)
    if dtype == "bf16":
        return _bf16_bits(x)
    if dtype == "f16":
        with np.errstate(over="ignore"):
            return np.ascontiguousarray(x.astype(np.float16))
    return np.ascontiguousarray(x, dtype=np.float32)


def workload_gradients(w, step, n=None):
    """All N contributions of workload ``w`` at ``step`` (full flat length unless n given)."""
    n = w.psi_padded if n is None else n
    return [gradient(n, w.seed, step, r, w.grad_dtype, w.grad_std * w.loss_scale, w.outlier_frac,
                     w.outlier_mult, w.student_t_dof) for r in range(w.n_devices)]

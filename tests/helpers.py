"""Shared test plumbing: moving bf16 bit patterns between numpy and the GPU, and
the parity rule. No arithmetic of the method lives here."""
import numpy as np


def to_gpu(bits):
    """uint16 bf16 bit patterns -> torch.bfloat16 tensor on cuda:0 (same bits)."""
    import torch
    a = np.ascontiguousarray(bits, dtype=np.uint16)
    return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).to("cuda:0")


def to_bits(t):
    """torch.bfloat16 tensor -> uint16 bit patterns on the host."""
    import torch
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


# |gpu - ref| <= 1e-2 * |ref| + 1e-3 per element, ref the unrounded fp64 oracle
# value, gpu the bf16 output decoded exactly. bf16 rounding alone costs up to
# 2^-8 = 0.39 % relative; fp32 accumulation adds ~1e-6.
RTOL = 1e-2
ATOL = 1e-3


def assert_parity(gpu_f64, ref_f64, what):
    gpu_f64 = np.asarray(gpu_f64, dtype=np.float64)
    ref_f64 = np.asarray(ref_f64, dtype=np.float64)
    assert gpu_f64.shape == ref_f64.shape, (what, gpu_f64.shape, ref_f64.shape)
    both_nan = np.isnan(gpu_f64) & np.isnan(ref_f64)
    same_inf = np.isinf(ref_f64) & (gpu_f64 == ref_f64)
    with np.errstate(invalid="ignore"):
        err = np.abs(gpu_f64 - ref_f64)
        ok = (err <= RTOL * np.abs(ref_f64) + ATOL) | both_nan | same_inf
    if not ok.all():
        bad = np.argwhere(~ok)
        i = tuple(bad[0])
        raise AssertionError("%s: %d of %d elements out of tolerance; first at %s: gpu=%r ref=%r"
                             % (what, len(bad), ok.size, i, gpu_f64[i], ref_f64[i]))

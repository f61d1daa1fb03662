"""Shared helpers of the parity tests: the error metric and device plumbing."""
import numpy as np

# Tolerance of the floating-point comparison (fp32 accumulation, fp16 output):
#   |y_gpu - y_ref| <= REL_TOL * max(|y_ref|, FLOOR_FRAC * rms(y_ref[m, :]))
# y_ref is the oracle's unrounded fp64 value.  The floor keeps the test well posed for
# outputs that cancel to almost zero, where a pure relative error is meaningless.
REL_TOL = 2e-3
FLOOR_FRAC = 1e-2


def rel_err(y_gpu, y_ref):
    """Largest |y_gpu - y_ref| / max(|y_ref|, FLOOR_FRAC * row rms).  y_gpu fp16, y_ref fp64."""
    yg = np.asarray(y_gpu).astype(np.float64)
    yr = np.asarray(y_ref, dtype=np.float64)
    assert yg.shape == yr.shape
    if yr.size == 0:
        return 0.0
    rms = np.sqrt(np.mean(yr * yr, axis=-1, keepdims=True))
    den = np.maximum(np.abs(yr), FLOOR_FRAC * rms)
    den = np.where(den == 0.0, 1.0, den)
    return float(np.max(np.abs(yg - yr) / den))


def assert_close(y_gpu, y_ref, what=""):
    assert np.all(np.isfinite(np.asarray(y_gpu).astype(np.float64))), f"{what}: non-finite output"
    e = rel_err(y_gpu, y_ref)
    assert e <= REL_TOL, f"{what}: max relative error {e:.3e} > {REL_TOL}"
    return e


def to_dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def dev_u32(a):
    """uint32 numpy -> device tensor (torch has no uint32 arithmetic; int32 view carries the bits)."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int32)).cuda()

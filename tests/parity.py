"""Shared helpers of the parity tests: the error metric and device plumbing."""
import numpy as np

# Tolerance of the floating-point comparison (fp32 accumulation, fp16 output):
#   |y_gpu - y_ref| <= REL_TOL * max(|y_ref|, floor_m)
#   floor_m = gamma * ACC_C * 2^-24 * sqrt(K) * ||x_m||_2 / REL_TOL
# y_ref is the oracle's unrounded fp64 value.  The first term is the stated bound on the
# relative error (fp16 rounding alone is 2^-11 = 4.9e-4).  The floor keeps the test well
# posed for outputs that cancel to almost zero: an fp32 accumulation of K terms of size
# |x_k| carries rounding noise of about 2^-24 sqrt(K) ||x||_2 whatever the weights are,
# and ACC_C = 4 allows four times that.  For the iid weights of the workloads (rms of a
# row of y is gamma * sqrt(0.6) * ||x||_2) the floor is 1e-2 of that rms at K = 4096.
REL_TOL = 2e-3
ACC_C = 4.0


def floors(x, gamma, K):
    """floor_m of the comment above, one per activation row, as a column vector."""
    xn = np.sqrt(np.sum(np.asarray(x).astype(np.float64) ** 2, axis=1, keepdims=True))
    return float(gamma) * ACC_C * 2.0 ** -24 * np.sqrt(K) * xn / REL_TOL


def rel_err(y_gpu, y_ref, x, gamma):
    """Largest |y_gpu - y_ref| / max(|y_ref|, floor_m).  y_gpu fp16, y_ref fp64, x fp16 [M][K]."""
    yg = np.asarray(y_gpu).astype(np.float64)
    yr = np.asarray(y_ref, dtype=np.float64)
    assert yg.shape == yr.shape
    if yr.size == 0:
        return 0.0
    den = np.maximum(np.abs(yr), floors(x, gamma, np.asarray(x).shape[1]))
    den = np.where(den == 0.0, 1.0, den)
    return float(np.max(np.abs(yg - yr) / den))


def assert_close(y_gpu, y_ref, x, gamma, what=""):
    assert np.all(np.isfinite(np.asarray(y_gpu).astype(np.float64))), f"{what}: non-finite output"
    e = rel_err(y_gpu, y_ref, x, gamma)
    assert e <= REL_TOL, f"{what}: max relative error {e:.3e} > {REL_TOL}"
    return e


def to_dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def dev_u32(a):
    """uint32 numpy -> device tensor (torch has no uint32 arithmetic; int32 view carries the bits)."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int32)).cuda()

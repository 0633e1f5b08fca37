"""Helpers for the GPU parity tests: device buffers for numpy inputs."""
import numpy as np
import torch


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def dev_params(params):
    return {k: dev(v) for k, v in params.items()}


def padded_matrix(W, pad_to=4):
    """Device copy of an int32 matrix with its row pitch rounded up to a multiple of four."""
    n, m = W.shape
    ld = (m + pad_to - 1) // pad_to * pad_to
    buf = torch.full((n, ld), -7, dtype=torch.int32, device="cuda")
    buf[:, :m] = dev(W)
    return buf


def empty_matrix(n, m, pad_to=4):
    ld = (m + pad_to - 1) // pad_to * pad_to
    return torch.full((n, ld), -7, dtype=torch.int32, device="cuda")


def weight_tolerance(scale):
    """Allowed difference between quantised weights whose scores agree to 1e-5 relative."""
    return int(np.ceil(1e-5 * scale)) + 1


def assert_weights_close(Wg, Wc, scale, feasible=None):
    """Quantised weights of two scorers whose scores agree to 1e-5 relative.

    For a large scale that is a difference of at most ceil(1e-5 * scale) + 1 levels.  With few
    levels (1e-5 * scale < 1) scores that close land on the same level except where the scaled score
    sits next to a rounding boundary: there the difference is exactly one level, and it may happen to
    at most one entry in a thousand (one entry of a matrix smaller than that; an error of 1e-5 relative moves under 2e-5 * scale of the
    entries across a boundary, 0.5 percent of that at 255 levels)."""
    a = np.asarray(Wg).astype(np.int64)
    b = np.asarray(Wc).astype(np.int64)
    if feasible is not None:
        a, b = a[feasible], b[feasible]
    diff = np.abs(a - b)
    if diff.size == 0:
        return
    if 1e-5 * scale >= 1.0:
        assert diff.max() <= weight_tolerance(scale), f"weight difference {diff.max()}"
    else:
        assert diff.max() <= 1, f"weight difference {diff.max()} at {scale:g} levels"
        assert (diff != 0).sum() <= max(1, int(1e-3 * diff.size)), f"{(diff != 0).mean():.2e} of the weights differ by a level"

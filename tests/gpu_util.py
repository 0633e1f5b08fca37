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

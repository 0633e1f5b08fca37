"""Seeded synthetic inputs shaped like a cluster scheduling round.

The paper's scheduler sees thousands of online and offline workloads per
cluster, each described by a handful of separately-profiled execution
features (Section "Matching-based scheduling"), and a trained predictor.
None of that data is public, so these generators stand in for it: feature
rows, predictor parameters and, for solver-only tests, integer weight
matrices.  They are handed unchanged to both the CPU checker and the GPU
library; nothing here evaluates the predictor or solves a matching.
"""
from dataclasses import dataclass

import numpy as np

from . import rng

INFEASIBLE = np.int32(-2147483648)


@dataclass(frozen=True)
class RoundConfig:
    name: str
    n: int            # online workloads (rows)
    m: int            # offline workloads (columns), n <= m
    F: int            # features per workload
    H: int            # hidden width of the predictor
    scale: float      # quantisation scale S: weights are integers in [0, S]
    features: str     # "uniform" or "mixture"
    masked: float     # target fraction of memory-infeasible pairs (None: leave as drawn)


CONFIGS = {
    "C1": RoundConfig("C1", 64, 64, 16, 64, float(2 ** 20), "uniform", None),
    "C2": RoundConfig("C2", 1024, 1024, 16, 64, float(2 ** 20), "uniform", 0.10),
    "C3": RoundConfig("C3", 4096, 8192, 32, 128, float(2 ** 24), "uniform", 0.25),
    "C4": RoundConfig("C4", 20000, 20000, 32, 128, float(2 ** 24), "mixture", 0.20),
    "C5": RoundConfig("C5", 20000, 40000, 32, 128, 255.0, "mixture", 0.90),
}


def uniform_features(seed, stream, rows, F):
    """rows x F float32 features, independent U[0,1)."""
    return rng.uniform24(seed, stream, rows * F).reshape(rows, F)


def mixture_features(seed, stream, rows, F, components=4):
    """rows x F float32 features from an equal-weight Gaussian mixture, clipped to [0,1].

    Component means are U(0.15,0.85) and standard deviations U(0.05,0.20) per
    feature, drawn from the seed; the number of components mirrors the four
    model families the paper names on each side of its testbed.
    """
    par = rng.uniform53(seed, rng.STREAM_MIXTURE, 2 * components * F, offset=stream * 2 * components * F)
    mu = 0.15 + 0.70 * par[: components * F].reshape(components, F)
    sd = 0.05 + 0.15 * par[components * F:].reshape(components, F)
    comp = rng.integers(seed, rng.STREAM_PERM, rows, components, offset=stream * rows)
    z = rng.normal(seed, stream, rows * F).reshape(rows, F)
    x = mu[comp] + sd[comp] * z
    return np.clip(x, 0.0, 1.0).astype(np.float32)


def _masked_fraction(a, b):
    """Approximate share of pairs with a_i + b_j > 1 (float64, sorting)."""
    bs = np.sort(b.astype(np.float64))
    over = len(bs) - np.searchsorted(bs, 1.0 - a.astype(np.float64), side="right")
    return float(over.sum()) / (len(a) * len(b))


def fit_memory_scale(x_on, x_off, target):
    """Rescale feature 0 (memory fraction) of both sides by one scalar c, clipped
    at 1, so that about `target` of all pairs exceed a combined memory of 1.
    Returns (x_on, x_off, c); the inputs are not modified."""
    a0, b0 = x_on[:, 0].astype(np.float64), x_off[:, 0].astype(np.float64)
    lo, hi = 0.0, 64.0
    for _ in range(60):
        c = 0.5 * (lo + hi)
        frac = _masked_fraction(np.minimum(1.0, c * a0), np.minimum(1.0, c * b0))
        if frac < target:
            lo = c
        else:
            hi = c
    c = 0.5 * (lo + hi)
    x_on, x_off = x_on.copy(), x_off.copy()
    x_on[:, 0] = np.minimum(1.0, c * a0).astype(np.float32)
    x_off[:, 0] = np.minimum(1.0, c * b0).astype(np.float32)
    return x_on, x_off, c


def predictor_params(seed, F, H):
    """Xavier-uniform weights (gain 1) and U(-0.1,0.1) biases for an MLP 2F -> H -> H -> 1.

    Returns a dict of float32 arrays: W1 [H,2F], b1 [H], W2 [H,H], b2 [H], W3 [H], b3 [1].
    """
    def xavier(stream, fan_out, fan_in):
        a = np.sqrt(6.0 / (fan_in + fan_out))
        u = rng.uniform53(seed, stream, fan_out * fan_in).reshape(fan_out, fan_in)
        return ((2.0 * u - 1.0) * a).astype(np.float32)

    def bias(stream, count):
        return ((2.0 * rng.uniform53(seed, stream, count) - 1.0) * 0.1).astype(np.float32)

    return {
        "W1": xavier(rng.STREAM_W1, H, 2 * F), "b1": bias(rng.STREAM_B1, H),
        "W2": xavier(rng.STREAM_W2, H, H), "b2": bias(rng.STREAM_B2, H),
        "W3": xavier(rng.STREAM_W3, 1, H).reshape(H), "b3": bias(rng.STREAM_B3, 1),
    }


def with_sm_input(params, seed):
    """The same predictor with one more input column for a pair-dependent SM share: W1 becomes
    [H, 2F + 1]; the new column is drawn like the others (Xavier-uniform for the wider layer)."""
    H, two_f = params["W1"].shape
    a = np.sqrt(6.0 / (two_f + 1 + H))
    col = ((2.0 * rng.uniform53(seed, rng.STREAM_SM, H) - 1.0) * a).astype(np.float32)
    out = dict(params)
    out["W1"] = np.ascontiguousarray(np.concatenate([params["W1"], col[:, None]], axis=1))
    return out


def with_slowdown_unit(params, seed):
    """The same predictor with a second output unit on the same hidden layers (the predicted
    slowdown of the online workload): W3slow [H], b3slow [1], drawn like W3 and b3."""
    H = params["W3"].shape[0]
    a = np.sqrt(6.0 / (H + 1))
    u = rng.uniform53(seed, rng.STREAM_SLOW, H + 1)
    out = dict(params)
    out["W3slow"] = ((2.0 * u[:H] - 1.0) * a).astype(np.float32)
    out["b3slow"] = ((2.0 * u[H:] - 1.0) * 0.1).astype(np.float32)
    return out


def gpu_types(seed, n, n_types):
    """GPU type of each online workload's device: type t has a share proportional to 1/(t+1)
    (a cluster holds a few GPU generations in uneven numbers).  Returns int32 [n]."""
    share = 1.0 / np.arange(1, n_types + 1)
    edges = np.cumsum(share / share.sum())
    u = rng.uniform53(seed, rng.STREAM_TYPE, n)
    return np.minimum(np.searchsorted(edges, u, side="right"), n_types - 1).astype(np.int32)


def typed_predictors(seed, F, hidden):
    """One predictor per GPU type, hidden[t] wide, drawn from seeds seed, seed + 1000, ..."""
    return [predictor_params(seed + 1000 * t, F, H) for t, H in enumerate(hidden)]


def scheduling_round(config, seed, n=None, m=None):
    """Feature matrices and predictor for one named configuration.

    `n`/`m` override the row counts (used for reduced-size parity cases that
    keep the configuration's feature law, widths and scale).
    Returns dict(x_on, x_off, params, cfg, mem_scale).
    """
    cfg = CONFIGS[config] if isinstance(config, str) else config
    n = cfg.n if n is None else n
    m = cfg.m if m is None else m
    draw = uniform_features if cfg.features == "uniform" else mixture_features
    x_on = draw(seed, rng.STREAM_X_ON, n, cfg.F)
    x_off = draw(seed, rng.STREAM_X_OFF, m, cfg.F)
    c = 1.0
    if cfg.masked is not None:
        x_on, x_off, c = fit_memory_scale(x_on, x_off, cfg.masked)
    return {"x_on": x_on, "x_off": x_off, "params": predictor_params(seed, cfg.F, cfg.H),
            "cfg": cfg, "mem_scale": c, "n": n, "m": m}


# ---------------------------------------------------------------- integer matrices

def uniform_matrix(seed, n, m, high, masked=0.0):
    """n x m int32 weights uniform in [0, high], each entry independently
    replaced by INFEASIBLE with probability `masked`."""
    w = rng.integers(seed, rng.STREAM_MATRIX, n * m, int(high) + 1).astype(np.int32).reshape(n, m)
    if masked > 0.0:
        hide = rng.uniform53(seed, rng.STREAM_MASK, n * m).reshape(n, m) < masked
        w[hide] = INFEASIBLE
    return w


def device_masked_matrix(seed, n, m, high, keep_one_in, device="cuda", pitch=None):
    """uniform_matrix for cluster-sized shapes, drawn on the device: an int32 torch tensor [n, pitch]
    (pitch >= m, default m rounded up to a multiple of four; padding columns hold -7) with weights
    uniform in [0, high], of which one entry in `keep_one_in`, chosen independently per entry, stays
    feasible.  Hundreds of millions of entries take minutes through the counter-based generator on
    the host; the framework's seeded device generator draws them in a blink, and whoever needs the
    matrix on the host copies it back, so both sides still see the same numbers."""
    import torch
    pitch = (m + 3) // 4 * 4 if pitch is None else pitch
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))
    out = torch.full((n, pitch), -7, dtype=torch.int32, device=device)
    step = max(1, (1 << 27) // max(m, 1))                       # about 128 M entries at a time
    for i0 in range(0, n, step):
        rows = min(step, n - i0)
        w = torch.randint(0, int(high) + 1, (rows, m), generator=gen, device=device, dtype=torch.int32)
        drop = torch.randint(0, int(keep_one_in), (rows, m), generator=gen, device=device, dtype=torch.int32) != 0
        w[drop] = int(INFEASIBLE)
        out[i0:i0 + rows, :m] = w
    return out


def permutation(seed, count, salt=0):
    """A seeded permutation of range(count)."""
    return np.argsort(rng.bits64(seed, rng.STREAM_PERM, count, offset=salt * count), kind="stable")


def planted_matrix(seed, n, m, high):
    """Background uniform in [0, high//2]; row i additionally holds `high` at a
    hidden distinct column.  Returns (W, hidden_columns)."""
    w = rng.integers(seed, rng.STREAM_MATRIX, n * m, int(high) // 2 + 1).astype(np.int32).reshape(n, m)
    cols = permutation(seed, m)[:n]
    w[np.arange(n), cols] = np.int32(high)
    return w, cols


def rank_one_matrix(seed, n, m, high):
    """W[i][j] = a[i] * b[j] with non-negative integer factors, a*b <= high.
    Returns (W, a, b)."""
    root = int(np.sqrt(high))
    a = rng.integers(seed, rng.STREAM_MATRIX, n, root + 1)
    b = rng.integers(seed, rng.STREAM_MASK, m, root + 1)
    return (a[:, None] * b[None, :]).astype(np.int32), a, b


def threshold_matrix(seed, n, m, levels, masked):
    """Few-level weights on a nested-neighbourhood feasibility pattern: entry
    (i,j) is feasible iff r_i + c_j <= t for seeded r, c in [0,1) and a
    threshold t chosen for the requested masked share.  Mirrors the structure
    of a memory-fit rule with heavy ties."""
    r = rng.uniform53(seed, rng.STREAM_X_ON, n)
    c = rng.uniform53(seed, rng.STREAM_X_OFF, m)
    lo, hi = 0.0, 2.0
    for _ in range(50):
        t = 0.5 * (lo + hi)
        frac = _masked_fraction(r / t if t > 0 else r * 1e9, c / t if t > 0 else c * 1e9)
        if frac > masked:
            lo = t
        else:
            hi = t
    t = 0.5 * (lo + hi)
    w = rng.integers(seed, rng.STREAM_MATRIX, n * m, int(levels)).astype(np.int32).reshape(n, m)
    w[(r[:, None] + c[None, :]) > t] = INFEASIBLE
    return w

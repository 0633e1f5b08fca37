"""Pins for the CPU checker's matching routines (no GPU).

Each test fixes the checker to something other than itself: the paper's worked
example, exhaustive enumeration, closed forms, a library routine used as a
black box, and linear-programming duality."""
import itertools
import os

import numpy as np
import pytest
from scipy.optimize import linear_sum_assignment

import synth

INF = synth.INFEASIBLE
GOLD = os.path.join(os.path.dirname(__file__), "golden", "worked_example.txt")


def _worked_example(scale):
    on, off, edges, plans = ["A", "B"], ["C", "D", "E"], [], {}
    for line in open(GOLD):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        if t[0] == "edge":
            edges.append((on.index(t[1]), off.index(t[2]), float(t[3])))
        elif t[0] == "plan":
            plans[int(t[1])] = ([tuple(p.split("-")) for p in t[2:-1]], float(t[-1]))
    W = np.full((2, 3), INF, np.int32)
    for i, j, x in edges:
        W[i, j] = int(np.rint(np.float32(x) * np.float32(scale)))
    return W, on, off, plans


def _python_enumeration(W):
    """Optimum by definition in pure Python: independent of the C enumeration."""
    n, m = W.shape
    best = 0
    for cols in itertools.product(range(-1, m), repeat=n):
        used = [c for c in cols if c >= 0]
        if len(set(used)) != len(used):
            continue
        if any(c >= 0 and W[i, c] == INF for i, c in enumerate(cols)):
            continue
        best = max(best, sum(int(W[i, c]) for i, c in enumerate(cols) if c >= 0))
    return best


@pytest.mark.parametrize("scale", [2 ** 20, 2 ** 24, 255])
def test_paper_worked_example(orc, scale):
    W, on, off, plans = _worked_example(scale)
    total, r2c, u, v = orc.max_weight_matching(W)
    # the paper's better plan: A with D, B with C
    assert [off[j] for j in r2c] == ["D", "C"]
    plan1 = sum(int(W[on.index(a), off.index(b)]) for a, b in plans[1][0])
    plan2 = sum(int(W[on.index(a), off.index(b)]) for a, b in plans[2][0])
    assert total == plan1 > plan2
    assert abs(plan1 / scale - plans[1][1]) < 2.0 / scale + 4e-3 * (scale == 255)
    assert abs(plan2 / scale - plans[2][1]) < 2.0 / scale + 4e-3 * (scale == 255)
    if scale == 2 ** 20:
        assert total == 1677722
    if scale == 2 ** 24:
        assert total == 26843546
    assert orc.brute_force(W)[0] == total
    assert orc.check_certificate(W, r2c, u, v, 1)[0] == 0


def test_enumeration_matches_pure_python(orc):
    for seed in range(60):
        n = 1 + seed % 4
        m = n + seed % 3
        W = synth.uniform_matrix(seed, n, m, 9, masked=0.35)
        assert orc.brute_force(W)[0] == _python_enumeration(W)


@pytest.mark.parametrize("high,masked", [(20, 0.0), (20, 0.4), (3, 0.2), (255, 0.9), (2 ** 24, 0.25), (0, 0.0)])
def test_matching_equals_enumeration(orc, high, masked):
    for seed in range(120):
        n = 1 + seed % 8
        m = min(8, n + seed % 4)
        W = synth.uniform_matrix(1000 + seed, n, m, high, masked)
        if seed % 10 == 0:
            W[seed % n, :] = INF                      # a row with no feasible column
        total, r2c, u, v = orc.max_weight_matching(W)
        bt, br = orc.brute_force(W)
        assert total == bt
        # the returned matching is valid and realises the total
        used = [c for c in r2c if c >= 0]
        assert len(set(used)) == len(used)
        assert all(W[i, c] != INF for i, c in enumerate(r2c) if c >= 0)
        assert sum(int(W[i, c]) for i, c in enumerate(r2c) if c >= 0) == total
        code, P, D = orc.check_certificate(W, r2c, u, v, 1)
        assert (code, P, D) == (0, total, total)


@pytest.mark.parametrize("n,m,high,masked", [(64, 64, 2 ** 20, 0.5), (200, 333, 2 ** 24, 0.25),
                                             (512, 512, 255, 0.9), (300, 1000, 7, 0.0)])
def test_matching_equals_library_assignment(orc, n, m, high, masked):
    W = synth.uniform_matrix(7, n, m, high, masked)
    total, r2c, u, v = orc.max_weight_matching(W)
    dense = np.where(W == INF, 0, W).astype(np.int64)
    ri, ci = linear_sum_assignment(dense, maximize=True)
    assert total == int(dense[ri, ci].sum())
    assert orc.check_certificate(W, r2c, u, v, 1) == (0, total, total)
    assert (u >= 0).all() and (v >= 0).all()
    free_cols = np.setdiff1d(np.arange(m), r2c[r2c >= 0])
    assert (v[free_cols] == 0).all()


def test_closed_forms(orc):
    n, m, S = 150, 220, 2 ** 20
    W, cols = synth.planted_matrix(3, n, m, S)
    total, r2c, _, _ = orc.max_weight_matching(W)
    assert total == n * S and (r2c == cols).all()

    W, a, b = synth.rank_one_matrix(4, n, m, S)
    expect = int((np.sort(a)[::-1] * np.sort(b)[::-1][:n]).sum())     # rearrangement inequality
    assert orc.max_weight_matching(W)[0] == expect

    assert orc.max_weight_matching(np.full((n, m), 77, np.int32))[0] == 77 * n
    total, r2c, u, v = orc.max_weight_matching(np.full((n, m), INF, np.int32))
    assert total == 0 and (r2c == -1).all() and not u.any() and not v.any()

    W = synth.uniform_matrix(5, n, m, S, 0.3)
    base = orc.max_weight_matching(W)[0]
    pr, pc = synth.permutation(5, n, 1), synth.permutation(5, m, 2)
    assert orc.max_weight_matching(np.ascontiguousarray(W[pr][:, pc]))[0] == base


def test_zero_weight_edge_versus_unmatched(orc):
    # a row whose only feasible entry is 0 may be matched or not; a row placed on an
    # infeasible entry must be reported unmatched
    W = np.array([[5, INF], [INF, INF]], np.int32)
    total, r2c, u, v = orc.max_weight_matching(W)
    assert total == 5 and r2c[0] == 0 and r2c[1] == -1


def test_certificate_rejects_planted_mistakes(orc):
    W = synth.uniform_matrix(11, 40, 60, 1000, 0.3)
    total, r2c, u, v = orc.max_weight_matching(W)
    assert orc.check_certificate(W, r2c, u, v, 1)[0] == 0
    # duplicate column
    bad = r2c.copy(); i, k = np.where(r2c >= 0)[0][:2]; bad[k] = bad[i]
    assert orc.check_certificate(W, bad, u, v, 1)[0] == 1
    # matched pair on an infeasible entry
    i = int(np.where(r2c >= 0)[0][0]); W2 = W.copy(); W2[i, r2c[i]] = INF
    assert orc.check_certificate(W2, r2c, u, v, 1)[0] == 2
    # negative dual
    un = u.copy(); un[0] = -1
    assert orc.check_certificate(W, r2c, un, v, 1)[0] == 3
    # an uncovered edge
    i = int(np.argmax(u)); ub = u.copy(); ub[i] -= 1
    assert orc.check_certificate(W, r2c, ub, v, 1)[0] == 4
    # a sub-optimal matching with valid duals leaves a gap
    sub = r2c.copy(); sub[int(np.where(r2c >= 0)[0][0])] = -1
    assert orc.check_certificate(W, sub, u, v, 1)[0] == 5
    # duals inflated beyond the gap allowance
    up = u.copy(); up[0] += 1
    assert orc.check_certificate(W, r2c, up, v, 1)[0] == 5


def test_certificate_scaled_duals(orc):
    # duals in units of 1/K: feasibility against K*w and a gap below K still prove optimality
    W = synth.uniform_matrix(12, 30, 45, 500, 0.2)
    total, r2c, u, v = orc.max_weight_matching(W)
    K = 31
    uk, vk = u * K, v * K
    assert orc.check_certificate(W, r2c, uk, vk, K) == (0, total, K * total)
    uk2 = uk.copy(); uk2[:K - 1] += 1                    # gap K-1: still a proof
    assert orc.check_certificate(W, r2c, uk2, vk, K)[0] == 0
    uk2[K - 1 if K - 1 < len(uk2) else 0] += 1            # gap K: no longer a proof
    assert orc.check_certificate(W, r2c, uk2, vk, K)[0] == 5


def test_rejects_more_rows_than_columns(orc):
    with pytest.raises(ValueError):
        orc.max_weight_matching(np.zeros((3, 2), np.int32))

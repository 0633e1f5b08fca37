"""GPU parity: mf_solve_assignment / mf_check_certificate / mf_schedule_round against the CPU checker.

The optimum weight is unique and must match bit for bit; which optimal matching is returned is
not unique, so the matching is checked for validity and the duals are re-verified on the host."""
import numpy as np
import pytest
import torch

import synth
from gpu_util import assert_weights_close, dev, dev_params, empty_matrix, padded_matrix, weight_tolerance

pytestmark = pytest.mark.gpu
INF = synth.INFEASIBLE


@pytest.fixture(scope="module")
def mm():
    import paper_2303_13803_amd as mm
    return mm


def _solve(mm, ctx, W):
    n, m = W.shape
    Wd = padded_matrix(W)
    r2c = torch.empty(n, dtype=torch.int32, device="cuda")
    u = torch.empty(n, dtype=torch.int64, device="cuda")
    v = torch.empty(m, dtype=torch.int64, device="cuda")
    res = ctx.solve_assignment(Wd, n, m, r2c, u, v)
    return res, r2c.cpu().numpy(), u.cpu().numpy(), v.cpu().numpy()


def _verify(orc, W, res, r2c, u, v, exact_total=None):
    n, m = W.shape
    assert res.cert_ok == 1 and res.K == min(n, m) + 1
    code, P, D = orc.check_certificate(W, r2c, u, v, res.K)       # host re-verification
    assert code == 0, f"host certificate check failed with code {code}"
    assert (P, D) == (res.primal, res.dual)
    assert res.matched == int((r2c >= 0).sum())
    assert res.min_reduced_cost >= 0
    assert res.fallbacks == 0, "a bounded wait ran out in a solve nothing was forced to give up in"
    if exact_total is not None:
        assert res.primal == exact_total


def test_paper_worked_example(mm, orc):
    W = np.full((2, 3), INF, np.int32)
    for i, j, x in [(0, 0, 0.3), (0, 1, 0.8), (1, 0, 0.8), (1, 2, 0.4)]:
        W[i, j] = int(np.rint(np.float32(x) * np.float32(2 ** 20)))
    ctx = mm.Context(2, 3)
    res, r2c, u, v = _solve(mm, ctx, W)
    _verify(orc, W, res, r2c, u, v, 1677722)
    assert list(r2c) == [1, 0]
    ctx.close()


def test_tiny_against_enumeration(mm, orc):
    ctx = mm.Context(8, 8)
    for seed in range(40):
        n = 1 + seed % 8
        m = min(8, n + seed % 3)
        W = synth.uniform_matrix(500 + seed, n, m, [9, 255, 2 ** 20][seed % 3], [0.0, 0.3, 0.7][seed % 3])
        if seed % 7 == 0:
            W[0, :] = INF
        res, r2c, u, v = _solve(mm, ctx, W)
        _verify(orc, W, res, r2c, u, v, orc.brute_force(W)[0])
    ctx.close()


@pytest.mark.parametrize("n,m,high,masked", [(64, 64, 2 ** 20, 0.5), (257, 300, 2 ** 24, 0.25),
                                             (1024, 1024, 2 ** 20, 0.1), (333, 1500, 255, 0.9),
                                             (500, 500, 3, 0.0), (700, 1201, 2 ** 24, 0.0)])
def test_uniform_matrices_against_exact_solver(mm, orc, n, m, high, masked):
    W = synth.uniform_matrix(21, n, m, high, masked)
    ctx = mm.Context(n, m)
    res, r2c, u, v = _solve(mm, ctx, W)
    _verify(orc, W, res, r2c, u, v, orc.max_weight_matching(W)[0])
    ctx.close()


def test_more_online_than_offline_workloads(mm, orc):
    """n > m: the optimum is that of the transposed matrix, which the exact solver can take."""
    ctx = mm.Context(8, 8)
    for seed in range(24):
        m = 1 + seed % 7
        n = min(8, m + 1 + seed % 3)
        W = synth.uniform_matrix(900 + seed, n, m, [9, 255, 2 ** 20][seed % 3], [0.0, 0.3, 0.7][seed % 3])
        res, r2c, u, v = _solve(mm, ctx, W)
        _verify(orc, W, res, r2c, u, v, orc.brute_force(np.ascontiguousarray(W.T))[0])
    ctx.close()
    for n, m, high, masked in [(300, 257, 2 ** 24, 0.25), (1500, 333, 255, 0.9), (1201, 700, 2 ** 24, 0.0),
                               (2100, 64, 2 ** 20, 0.5)]:
        W = synth.uniform_matrix(23, n, m, high, masked)
        ctx = mm.Context(n, m)
        res, r2c, u, v = _solve(mm, ctx, W)
        _verify(orc, W, res, r2c, u, v, orc.max_weight_matching(np.ascontiguousarray(W.T))[0])
        ctx.close()
    r = synth.scheduling_round("C3", 2, n=1024, m=512)              # scored, then matched, 2:1
    ctx = mm.Context(1024, 512)
    pred = ctx.predictor(dev_params(r["params"]), r["cfg"].scale)
    Wd = empty_matrix(1024, 512)
    r2c = torch.empty(1024, dtype=torch.int32, device="cuda")
    u = torch.empty(1024, dtype=torch.int64, device="cuda"); v = torch.empty(512, dtype=torch.int64, device="cuda")
    res = ctx.schedule_round(pred, dev(r["x_on"]), dev(r["x_off"]), Wd, r2c, u, v)
    W = Wd[:, :512].cpu().numpy()
    _verify(orc, W, res, r2c.cpu().numpy(), u.cpu().numpy(), v.cpu().numpy(),
            orc.max_weight_matching(np.ascontiguousarray(W.T))[0])
    ctx.close()


def test_largest_dimension_the_packed_words_allow(mm, orc):
    """m = 2^20 - 2 columns (holder ids fill the 20-bit field of a packed word), a few rows:
    scored, matched, certified; and the transposed shape, where the ids are the bidders'."""
    m = (1 << 20) - 2
    r = synth.scheduling_round("C2", 8, n=3, m=m)
    ctx = mm.Context(3, m)
    pred = ctx.predictor(dev_params(r["params"]), r["cfg"].scale)
    Wd = empty_matrix(3, m)
    r2c = torch.empty(3, dtype=torch.int32, device="cuda")
    u = torch.empty(3, dtype=torch.int64, device="cuda"); v = torch.empty(m, dtype=torch.int64, device="cuda")
    res = ctx.schedule_round(pred, dev(r["x_on"]), dev(r["x_off"]), Wd, r2c, u, v)
    W = Wd[:, :m].cpu().numpy()
    _, Wc = orc.score_pairs(r["x_on"], r["x_off"], r["params"], r["cfg"].scale)
    assert ((W == INF) == (Wc == INF)).all()
    ok = Wc != INF
    assert_weights_close(W, Wc, r["cfg"].scale, ok)
    _verify(orc, W, res, r2c.cpu().numpy(), u.cpu().numpy(), v.cpu().numpy(), orc.max_weight_matching(W)[0])
    ctx.close()
    Wt = np.ascontiguousarray(W.T)                                    # 1,048,574 rows x 3 columns
    ctx = mm.Context(m, 3)
    res, r2c, u, v = _solve(mm, ctx, Wt)
    _verify(orc, Wt, res, r2c, u, v, orc.max_weight_matching(W)[0])
    ctx.close()


def test_weights_at_the_edge_of_exact_arithmetic(mm, orc):
    """Duals are exact integers below 2^43: K * max W must stay under that.  8,000 rows with a
    weight of 2^30 still solve; 8,200 rows are refused with MF_ERR_RANGE rather than answered."""
    for n, fits in ((8000, True), (8200, False)):
        Wd = torch.zeros((n, n), dtype=torch.int32, device="cuda")
        Wd[5, 7] = 2 ** 30
        Wd[6, 7] = 2 ** 30 - 3
        Wd[5, 9] = 11
        ctx = mm.Context(n, n)
        r2c = torch.empty(n, dtype=torch.int32, device="cuda")
        u = torch.empty(n, dtype=torch.int64, device="cuda"); v = torch.empty(n, dtype=torch.int64, device="cuda")
        if fits:
            res = ctx.solve_assignment(Wd, n, n, r2c, u, v)
            assert res.cert_ok == 1 and res.primal == 2 ** 30 - 3 + 11 + 0      # rows 5 and 6 swap for 8 more
            code, P, D = orc.check_certificate(Wd.cpu().numpy(), r2c.cpu().numpy(), u.cpu().numpy(),
                                               v.cpu().numpy(), res.K)
            assert code == 0 and P == res.primal
        else:
            with pytest.raises(mm.MuxmatchError) as e:
                ctx.solve_assignment(Wd, n, n, r2c, u, v)
            assert e.value.code == mm.ERR_RANGE
        ctx.close()


def test_empty_problems_are_refused(mm):
    ctx = mm.Context(4, 4)
    W = torch.zeros((4, 4), dtype=torch.int32, device="cuda")
    r2c = torch.empty(4, dtype=torch.int32, device="cuda")
    u = torch.empty(4, dtype=torch.int64, device="cuda"); v = torch.empty(4, dtype=torch.int64, device="cuda")
    for n, m in ((0, 4), (4, 0), (0, 0)):
        with pytest.raises(mm.MuxmatchError) as e:
            ctx.solve_assignment(W, n, m, r2c, u, v)
        assert e.value.code == mm.ERR_ARG
    ctx.close()


def test_degenerate_matrices(mm, orc):
    ctx = mm.Context(300, 400)
    n, m, S = 300, 400, 2 ** 20
    W, cols = synth.planted_matrix(3, n, m, S)
    res, r2c, u, v = _solve(mm, ctx, W)
    _verify(orc, W, res, r2c, u, v, n * S)
    assert (r2c == cols).all()
    W, a, b = synth.rank_one_matrix(4, n, m, S)
    res, r2c, u, v = _solve(mm, ctx, W)
    _verify(orc, W, res, r2c, u, v, int((np.sort(a)[::-1] * np.sort(b)[::-1][:n]).sum()))
    W = np.full((n, m), 77, np.int32)                               # all equal
    res, r2c, u, v = _solve(mm, ctx, W)
    _verify(orc, W, res, r2c, u, v, 77 * n)
    W = np.full((n, m), INF, np.int32)                              # nothing feasible
    res, r2c, u, v = _solve(mm, ctx, W)
    _verify(orc, W, res, r2c, u, v, 0)
    assert (r2c == -1).all() and not u.any() and not v.any()
    W = np.zeros((n, m), np.int32)                                  # all zero
    res, r2c, u, v = _solve(mm, ctx, W)
    _verify(orc, W, res, r2c, u, v, 0)
    W = synth.threshold_matrix(5, n, m, 256, 0.9)                   # few levels, nested neighbourhoods
    res, r2c, u, v = _solve(mm, ctx, W)
    _verify(orc, W, res, r2c, u, v, orc.max_weight_matching(W)[0])
    ctx.close()


def test_certificate_entry_point(mm, orc):
    W = synth.uniform_matrix(31, 120, 200, 1000, 0.3)
    total, r2c, u, v = orc.max_weight_matching(W)          # the checker's own optimal duals, K = 1
    ctx = mm.Context(120, 200)
    Wd = padded_matrix(W)
    ok = ctx.check_certificate(Wd, 120, 200, dev(r2c), dev(u), dev(v), 1)
    assert ok.cert_ok == 1 and ok.primal == total and ok.dual == total and ok.min_reduced_cost == 0
    ub = u.copy(); ub[int(np.argmax(u))] -= 1              # uncovers an edge
    bad = ctx.check_certificate(Wd, 120, 200, dev(r2c), dev(ub), dev(v), 1)
    assert bad.cert_ok == 0 and bad.min_reduced_cost == -1
    dup = r2c.copy(); i, k = np.where(r2c >= 0)[0][:2]; dup[k] = dup[i]
    assert ctx.check_certificate(Wd, 120, 200, dev(dup), dev(u), dev(v), 1).cert_ok == 0
    sub = r2c.copy(); sub[int(np.where(r2c >= 0)[0][0])] = -1
    assert ctx.check_certificate(Wd, 120, 200, dev(sub), dev(u), dev(v), 1).cert_ok == 0
    neg = v.copy(); neg[0] = -1
    assert ctx.check_certificate(Wd, 120, 200, dev(r2c), dev(u), dev(neg), 1).cert_ok == 0
    ctx.close()
    # a ragged, several-loads-wide matrix; duals scaled by factors within and beyond 32 bits
    W = synth.uniform_matrix(32, 77, 4131, 2 ** 20, 0.4)
    total, r2c, u, v = orc.max_weight_matching(W)
    ctx = mm.Context(77, 4131)
    Wd = padded_matrix(W)
    for K in (1, 78, 2 ** 31 - 1, 2 ** 31, 2 ** 33 + 1):
        got = ctx.check_certificate(Wd, 77, 4131, dev(r2c), dev(u * K), dev(v * K), K)
        code, P, D = orc.check_certificate(W, r2c, u * K, v * K, K)
        assert code == 0 and got.cert_ok == 1 and (got.primal, got.dual) == (P, D) == (total, K * total)
        assert got.min_reduced_cost == 0
        short = u * K; short[int(np.argmax(u))] -= 3
        got = ctx.check_certificate(Wd, 77, 4131, dev(r2c), dev(short), dev(v * K), K)
        assert got.cert_ok == 0 and got.min_reduced_cost == -3
    ctx.close()


def test_argument_errors(mm):
    ctx = mm.Context(16, 16)
    W = padded_matrix(synth.uniform_matrix(1, 17, 17, 10))
    r2c = torch.empty(17, dtype=torch.int32, device="cuda")
    u = torch.empty(17, dtype=torch.int64, device="cuda"); v = torch.empty(17, dtype=torch.int64, device="cuda")
    with pytest.raises(mm.MuxmatchError) as e:
        ctx.solve_assignment(W, 17, 17, r2c, u, v)
    assert e.value.code == mm.ERR_SHAPE
    ctx.set_option("max_rounds", 1)
    Wok = padded_matrix(synth.uniform_matrix(1, 16, 16, 1000))
    with pytest.raises(mm.MuxmatchError) as e:
        ctx.solve_assignment(Wok, 16, 16, r2c, u, v)
    assert e.value.code == mm.ERR_NOT_CONVERGED
    ctx.close()


@pytest.mark.parametrize("prefix_below", [50, 101, 0])
@pytest.mark.parametrize("cfg,n,m,exact", [("C1", None, None, True), ("C2", None, None, True),
                                           ("C3", 512, 1024, True), ("C5", 400, 800, True),
                                           ("C5", 900, 350, True), ("C4", 300, 301, True)])
def test_schedule_round(mm, orc, cfg, n, m, exact, prefix_below):
    """prefix_below: share of pairs that can share GPU memory below which the matching runs on the
    context's memory-ordered copy of the matrix and reads only the feasible prefix of each line
    (101: always, 0: never, 50: the default); results come back in the caller's coordinates."""
    r = synth.scheduling_round(cfg, 1, n=n, m=m)
    n, m, S = r["n"], r["m"], r["cfg"].scale
    ctx = mm.Context(n, m)
    ctx.set_option("fit_prefix_below", prefix_below)
    pred = ctx.predictor(dev_params(r["params"]), S)
    W = empty_matrix(n, m)
    r2c = torch.empty(n, dtype=torch.int32, device="cuda")
    u = torch.empty(n, dtype=torch.int64, device="cuda"); v = torch.empty(m, dtype=torch.int64, device="cuda")
    res = ctx.schedule_round(pred, dev(r["x_on"]), dev(r["x_off"]), W, r2c, u, v)
    Wg = W.cpu().numpy()[:, :m].copy()
    # the scored matrix agrees with the checker's within the score tolerance, masks exactly
    _, Wc = orc.score_pairs(r["x_on"], r["x_off"], r["params"], S)
    assert ((Wg == INF) == (Wc == INF)).all()
    ok = Wc != INF
    assert_weights_close(Wg, Wc, S, ok)
    # the matching is optimal for the matrix the GPU scored: bit-exact total, host-verified duals
    exact_total = orc.max_weight_matching(Wg if n <= m else np.ascontiguousarray(Wg.T))[0] if exact else None
    _verify(orc, Wg, res, r2c.cpu().numpy(), u.cpu().numpy(), v.cpu().numpy(), exact_total)
    ctx.close()


@pytest.mark.parametrize("n,m,high,masked", [(2100, 2100, 2 ** 24, 0.9), (2048, 5000, 2 ** 20, 0.6), (2500, 3000, 255, 0.97),
                                             (2051, 2049, 2 ** 24, 0.999)])
def test_mostly_infeasible_matrix_is_matched_from_edge_lists(mm, orc, n, m, high, masked):
    """A matrix the caller brings, masked in no particular pattern: with few feasible pairs the rounds
    with many bidders read per-row lists of them (forced on here for a few thousand rows).  Same
    optimum as the exact solver, host-verified proof, and fewer bytes read than the rows hold."""
    W = synth.uniform_matrix(61, n, m, high, masked)
    W[5, :] = INF                                   # a row with no feasible pair: an empty list
    W[:, 7] = INF
    expect = orc.max_weight_matching(W if n <= m else np.ascontiguousarray(W.T))[0]
    scanned = {}
    for lists_from in (0, 1):
        ctx = mm.Context(n, m)
        ctx.set_option("edge_lists_from", lists_from)
        res, r2c, u, v = _solve(mm, ctx, W)
        _verify(orc, W, res, r2c, u, v, expect)
        scanned[lists_from] = res.bytes_scanned
        ctx.close()
    if n <= m:                                      # (with more rows than columns the transposed problem is solved, from its rows)
        assert scanned[1] < scanned[0]

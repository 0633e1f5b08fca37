"""GPU parity: mf_schedule_round_update (re-score what changed, warm-started matching) must give
exactly what a full round on the updated features gives."""
import numpy as np
import pytest
import torch

import synth
from gpu_util import assert_weights_close, dev, dev_params, empty_matrix, weight_tolerance

pytestmark = pytest.mark.gpu
INF = synth.INFEASIBLE


@pytest.fixture(scope="module")
def mm():
    import paper_2303_13803_amd as mm
    return mm


def _churn(r, seed, share):
    """Replace `share` of the online and of the offline workloads by fresh draws of the same law."""
    fresh = synth.scheduling_round(r["cfg"], seed, n=r["n"], m=r["m"])
    k_on = max(1, int(share * r["n"])); k_off = max(1, int(share * r["m"]))
    rows = np.sort(synth.permutation(seed, r["n"], 3)[:k_on]).astype(np.int32)
    cols = np.sort(synth.permutation(seed, r["m"], 4)[:k_off]).astype(np.int32)
    x_on, x_off = r["x_on"].copy(), r["x_off"].copy()
    x_on[rows] = fresh["x_on"][rows]; x_off[cols] = fresh["x_off"][cols]
    return x_on, x_off, rows, cols


@pytest.mark.parametrize("cfg,n,m,share,warm", [("C2", None, None, 0.03, 0), ("C3", 700, 1500, 0.05, 0),
                                                ("C5", 600, 1300, 0.02, 0), ("C1", None, None, 0.1, 0),
                                                ("C2", 512, 512, 0.03, 4096), ("C3", 300, 700, 0.05, 64)])
def test_update_round_equals_full_round(mm, orc, cfg, n, m, share, warm):
    r = synth.scheduling_round(cfg, 1, n=n, m=m)
    n, m, S = r["n"], r["m"], r["cfg"].scale
    ctx = mm.Context(n, m)
    ctx.set_option("warm_eps_units", warm)       # > 0: start the matching from the previous prices
    pred = ctx.predictor(dev_params(r["params"]), S)
    W = empty_matrix(n, m)
    r2c = torch.empty(n, dtype=torch.int32, device="cuda")
    u = torch.empty(n, dtype=torch.int64, device="cuda"); v = torch.empty(m, dtype=torch.int64, device="cuda")
    ctx.schedule_round(pred, dev(r["x_on"]), dev(r["x_off"]), W, r2c, u, v)
    W_before = W.cpu().numpy()[:, :m].copy()
    for step in range(3):                                    # three successive rounds of churn
        x_on, x_off, rows, cols = _churn(r, 100 + step, share)
        r["x_on"], r["x_off"] = x_on, x_off
        res = ctx.schedule_round_update(pred, dev(x_on), dev(x_off), dev(rows), dev(cols), W, r2c, u, v)
        Wg = W.cpu().numpy()[:, :m].copy()
        # what a full scoring of the new features gives, bit for bit (same kernel arithmetic per pair)
        W_full = empty_matrix(n, m)
        ctx.score_pairs(pred, dev(x_on), dev(x_off), W_full)
        assert (Wg == W_full.cpu().numpy()[:, :m]).all()
        # entries of unchanged pairs were not touched
        keep_r = np.setdiff1d(np.arange(n), rows); keep_c = np.setdiff1d(np.arange(m), cols)
        assert (Wg[np.ix_(keep_r, keep_c)] == W_before[np.ix_(keep_r, keep_c)]).all()
        # and the matching is the exact optimum of that matrix, with a certificate the host accepts
        assert res.cert_ok == 1 and res.primal == orc.max_weight_matching(Wg)[0]
        assert orc.check_certificate(Wg, r2c.cpu().numpy(), u.cpu().numpy(), v.cpu().numpy(), res.K)[0] == 0
        W_before = Wg
    # against the checker's scores, within the score tolerance
    _, Wc = orc.score_pairs(r["x_on"], r["x_off"], r["params"], S)
    ok = Wc != INF
    assert ((Wg == INF) == (Wc == INF)).all()
    assert_weights_close(Wg, Wc, S, ok)
    ctx.close()


def test_update_without_history_and_bad_lists(mm, orc):
    r = synth.scheduling_round("C1", 2)
    n, m, S = r["n"], r["m"], r["cfg"].scale
    ctx = mm.Context(n, m)
    pred = ctx.predictor(dev_params(r["params"]), S)
    W = empty_matrix(n, m)
    r2c = torch.empty(n, dtype=torch.int32, device="cuda")
    u = torch.empty(n, dtype=torch.int64, device="cuda"); v = torch.empty(m, dtype=torch.int64, device="cuda")
    x_on, x_off = dev(r["x_on"]), dev(r["x_off"])
    # no previous round on this context: every row listed, so the whole matrix is scored; full solve
    everything = dev(np.arange(n, dtype=np.int32))
    res = ctx.schedule_round_update(pred, x_on, x_off, everything, None, W, r2c, u, v)
    Wg = W.cpu().numpy()[:, :m]
    assert res.cert_ok == 1 and res.primal == orc.max_weight_matching(Wg)[0]
    # nothing changed: same optimum again, from the retained prices
    res2 = ctx.schedule_round_update(pred, x_on, x_off, None, None, W, r2c, u, v)
    assert res2.cert_ok == 1 and res2.primal == res.primal
    # an index outside the matrix is refused before any kernel uses it
    with pytest.raises(mm.MuxmatchError) as e:
        ctx.schedule_round_update(pred, x_on, x_off, dev(np.array([0, n], np.int32)), None, W, r2c, u, v)
    assert e.value.code == mm.ERR_ARG
    with pytest.raises(mm.MuxmatchError) as e:
        ctx.schedule_round_update(pred, x_on, x_off, None, dev(np.array([-1], np.int32)), W, r2c, u, v)
    assert e.value.code == mm.ERR_ARG
    ctx.close()


def test_update_round_at_cluster_scale(mm, orc):
    r = synth.scheduling_round("C4", 1)
    n, m, S = r["n"], r["m"], r["cfg"].scale
    ctx = mm.Context(n, m)
    pred = ctx.predictor(dev_params(r["params"]), S)
    W = torch.empty((n, m), dtype=torch.int32, device="cuda")
    r2c = torch.empty(n, dtype=torch.int32, device="cuda")
    u = torch.empty(n, dtype=torch.int64, device="cuda"); v = torch.empty(m, dtype=torch.int64, device="cuda")
    ctx.schedule_round(pred, dev(r["x_on"]), dev(r["x_off"]), W, r2c, u, v)
    x_on, x_off, rows, cols = _churn(r, 77, 0.02)
    res = ctx.schedule_round_update(pred, dev(x_on), dev(x_off), dev(rows), dev(cols), W, r2c, u, v)
    Wg = W.cpu().numpy()
    assert res.cert_ok == 1
    code, P, D = orc.check_certificate(Wg, r2c.cpu().numpy(), u.cpu().numpy(), v.cpu().numpy(), res.K)
    assert code == 0 and (P, D) == (res.primal, res.dual)
    # re-scored rows agree with the checker
    _, Wr = orc.score_pairs(x_on[rows[:32]], x_off, r["params"], S)
    ok = Wr != INF
    assert ((Wg[rows[:32]] == INF) == (Wr == INF)).all()
    assert_weights_close(Wg[rows[:32]], Wr, S, ok)
    ctx.close()

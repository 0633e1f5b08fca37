"""GPU parity: the second output unit of the predictor (predicted slowdown of the online workload)
and the limit that makes pairs above it infeasible."""
import numpy as np
import pytest
import torch

import synth
from gpu_util import assert_weights_close, dev, empty_matrix

pytestmark = pytest.mark.gpu
INF = synth.INFEASIBLE
SM = (2, 3)


@pytest.fixture(scope="module")
def mm():
    import paper_2303_13803_amd as mm
    return mm


def _device_params(full, with_sm):
    p = {k: dev(v) for k, v in full.items() if k != "W1"}
    if with_sm:
        p["W1"] = dev(full["W1"][:, :-1]); p["W1sm"] = dev(full["W1"][:, -1])
    else:
        p["W1"] = dev(full["W1"])
    return p


@pytest.mark.parametrize("cfg,n,m,with_sm,limit", [("C1", None, None, False, 0.5), ("C3", 150, 700, False, 0.45),
                                                   ("C4", 97, 1031, True, 0.55), ("C5", 257, 300, True, 0.5),
                                                   ("C2", 3, 5, False, 0.5), ("C4", 300, 333, False, 0.0),
                                                   ("C4", 300, 333, False, 1.0)])
def test_slowdown_mask_matches_checker(mm, orc, cfg, n, m, with_sm, limit):
    r = synth.scheduling_round(cfg, 5, n=n, m=m)
    n, m, S = r["n"], r["m"], r["cfg"].scale
    full = synth.with_sm_input(r["params"], 12) if with_sm else r["params"]
    full = synth.with_slowdown_unit(full, 13)
    full["W3slow"] *= 3.0                                       # spread the predictions around the limit
    sm = SM if with_sm else None
    sig, W = orc.score_pairs(r["x_on"], r["x_off"], full, S, sm=sm, slow_limit=limit)
    unit = {k: v for k, v in full.items() if k not in ("W3slow", "b3slow")}
    sig_plain, W_plain = orc.score_pairs(r["x_on"], r["x_off"], unit, S, sm=sm)
    unit["W3"], unit["b3"] = full["W3slow"], full["b3slow"]
    slow_ref = orc.score_pairs(r["x_on"], r["x_off"], unit, S, sm=sm)[0].astype(np.float64)
    if 0.0 < limit < 1.0:
        assert (slow_ref > limit).any() and (slow_ref <= limit).any()      # otherwise the case proves nothing

    ctx = mm.Context(n, m)
    p = _device_params(full, with_sm)
    pred = ctx.predictor(p, S, sm=sm, slow_limit=limit)
    x_on, x_off = dev(r["x_on"]), dev(r["x_off"])
    Wd = empty_matrix(n, m); sg = torch.empty((n, m), dtype=torch.float32, device="cuda")
    ctx.score_pairs(pred, x_on, x_off, Wd, sg)
    # the library's own prediction of the slowdown: the unit scored as if it were the main output
    q = dict(p); q["W3"], q["b3"] = p["W3slow"], p["b3slow"]
    Ws = empty_matrix(n, m); slow_gpu = torch.empty((n, m), dtype=torch.float32, device="cuda")
    ctx.score_pairs(ctx.predictor(q, S, sm=sm), x_on, x_off, Ws, slow_gpu)
    torch.cuda.synchronize()
    Wg = Wd.cpu().numpy()[:, :m]
    slow_gpu = slow_gpu.cpu().numpy()

    rel = np.abs(sg.cpu().numpy().astype(np.float64) - sig) / sig
    assert rel.max() <= 1e-5, f"score relative error {rel.max():.3e}"       # scores are written for every pair
    assert (np.abs(slow_gpu - slow_ref) <= 1e-5 * slow_ref).all()
    # a float decides a bit: both sides take the decision in float32, and they may differ only
    # where the prediction is within the scores' tolerance of the limit
    by_memory = W_plain == INF
    mask_gpu = Wg == INF
    assert (mask_gpu == (by_memory | (slow_gpu > np.float32(limit)))).all(), "mask is not the library's own prediction"
    clear = np.abs(slow_ref - limit) > 1e-5 * slow_ref
    assert ((mask_gpu == (W == INF)) | ~clear).all(), "mask bits differ away from the limit"
    assert (~clear).mean() < 1e-3
    both = ~mask_gpu & (W != INF)
    assert_weights_close(Wg, W, S, both)
    Wd2 = empty_matrix(n, m)                                    # weights only: memory order, skipping
    ctx.score_pairs(pred, x_on, x_off, Wd2)
    torch.cuda.synchronize()
    assert (Wd2.cpu().numpy()[:, :m] == Wg).all()
    ctx.close()


def test_round_with_slowdown_limit_and_argument_errors(mm, orc):
    r = synth.scheduling_round("C3", 6, n=300, m=640)
    n, m, S = r["n"], r["m"], r["cfg"].scale
    full = synth.with_slowdown_unit(r["params"], 7); full["W3slow"] *= 3.0
    ctx = mm.Context(n, m)
    p = _device_params(full, False)
    pred = ctx.predictor(p, S, slow_limit=0.5)
    W = empty_matrix(n, m)
    r2c = torch.empty(n, dtype=torch.int32, device="cuda")
    u = torch.empty(n, dtype=torch.int64, device="cuda"); v = torch.empty(m, dtype=torch.int64, device="cuda")
    res = ctx.schedule_round(pred, dev(r["x_on"]), dev(r["x_off"]), W, r2c, u, v)
    Wg = W.cpu().numpy()[:, :m]
    plain = empty_matrix(n, m)
    ctx.score_pairs(ctx.predictor(p, S), dev(r["x_on"]), dev(r["x_off"]), plain)
    torch.cuda.synchronize()
    plain = plain.cpu().numpy()[:, :m]
    assert ((Wg == INF) & (plain != INF)).sum() > n            # the limit removed pairs the memory mask kept
    assert (Wg[Wg != INF] == plain[Wg != INF]).all()
    # the matching is the exact optimum of the matrix the library built, and avoids the removed pairs
    code, P, D = orc.check_certificate(Wg, r2c.cpu().numpy(), u.cpu().numpy(), v.cpu().numpy(), res.K)
    assert code == 0 and res.cert_ok == 1 and res.fallbacks == 0
    assert res.primal == orc.max_weight_matching(Wg)[0]
    cols = r2c.cpu().numpy()
    assert (Wg[np.nonzero(cols >= 0)[0], cols[cols >= 0]] != INF).all()
    # a unit without its bias, a limit that is not a number
    q = dict(p)
    bad = ctx.predictor(q, S, slow_limit=float("nan"))
    with pytest.raises(mm.MuxmatchError) as e:
        ctx.score_pairs(bad, dev(r["x_on"]), dev(r["x_off"]), W)
    assert e.value.code == mm.ERR_ARG
    ctx.close()

"""GPU parity: the pair-dependent SM share as a third predictor input (d_W1sm)."""
import numpy as np
import pytest
import torch

import synth
from gpu_util import assert_weights_close, dev, empty_matrix, weight_tolerance

pytestmark = pytest.mark.gpu
INF = synth.INFEASIBLE
SM = (2, 3)            # online feature 2: SM activity; offline feature 3: SM share it can use


@pytest.fixture(scope="module")
def mm():
    import paper_2303_13803_amd as mm
    return mm


def _device_predictor(ctx, full, scale):
    """The checker holds W1 as [H, 2F+1]; the library takes W1 [H, 2F] and the last column apart."""
    p = {k: dev(v) for k, v in full.items() if k != "W1"}
    p["W1"] = dev(full["W1"][:, :-1])
    p["W1sm"] = dev(full["W1"][:, -1])
    return ctx.predictor(p, scale, sm=SM)


@pytest.mark.parametrize("cfg,n,m", [("C1", None, None), ("C3", 150, 700), ("C4", 97, 1031), ("C5", 257, 300),
                                     ("C2", 3, 5)])
def test_scores_with_sm_input_match_checker(mm, orc, cfg, n, m):
    r = synth.scheduling_round(cfg, 2, n=n, m=m)
    n, m, S = r["n"], r["m"], r["cfg"].scale
    full = synth.with_sm_input(r["params"], 11)
    full["W1"][:, -1] *= 4.0                      # make the new input matter
    sig, W = orc.score_pairs(r["x_on"], r["x_off"], full, S, sm=SM)
    plain = orc.score_pairs(r["x_on"], r["x_off"], r["params"], S)[0]
    assert np.abs(sig - plain).max() > 1e-3       # otherwise the case proves nothing
    ctx = mm.Context(n, m)
    pred = _device_predictor(ctx, full, S)
    x_on, x_off = dev(r["x_on"]), dev(r["x_off"])
    Wd = empty_matrix(n, m); sg = torch.empty((n, m), dtype=torch.float32, device="cuda")
    ctx.score_pairs(pred, x_on, x_off, Wd, sg)
    torch.cuda.synchronize()
    Wg = Wd.cpu().numpy()[:, :m]
    assert ((Wg == INF) == (W == INF)).all(), "mask bits differ"
    rel = np.abs(sg.cpu().numpy().astype(np.float64) - sig) / sig
    assert rel.max() <= 1e-5, f"score relative error {rel.max():.3e}"
    ok = W != INF
    assert_weights_close(Wg, W, S, ok)
    Wd2 = empty_matrix(n, m)                       # weights only: memory order, skipping
    ctx.score_pairs(pred, x_on, x_off, Wd2)
    torch.cuda.synchronize()
    assert (Wd2.cpu().numpy()[:, :m] == Wg).all()
    ctx.close()


def test_round_with_sm_input_and_argument_errors(mm, orc):
    r = synth.scheduling_round("C3", 4, n=300, m=640)
    n, m, S = r["n"], r["m"], r["cfg"].scale
    full = synth.with_sm_input(r["params"], 5)
    ctx = mm.Context(n, m)
    pred = _device_predictor(ctx, full, S)
    W = empty_matrix(n, m)
    r2c = torch.empty(n, dtype=torch.int32, device="cuda")
    u = torch.empty(n, dtype=torch.int64, device="cuda"); v = torch.empty(m, dtype=torch.int64, device="cuda")
    res = ctx.schedule_round(pred, dev(r["x_on"]), dev(r["x_off"]), W, r2c, u, v)
    Wg = W.cpu().numpy()[:, :m]
    _, Wc = orc.score_pairs(r["x_on"], r["x_off"], full, S, sm=SM)
    assert ((Wg == INF) == (Wc == INF)).all()
    okm = Wc != INF
    assert_weights_close(Wg, Wc, S, okm)
    assert res.cert_ok == 1 and res.primal == orc.max_weight_matching(Wg)[0]
    # a feature index outside [0, F)
    p = {k: dev(val) for k, val in full.items() if k != "W1"}
    p["W1"] = dev(full["W1"][:, :-1]); p["W1sm"] = dev(full["W1"][:, -1])
    bad = ctx.predictor(p, S, sm=(2, r["cfg"].F))
    with pytest.raises(mm.MuxmatchError) as e:
        ctx.score_pairs(bad, dev(r["x_on"]), dev(r["x_off"]), W)
    assert e.value.code == mm.ERR_ARG
    ctx.close()

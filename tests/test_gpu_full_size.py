"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

C3 is small enough for the exact CPU solver; at C4 and C5 the optimum is proved by re-checking the
device's dual certificate on the host in O(n m), and the scorer is compared on sampled rows and
columns (every mask bit is compared)."""
import numpy as np
import pytest
import torch

import synth
from gpu_util import dev, dev_params, weight_tolerance

pytestmark = pytest.mark.gpu
INF = synth.INFEASIBLE


@pytest.fixture(scope="module")
def mm():
    import paper_2303_13803_amd as mm
    return mm


def _round(mm, cfg_name, seed):
    r = synth.scheduling_round(cfg_name, seed)
    n, m, S = r["n"], r["m"], r["cfg"].scale
    ctx = mm.Context(n, m)
    pred = ctx.predictor(dev_params(r["params"]), S)
    ld = (m + 3) // 4 * 4
    W = torch.empty((n, ld), dtype=torch.int32, device="cuda")
    r2c = torch.empty(n, dtype=torch.int32, device="cuda")
    u = torch.empty(n, dtype=torch.int64, device="cuda")
    v = torch.empty(m, dtype=torch.int64, device="cuda")
    res = ctx.schedule_round(pred, dev(r["x_on"]), dev(r["x_off"]), W, r2c, u, v)
    Wg = W.cpu().numpy()[:, :m]
    out = (r, res, np.ascontiguousarray(Wg), r2c.cpu().numpy(), u.cpu().numpy(), v.cpu().numpy())
    ctx.close()
    del W
    torch.cuda.empty_cache()
    return out


def _check_scores_sampled(orc, r, Wg, rows, cols):
    S = r["cfg"].scale
    tol = weight_tolerance(S)
    # every mask bit, by the rule itself (one float32 addition), block by block
    a, b = r["x_on"][:, 0], r["x_off"][:, 0]
    for i0 in range(0, r["n"], 2048):
        masked = (a[i0:i0 + 2048, None] + b[None, :]) > np.float32(1.0)
        assert ((Wg[i0:i0 + 2048] == INF) == masked).all()
    # sampled rows x all columns, all rows x sampled columns
    _, Wr = orc.score_pairs(r["x_on"][rows], r["x_off"], r["params"], S)
    ok = Wr != INF
    assert np.abs(Wg[rows][ok].astype(np.int64) - Wr[ok]).max() <= tol
    _, Wc = orc.score_pairs(r["x_on"], r["x_off"][cols], r["params"], S)
    ok = Wc != INF
    assert np.abs(Wg[:, cols][ok].astype(np.int64) - Wc[ok]).max() <= tol
    return float((Wg == INF).mean())


def _check_certificate(orc, Wg, res, r2c, u, v):
    n = Wg.shape[0]
    assert res.cert_ok == 1 and res.K == n + 1
    code, P, D = orc.check_certificate(Wg, r2c, u, v, res.K)
    assert code == 0, f"host certificate check failed with code {code}"
    assert (P, D) == (res.primal, res.dual)
    assert 0 <= D - res.K * P < res.K
    assert res.matched == int((r2c >= 0).sum())


def test_c3_full_size_exact(mm, orc):
    r, res, Wg, r2c, u, v = _round(mm, "C3", 1)
    rows = synth.permutation(7, r["n"])[:96]
    cols = synth.permutation(8, r["m"])[:48]
    masked = _check_scores_sampled(orc, r, Wg, rows, cols)
    assert abs(masked - 0.25) < 0.01
    _check_certificate(orc, Wg, res, r2c, u, v)
    assert res.primal == orc.max_weight_matching(Wg)[0]          # bit-exact optimum


@pytest.mark.parametrize("cfg,target", [("C4", 0.20), ("C5", 0.90)])
def test_cluster_scale_round(mm, orc, cfg, target):
    r, res, Wg, r2c, u, v = _round(mm, cfg, 1)
    rows = synth.permutation(7, r["n"])[:48]
    cols = synth.permutation(8, r["m"])[:48]
    masked = _check_scores_sampled(orc, r, Wg, rows, cols)
    assert abs(masked - target) < 0.01
    _check_certificate(orc, Wg, res, r2c, u, v)
    if cfg == "C5":
        assert set(np.unique(Wg[Wg != INF]).tolist()) <= set(range(256))   # few-level weights


def test_cluster_scale_round_with_unmatched_workloads(mm, orc):
    """Seed 7 of the C4 recipe leaves online workloads without a partner at the optimum (too few
    offline workloads fit beside them): rows rest, columns stay unused but priced, and the second
    side of the auction runs in every phase, also in those that end early.  Same contract: the
    host re-checks the proof of optimality."""
    r, res, Wg, r2c, u, v = _round(mm, "C4", 7)
    _check_certificate(orc, Wg, res, r2c, u, v)
    assert res.matched < r["n"], "the instance no longer exercises the second side"

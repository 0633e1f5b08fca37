"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

C3 is small enough for the exact CPU solver; at C4 and C5 the optimum is proved by re-checking the
device's dual certificate on the host in O(n m), and the scorer is compared on sampled rows and
columns (every mask bit is compared)."""
import numpy as np
import pytest
import torch

import synth
from gpu_util import assert_weights_close, dev, dev_params

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
    # every mask bit, by the rule itself (one float32 addition), block by block
    a, b = r["x_on"][:, 0], r["x_off"][:, 0]
    for i0 in range(0, r["n"], 2048):
        masked = (a[i0:i0 + 2048, None] + b[None, :]) > np.float32(1.0)
        assert ((Wg[i0:i0 + 2048] == INF) == masked).all()
    # sampled rows x all columns, all rows x sampled columns
    _, Wr = orc.score_pairs(r["x_on"][rows], r["x_off"], r["params"], S)
    assert_weights_close(Wg[rows], Wr, S, Wr != INF)
    _, Wc = orc.score_pairs(r["x_on"], r["x_off"][cols], r["params"], S)
    assert_weights_close(Wg[:, cols], Wc, S, Wc != INF)
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
    cols = synth.permutation(8, r["m"])[:64]
    masked = _check_scores_sampled(orc, r, Wg, rows, cols)
    assert abs(masked - 0.25) < 0.01
    _check_certificate(orc, Wg, res, r2c, u, v)
    assert res.primal == orc.max_weight_matching(Wg)[0]          # bit-exact optimum


@pytest.mark.parametrize("cfg,seed,target", [("C4", 1, 0.20), ("C5", 1, 0.90), ("C5", 2, 0.90)])
def test_cluster_scale_round(mm, orc, cfg, seed, target):
    r, res, Wg, r2c, u, v = _round(mm, cfg, seed)
    rows = synth.permutation(7 + seed, r["n"])[:64]
    cols = synth.permutation(8 + seed, r["m"])[:64]
    masked = _check_scores_sampled(orc, r, Wg, rows, cols)
    assert abs(masked - target) < 0.01
    _check_certificate(orc, Wg, res, r2c, u, v)
    if cfg == "C5":
        assert set(np.unique(Wg[Wg != INF]).tolist()) <= set(range(256))   # few-level weights


@pytest.mark.parametrize("seed", [7, 12])
def test_cluster_scale_round_with_unmatched_workloads(mm, orc, seed):
    """Seeds 7 and 12 of the C4 recipe leave online workloads without a partner at the optimum (too
    few offline workloads fit beside them): rows rest, columns stay unused but priced, and the
    second side of the auction runs in every phase, also in those that end early.  Same contract:
    the host re-checks the proof of optimality."""
    r, res, Wg, r2c, u, v = _round(mm, "C4", seed)
    _check_certificate(orc, Wg, res, r2c, u, v)
    assert res.matched < r["n"], "the instance no longer exercises the second side"


def _mask_bits_agree(r, Wg):
    a, b = r["x_on"][:, 0], r["x_off"][:, 0]
    for i0 in range(0, r["n"], 2048):
        masked = (a[i0:i0 + 2048, None] + b[None, :]) > np.float32(1.0)
        assert ((Wg[i0:i0 + 2048] == INF) == masked).all()


def test_cluster_scale_scoring_with_one_predictor_per_gpu_type(mm, orc):
    """The typed scoring pass bench.py times (C4, three GPU types): sampled rows and columns against
    the checker's per-row choice of predictor, every mask bit against the rule itself."""
    r = synth.scheduling_round("C4", 1)
    n, m, S = r["n"], r["m"], r["cfg"].scale
    plist = synth.typed_predictors(1 + 7, r["cfg"].F, [r["cfg"].H] * 3)
    types = synth.gpu_types(1, n, 3)
    ctx = mm.Context(n, m)
    preds = [ctx.predictor(dev_params(p), S) for p in plist]
    W = torch.empty((n, (m + 3) // 4 * 4), dtype=torch.int32, device="cuda")
    ctx.score_pairs_typed(preds, dev(types), dev(r["x_on"]), dev(r["x_off"]), W)
    torch.cuda.synchronize()
    Wg = W.cpu().numpy()[:, :m]
    ctx.close()
    _mask_bits_agree(r, Wg)
    rows = np.sort(synth.permutation(17, n)[:64])
    assert len(set(types[rows].tolist())) == 3, "the sample misses a GPU type"
    _, Wr = orc.score_pairs_typed(r["x_on"][rows], r["x_off"], plist, types[rows], S)
    assert_weights_close(Wg[rows], Wr, S, Wr != INF)
    cols = np.sort(synth.permutation(18, m)[:64])
    _, Wc = orc.score_pairs_typed(r["x_on"], r["x_off"][cols], plist, types, S)
    assert_weights_close(Wg[:, cols], Wc, S, Wc != INF)


def test_cluster_scale_scoring_with_the_pair_dependent_sm_input(mm, orc):
    """The scoring pass with the third predictor input that bench.py times (C4): sampled rows and
    columns against the checker, every mask bit against the rule itself."""
    sm = (2, 3)                                   # as in bench.py: online SM activity, offline SM share
    r = synth.scheduling_round("C4", 1)
    n, m, S = r["n"], r["m"], r["cfg"].scale
    full = synth.with_sm_input(r["params"], 1 + 3)
    p = {k: dev(v) for k, v in full.items() if k != "W1"}
    p["W1"] = dev(full["W1"][:, :-1]); p["W1sm"] = dev(full["W1"][:, -1])
    ctx = mm.Context(n, m)
    pred = ctx.predictor(p, S, sm=sm)
    W = torch.empty((n, (m + 3) // 4 * 4), dtype=torch.int32, device="cuda")
    ctx.score_pairs(pred, dev(r["x_on"]), dev(r["x_off"]), W)
    torch.cuda.synchronize()
    Wg = W.cpu().numpy()[:, :m]
    ctx.close()
    _mask_bits_agree(r, Wg)
    rows = np.sort(synth.permutation(19, n)[:64])
    _, Wr = orc.score_pairs(r["x_on"][rows], r["x_off"], full, S, sm=sm)
    assert_weights_close(Wg[rows], Wr, S, Wr != INF)
    cols = np.sort(synth.permutation(20, m)[:64])
    _, Wc = orc.score_pairs(r["x_on"], r["x_off"][cols], full, S, sm=sm)
    assert_weights_close(Wg[:, cols], Wc, S, Wc != INF)


def test_cluster_scale_matrix_with_an_arbitrary_mask(mm, orc):
    """20,000 x 40,000 weights of which one pair in ten, in no pattern at all, may share: the caller
    brings the matrix, the rounds with many bidders read per-row lists of the feasible pairs, and
    the host re-checks the proof of optimality on the whole matrix."""
    n, m = 20000, 40000
    W = synth.device_masked_matrix(9, n, m, 2 ** 24, 10)
    ctx = mm.Context(n, m)
    r2c = torch.empty(n, dtype=torch.int32, device="cuda")
    u = torch.empty(n, dtype=torch.int64, device="cuda")
    v = torch.empty(m, dtype=torch.int64, device="cuda")
    res = ctx.solve_assignment(W, n, m, r2c, u, v)
    dense_bytes_of_first_rounds = 4.0 * n * m * res.phases
    assert res.bytes_scanned < dense_bytes_of_first_rounds, "the rounds did not read the lists"
    Wh = np.ascontiguousarray(W[:, :m].cpu().numpy())
    ctx.close()
    del W
    torch.cuda.empty_cache()
    assert abs((Wh == INF).mean() - 0.9) < 0.002
    _check_certificate(orc, Wh, res, r2c.cpu().numpy(), u.cpu().numpy(), v.cpu().numpy())
    assert res.fallbacks == 0

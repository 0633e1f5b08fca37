"""GPU parity: mf_score_pairs against the CPU checker, element by element."""
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


def _score_on_gpu(mm, ctx, r, scale=None, want_sigma=True):
    n, m = r["n"], r["m"]
    scale = r["cfg"].scale if scale is None else scale
    params = dev_params(r["params"])
    pred = ctx.predictor(params, scale)
    x_on, x_off = dev(r["x_on"]), dev(r["x_off"])
    W = empty_matrix(n, m)
    sigma = torch.empty((n, m), dtype=torch.float32, device="cuda") if want_sigma else None
    ctx.score_pairs(pred, x_on, x_off, W, sigma)
    torch.cuda.synchronize()
    Wh = W.cpu().numpy()
    assert (Wh[:, m:] == -7).all()                     # pitch padding untouched
    return Wh[:, :m], (sigma.cpu().numpy() if want_sigma else None)


def _compare(orc, r, Wg, sg, scale=None):
    scale = r["cfg"].scale if scale is None else scale
    sig, W = orc.score_pairs(r["x_on"], r["x_off"], r["params"], scale)
    assert ((Wg == INF) == (W == INF)).all(), "mask bits differ"
    rel = np.abs(sg.astype(np.float64) - sig) / sig
    assert rel.max() <= 1e-5, f"score relative error {rel.max():.3e}"
    ok = W != INF
    assert_weights_close(Wg, W, scale, ok)
    # the GPU's own quantisation of its own score is exact
    q = np.clip(np.rint(sg * np.float32(scale)), 0, scale).astype(np.int64)
    assert (Wg[ok] == q[ok]).all()
    return rel.max()


@pytest.mark.parametrize("cfg,n,m", [("C1", None, None), ("C2", None, None), ("C1", 1, 1), ("C1", 3, 5),
                                     ("C2", 130, 517), ("C3", 150, 700), ("C4", 97, 1031),
                                     ("C5", 64, 300), ("C3", 65, 257)])
def test_scores_match_checker(mm, orc, cfg, n, m):
    r = synth.scheduling_round(cfg, 1, n=n, m=m)
    for split in (1, 0):                # hidden-layer products from fp16 pieces (default) or from fp32 operands
        ctx = mm.Context(r["n"], max(r["m"], r["n"]))
        ctx.set_option("score_split", split)
        Wg, sg = _score_on_gpu(mm, ctx, r)
        _compare(orc, r, Wg, sg)
        ctx.close()


@pytest.mark.parametrize("case", ["huge projections", "tiny hidden weights", "huge hidden weights", "mixed magnitudes",
                                  "zero hidden layer"])
def test_scores_do_not_depend_on_the_size_of_the_numbers(mm, orc, case):
    """The fp16 pieces of the hidden layer's operands are scaled into fp16's range by powers of
    two found on the device: networks whose layers are scaled against each other (the same function
    up to rounding, or nearly) must still meet the score tolerance."""
    r = synth.scheduling_round("C3", 6, n=130, m=517)
    p = {k: v.copy() for k, v in r["params"].items()}
    if case == "huge projections":          # layer-1 values around 1e5, beyond fp16's 65,504
        p["W1"] *= np.float32(2.0 ** 17); p["b1"] *= np.float32(2.0 ** 17); p["W2"] *= np.float32(2.0 ** -17)
    elif case == "tiny hidden weights":     # W2 around 1e-7, where fp16 has no normal numbers
        p["W2"] *= np.float32(2.0 ** -20); p["b2"] *= np.float32(2.0 ** -20); p["W3"] *= np.float32(2.0 ** 20)
    elif case == "huge hidden weights":
        p["W2"] *= np.float32(2.0 ** 22); p["b2"] *= np.float32(2.0 ** 22); p["W3"] *= np.float32(2.0 ** -22)
    elif case == "mixed magnitudes":        # one hidden unit and one input a few thousand times larger than the rest
        p["W2"][3, :] *= np.float32(4096.0); p["b2"][3] *= np.float32(4096.0); p["W3"][3] *= np.float32(1.0 / 4096.0)
        p["W1"][5, :] *= np.float32(1024.0); p["b1"][5] *= np.float32(1024.0); p["W2"][:, 5] *= np.float32(1.0 / 1024.0)
    else:
        p["W2"][:] = 0.0
    r["params"] = p
    ctx = mm.Context(r["n"], r["m"])
    Wg, sg = _score_on_gpu(mm, ctx, r)
    worst = _compare(orc, r, Wg, sg)
    assert worst < 2e-6                      # well inside the bar: the scaling costs no accuracy
    ctx.close()


def test_scores_other_seeds_and_scales(mm, orc):
    ctx = mm.Context(300, 600)
    for seed in (2, 3):
        for scale in (255.0, float(2 ** 24)):
            r = synth.scheduling_round("C3", seed, n=200, m=333)
            Wg, sg = _score_on_gpu(mm, ctx, r, scale)
            _compare(orc, r, Wg, sg, scale)
    ctx.close()


@pytest.mark.parametrize("cfg,n,m", [("C1", None, None), ("C2", 130, 517), ("C4", 300, 1031), ("C5", 257, 700),
                                     ("C3", 65, 257), ("C5", 1, 40), ("C3", 700, 90), ("C3", 3, 40001),
                                     ("C5", 2, 70003)])
def test_memory_ordered_pass_gives_the_same_matrix(mm, orc, cfg, n, m):
    """Without a score buffer the kernel walks rows and columns by memory fraction and leaves out
    pairs that cannot fit: the matrix must equal the all-pairs pass bit for bit, and the checker's."""
    r = synth.scheduling_round(cfg, 4, n=n, m=m)
    n, m = r["n"], r["m"]
    ctx = mm.Context(n, m)
    Wg, _ = _score_on_gpu(mm, ctx, r, want_sigma=False)
    part = ctx.last_timings()["pairs_evaluated_fraction"]
    ctx.set_option("fit_order", 0)
    Wall, _ = _score_on_gpu(mm, ctx, r, want_sigma=False)
    assert ctx.last_timings()["pairs_evaluated_fraction"] == 1.0
    assert (Wg == Wall).all()
    _, W = orc.score_pairs(r["x_on"], r["x_off"], r["params"], r["cfg"].scale)
    assert ((Wg == INF) == (W == INF)).all(), "mask bits differ"
    ok = W != INF
    if ok.any():
        assert_weights_close(Wg, W, r["cfg"].scale, ok)
    # every feasible pair went through the MLP; skipped ones are only whole 32-column runs
    feasible = ok.mean()
    assert feasible - 1e-6 <= part <= 1.0
    if n >= 64 and m >= 256:
        assert part <= feasible + 0.35
    ctx.close()


def test_memory_order_with_ties_and_odd_pitch(mm, orc):
    """Many equal memory fractions (the ordering must still be a permutation), fractions of 0 and
    above the limit, and a matrix pitch that rules out 16-byte stores."""
    r = synth.scheduling_round("C3", 6, n=333, m=1001)
    n, m = r["n"], r["m"]
    r["x_on"][:, 0] = np.round(r["x_on"][:, 0] * 8) / np.float32(8)
    r["x_off"][:, 0] = np.round(r["x_off"][:, 0] * 8) / np.float32(8)
    r["x_on"][::7, 0] = 0.0; r["x_off"][::5, 0] = 1.5; r["x_off"][1::11, 0] = -0.0
    ctx = mm.Context(n, m)
    pred = ctx.predictor(dev_params(r["params"]), r["cfg"].scale)
    _, W = orc.score_pairs(r["x_on"], r["x_off"], r["params"], r["cfg"].scale)
    for pitch in (m, m + 3):
        Wd = torch.full((n, pitch), -7, dtype=torch.int32, device="cuda")
        ctx.score_pairs(pred, dev(r["x_on"]), dev(r["x_off"]), Wd)
        torch.cuda.synchronize()
        Wg = Wd.cpu().numpy()
        assert (Wg[:, m:] == -7).all()
        Wg = Wg[:, :m]
        assert ((Wg == INF) == (W == INF)).all()
        ok = W != INF
        assert_weights_close(Wg, W, r["cfg"].scale, ok)
    ctx.close()


def test_closed_form_predictors(mm):
    # zero network: every feasible weight is exactly S/2
    F, H, S = 16, 64, float(2 ** 20)
    zero = {"W1": np.zeros((H, 2 * F), np.float32), "b1": np.zeros(H, np.float32),
            "W2": np.zeros((H, H), np.float32), "b2": np.zeros(H, np.float32),
            "W3": np.zeros(H, np.float32), "b3": np.zeros(1, np.float32)}
    x_on = synth.uniform_features(1, 0, 70, F); x_off = synth.uniform_features(1, 1, 90, F)
    ctx = mm.Context(70, 90)
    W = empty_matrix(70, 90)
    ctx.score_pairs(ctx.predictor(dev_params(zero), S), dev(x_on), dev(x_off), W)
    Wh = W.cpu().numpy()[:, :90]
    masked = (x_on[:, 0][:, None] + x_off[:, 0][None, :]) > np.float32(1)
    assert (Wh[masked] == INF).all() and (Wh[~masked] == 2 ** 19).all()
    # identity network: z is the plain sum of all features of both workloads
    H = F = 64
    ident = {"W1": np.concatenate([np.eye(F), np.eye(F)], 1).astype(np.float32), "b1": np.zeros(H, np.float32),
             "W2": np.eye(H, dtype=np.float32), "b2": np.zeros(H, np.float32),
             "W3": np.ones(H, np.float32), "b3": np.zeros(1, np.float32)}
    x_on = synth.uniform_features(2, 0, 40, F) * np.float32(0.05)
    x_off = synth.uniform_features(2, 1, 50, F) * np.float32(0.05)
    W = empty_matrix(40, 50); sg = torch.empty((40, 50), dtype=torch.float32, device="cuda")
    ctx.score_pairs(ctx.predictor(dev_params(ident), S, mem_limit=4.0), dev(x_on), dev(x_off), W, sg)
    z = x_on.astype(np.float64).sum(1)[:, None] + x_off.astype(np.float64).sum(1)[None, :]
    np.testing.assert_allclose(sg.cpu().numpy(), 1 / (1 + np.exp(-z)), rtol=1e-5)
    ctx.close()


def test_argument_errors(mm):
    ctx = mm.Context(8, 8)
    r = synth.scheduling_round("C1", 1, n=8, m=8)
    params = dev_params(r["params"])
    x_on, x_off = dev(r["x_on"]), dev(r["x_off"])
    W = empty_matrix(8, 8)
    bad = ctx.predictor(params, 2.0 ** 20); bad.H = 48
    with pytest.raises(mm.MuxmatchError) as e:
        ctx.score_pairs(bad, x_on, x_off, W)
    assert e.value.code == mm.ERR_ARG
    big = synth.scheduling_round("C1", 1, n=9, m=9)
    with pytest.raises(mm.MuxmatchError) as e:
        ctx.score_pairs(ctx.predictor(params, 2.0 ** 20), dev(big["x_on"]), dev(big["x_off"]), empty_matrix(9, 9))
    assert e.value.code == mm.ERR_SHAPE
    ctx.close()

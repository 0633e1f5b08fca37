"""Pins for the CPU checker's pair scorer (no GPU): closed forms, special cases
that reduce to plain sums, and a black-box float64 library MLP."""
import numpy as np
import pytest
import torch

import synth

INF = synth.INFEASIBLE


def _zero_params(F, H):
    return {"W1": np.zeros((H, 2 * F), np.float32), "b1": np.zeros(H, np.float32),
            "W2": np.zeros((H, H), np.float32), "b2": np.zeros(H, np.float32),
            "W3": np.zeros(H, np.float32), "b3": np.zeros(1, np.float32)}


def test_all_zero_predictor_gives_half_scale(orc):
    F, H, S = 8, 16, 2 ** 20
    x_on = synth.uniform_features(1, 0, 12, F) * np.float32(0.4)
    x_off = synth.uniform_features(1, 1, 20, F) * np.float32(0.4)
    sig, W = orc.score_pairs(x_on, x_off, _zero_params(F, H), S)
    assert (sig == np.float32(0.5)).all() and (W == S // 2).all()


def test_identity_network_reduces_to_feature_sums(orc):
    # W1 = [I | I], W2 = I, W3 = 1, no biases, non-negative features:
    # z = sum_k (x_u[k] + x_v[k]); an operand swap or a dropped half of layer 1 changes it
    F = H = 8
    p = _zero_params(F, H)
    p["W1"][:, :F] = np.eye(F); p["W1"][:, F:] = np.eye(F)
    p["W2"][:] = np.eye(H); p["W3"][:] = 1.0
    x_on = synth.uniform_features(2, 0, 9, F) * np.float32(0.3)
    x_off = synth.uniform_features(2, 1, 14, F) * np.float32(0.3)
    sig, _ = orc.score_pairs(x_on, x_off, p, 2 ** 20)
    z = x_on.astype(np.float64).sum(1)[:, None] + x_off.astype(np.float64).sum(1)[None, :]
    np.testing.assert_allclose(sig, (1 / (1 + np.exp(-z))).astype(np.float32), rtol=1e-7)


def test_online_and_offline_halves_are_not_interchangeable(orc):
    # layer 1 reads the online features through columns [0,F) and the offline ones through [F,2F)
    F, H = 4, 4
    p = _zero_params(F, H)
    p["W1"][0, 0] = 1.0          # only online feature 0 feeds unit 0
    p["W2"][0, 0] = 1.0; p["W3"][0] = 1.0
    x_on = np.array([[0.25, 0, 0, 0]], np.float32); x_off = np.array([[0.75, 0, 0, 0]], np.float32)
    sig, _ = orc.score_pairs(x_on, x_off, p, 2 ** 20, mem_limit=2.0)
    assert sig[0, 0] == np.float32(1 / (1 + np.exp(-0.25)))


def test_dead_relu_leaves_bias_path(orc):
    F, H = 6, 10
    p = synth.predictor_params(3, F, H)
    p["W1"] = -np.abs(p["W1"]); p["b1"] = -np.abs(p["b1"])      # h1 == 0 for non-negative inputs
    x_on = synth.uniform_features(3, 0, 5, F); x_off = synth.uniform_features(3, 1, 7, F)
    sig, _ = orc.score_pairs(x_on, x_off, p, 2 ** 20)
    z = float(p["b3"][0]) + float((p["W3"].astype(np.float64) * np.maximum(p["b2"].astype(np.float64), 0)).sum())
    np.testing.assert_allclose(sig, np.float32(1 / (1 + np.exp(-z))), rtol=1e-7)


@pytest.mark.parametrize("cfg", ["C1", "C3"])
def test_matches_black_box_float64_mlp(orc, cfg):
    r = synth.scheduling_round(cfg, 5, n=48, m=80)
    p, F = r["params"], r["cfg"].F
    sig, W = orc.score_pairs(r["x_on"], r["x_off"], p, r["cfg"].scale)
    lin1 = torch.nn.Linear(2 * F, r["cfg"].H, dtype=torch.float64)
    lin2 = torch.nn.Linear(r["cfg"].H, r["cfg"].H, dtype=torch.float64)
    lin3 = torch.nn.Linear(r["cfg"].H, 1, dtype=torch.float64)
    with torch.no_grad():
        lin1.weight.copy_(torch.from_numpy(p["W1"]).double()); lin1.bias.copy_(torch.from_numpy(p["b1"]).double())
        lin2.weight.copy_(torch.from_numpy(p["W2"]).double()); lin2.bias.copy_(torch.from_numpy(p["b2"]).double())
        lin3.weight.copy_(torch.from_numpy(p["W3"]).double()[None, :]); lin3.bias.copy_(torch.from_numpy(p["b3"]).double())
        net = torch.nn.Sequential(lin1, torch.nn.ReLU(), lin2, torch.nn.ReLU(), lin3, torch.nn.Sigmoid())
        xo = torch.from_numpy(r["x_on"]).double(); xf = torch.from_numpy(r["x_off"]).double()
        pairs = torch.cat([xo[:, None, :].expand(-1, xf.shape[0], -1), xf[None, :, :].expand(xo.shape[0], -1, -1)], dim=2)
        ref = net(pairs)[..., 0].numpy()
    np.testing.assert_allclose(sig.astype(np.float64), ref, rtol=1e-7)
    # float32 evaluation of the same loops stays within float32 noise of the wide one
    sig32, _ = orc.score_pairs(r["x_on"], r["x_off"], p, r["cfg"].scale, wide=False)
    assert np.max(np.abs(sig32 - sig) / sig) < 5e-6


def test_quantisation_and_mask_rule(orc):
    r = synth.scheduling_round("C1", 9)
    S = r["cfg"].scale
    sig, W = orc.score_pairs(r["x_on"], r["x_off"], r["params"], S)
    mem = r["x_on"][:, 0][:, None] + r["x_off"][:, 0][None, :]          # one float32 addition
    assert mem.dtype == np.float32
    masked = mem > np.float32(1.0)
    assert ((W == INF) == masked).all()
    q = np.rint(sig * np.float32(S)).astype(np.int64)                   # float32 product, half-to-even
    assert (W[~masked] == q[~masked]).all()
    assert W[~masked].min() >= 0 and W[~masked].max() <= S
    # equality with the limit is feasible
    x_on = np.array([[0.5] + [0.0] * 15], np.float32); x_off = np.array([[0.5] + [0.0] * 15], np.float32)
    assert orc.score_pairs(x_on, x_off, r["params"], S)[1][0, 0] != INF
    # few-level scale
    _, W8 = orc.score_pairs(r["x_on"], r["x_off"], r["params"], 255.0)
    assert set(np.unique(W8[~masked])) <= set(range(256))
    assert (W8[~masked] == np.rint(sig * np.float32(255.0)).astype(np.int64)[~masked]).all()


def test_uniform_mask_fraction_matches_closed_form():
    # features U(0,1) scaled by c: P(c(a+b) > 1) = (2 - 1/c)^2 / 2 for 1/2 <= c <= 1
    for target in (0.10, 0.25):
        r = synth.scheduling_round(synth.RoundConfig("t", 1500, 1500, 4, 8, 1.0, "uniform", target), 2)
        c = r["mem_scale"]
        assert abs((2 - 1 / c) ** 2 / 2 - target) < 0.01
        realised = ((r["x_on"][:, 0][:, None] + r["x_off"][:, 0][None, :]) > np.float32(1)).mean()
        assert abs(realised - target) < 2e-3


def test_typed_scoring_is_a_per_row_choice_of_predictor(orc):
    """Pins score_pairs_typed: with one type it is score_pairs; with several, each row equals a
    one-row call under its own type's parameters (checked row by row)."""
    F, n, m = 16, 23, 31
    x_on = synth.uniform_features(5, 0, n, F); x_off = synth.uniform_features(5, 1, m, F)
    plist = synth.typed_predictors(9, F, [64, 128, 64])
    types = synth.gpu_types(5, n, 3)
    assert set(types.tolist()) == {0, 1, 2} and (np.bincount(types)[0] > np.bincount(types)[2])
    S = float(2 ** 20)
    s1, w1 = orc.score_pairs_typed(x_on, x_off, plist[:1], np.zeros(n, np.int32), S)
    s0, w0 = orc.score_pairs(x_on, x_off, plist[0], S)
    assert (s1 == s0).all() and (w1 == w0).all()
    st, wt = orc.score_pairs_typed(x_on, x_off, plist, types, S)
    for i in range(n):
        si, wi = orc.score_pairs(x_on[i:i + 1], x_off, plist[types[i]], S)
        assert (st[i] == si[0]).all() and (wt[i] == wi[0]).all()
    with pytest.raises(ValueError):
        orc.score_pairs_typed(x_on, x_off, plist, np.full(n, 3, np.int32), S)


def test_pair_dependent_sm_input(orc):
    """Pins the reading sm(u, v) = min(1 - x_u[a], x_v[d]) as a third predictor input."""
    F, H, S = 6, 8, float(2 ** 20)
    x_on = synth.uniform_features(4, 0, 11, F); x_off = synth.uniform_features(4, 1, 13, F)
    base = synth.predictor_params(4, F, H)
    # (i) a zero weight on the new input changes nothing, bit for bit
    p0 = synth.with_sm_input(base, 4); p0["W1"][:, -1] = 0.0
    s_plain, w_plain = orc.score_pairs(x_on, x_off, base, S)
    s_zero, w_zero = orc.score_pairs(x_on, x_off, p0, S, sm=(2, 3))
    assert (s_plain == s_zero).all() and (w_plain == w_zero).all()
    # (ii) a network that passes only the new input through: z = sm(u, v), by plain arithmetic
    p = {"W1": np.zeros((H, 2 * F + 1), np.float32), "b1": np.zeros(H, np.float32),
         "W2": np.zeros((H, H), np.float32), "b2": np.zeros(H, np.float32),
         "W3": np.zeros(H, np.float32), "b3": np.zeros(1, np.float32)}
    p["W1"][0, 2 * F] = 1.0; p["W2"][0, 0] = 1.0; p["W3"][0] = 1.0
    sig, _ = orc.score_pairs(x_on, x_off, p, S, sm=(2, 3))
    sm = np.minimum(np.float32(1.0) - x_on[:, 2][:, None], x_off[:, 3][None, :])
    assert sm.dtype == np.float32 and (sm > 0).any()
    np.testing.assert_allclose(sig, 1 / (1 + np.exp(-np.maximum(sm.astype(np.float64), 0))), rtol=1e-7)
    # the online and the offline feature index are not interchangeable
    other, _ = orc.score_pairs(x_on, x_off, p, S, sm=(3, 2))
    assert not np.allclose(other, sig)
    # (iii) black box: a float64 library MLP on the explicit concatenation [x_u ; x_v ; sm]
    pp = synth.with_sm_input(base, 9)
    got, _ = orc.score_pairs(x_on, x_off, pp, S, sm=(2, 3))
    lin1 = torch.nn.Linear(2 * F + 1, H, dtype=torch.float64); lin2 = torch.nn.Linear(H, H, dtype=torch.float64)
    lin3 = torch.nn.Linear(H, 1, dtype=torch.float64)
    with torch.no_grad():
        lin1.weight.copy_(torch.from_numpy(pp["W1"]).double()); lin1.bias.copy_(torch.from_numpy(pp["b1"]).double())
        lin2.weight.copy_(torch.from_numpy(pp["W2"]).double()); lin2.bias.copy_(torch.from_numpy(pp["b2"]).double())
        lin3.weight.copy_(torch.from_numpy(pp["W3"]).double()[None, :]); lin3.bias.copy_(torch.from_numpy(pp["b3"]).double())
        net = torch.nn.Sequential(lin1, torch.nn.ReLU(), lin2, torch.nn.ReLU(), lin3, torch.nn.Sigmoid())
        xo = torch.from_numpy(x_on).double(); xf = torch.from_numpy(x_off).double()
        pairs = torch.cat([xo[:, None, :].expand(-1, 13, -1), xf[None, :, :].expand(11, -1, -1),
                           torch.from_numpy(sm).double()[:, :, None]], dim=2)
        ref = net(pairs)[..., 0].numpy()
    np.testing.assert_allclose(got.astype(np.float64), ref, rtol=1e-7)
    with pytest.raises(ValueError):
        orc.score_pairs(x_on, x_off, pp, S, sm=(2, F))


def test_slowdown_unit_masks_pairs(orc):
    """Pins the second output unit: logistic(W3slow . h2 + b3slow) on the same hidden layers, pairs
    above the limit infeasible, everything else untouched."""
    F, H, S = 6, 8, float(2 ** 20)
    x_on = synth.uniform_features(6, 0, 12, F); x_off = synth.uniform_features(6, 1, 17, F)
    base = synth.predictor_params(6, F, H)
    s_plain, w_plain = orc.score_pairs(x_on, x_off, base, S)
    # (i) a zero unit predicts 1/2 for every pair: the limit decides for all of them at once
    p0 = synth.with_slowdown_unit(base, 6); p0["W3slow"][:] = 0.0; p0["b3slow"][:] = 0.0
    s_hi, w_hi = orc.score_pairs(x_on, x_off, p0, S, slow_limit=0.5)         # 1/2 > 1/2 is false
    assert (s_hi == s_plain).all() and (w_hi == w_plain).all()
    s_lo, w_lo = orc.score_pairs(x_on, x_off, p0, S, slow_limit=0.4999)
    assert (s_lo == s_plain).all() and (w_lo == INF).all()
    # (ii) black box: a float64 library MLP with two output units
    pp = synth.with_slowdown_unit(base, 8); pp["W3slow"] *= 3.0
    limit = 0.5
    sig, w = orc.score_pairs(x_on, x_off, pp, S, slow_limit=limit)
    lin1 = torch.nn.Linear(2 * F, H, dtype=torch.float64); lin2 = torch.nn.Linear(H, H, dtype=torch.float64)
    lin3 = torch.nn.Linear(H, 2, dtype=torch.float64)
    with torch.no_grad():
        lin1.weight.copy_(torch.from_numpy(pp["W1"]).double()); lin1.bias.copy_(torch.from_numpy(pp["b1"]).double())
        lin2.weight.copy_(torch.from_numpy(pp["W2"]).double()); lin2.bias.copy_(torch.from_numpy(pp["b2"]).double())
        lin3.weight.copy_(torch.from_numpy(np.stack([pp["W3"], pp["W3slow"]])).double())
        lin3.bias.copy_(torch.from_numpy(np.concatenate([pp["b3"], pp["b3slow"]])).double())
        net = torch.nn.Sequential(lin1, torch.nn.ReLU(), lin2, torch.nn.ReLU(), lin3, torch.nn.Sigmoid())
        xo = torch.from_numpy(x_on).double(); xf = torch.from_numpy(x_off).double()
        pairs = torch.cat([xo[:, None, :].expand(-1, 17, -1), xf[None, :, :].expand(12, -1, -1)], dim=2)
        ref = net(pairs).numpy()
    np.testing.assert_allclose(sig.astype(np.float64), ref[..., 0], rtol=1e-7)
    clear = np.abs(ref[..., 1] - limit) > 1e-6                # away from the limit both sides must agree
    too_slow = ref[..., 1] > limit
    assert too_slow.any() and (~too_slow).any()
    assert ((w == INF) == (too_slow | (w_plain == INF)))[clear].all()
    keep = (w != INF)
    assert (w[keep] == w_plain[keep]).all()                   # surviving pairs keep their weights
    # (iii) the memory mask and the slowdown mask add up
    tight, w_mem = orc.score_pairs(x_on, x_off, base, S, mem_feature=0, mem_limit=0.8)
    _, w_both = orc.score_pairs(x_on, x_off, pp, S, mem_feature=0, mem_limit=0.8, slow_limit=limit)
    assert (w_mem == INF).any() and ((w_both == INF) == ((w_mem == INF) | (w == INF))).all()

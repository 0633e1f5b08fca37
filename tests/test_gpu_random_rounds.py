"""GPU parity on randomly shaped scheduling rounds: any shape (also more online than offline
workloads, single rows and columns), any share of pairs that can share GPU memory, ties in the
memory fractions, the matching computed on either copy of the matrix.  Every case: mask bits equal
to the checker's, optimum bit-exact against the exact CPU solver, certificate re-verified on the host."""
import numpy as np
import pytest
import torch

import synth
from gpu_util import dev, dev_params, empty_matrix

pytestmark = pytest.mark.gpu
INF = synth.INFEASIBLE


@pytest.mark.parametrize("block", range(4))
def test_random_rounds(orc, block):
    import paper_2303_13803_amd as mm
    for case in range(block * 8, block * 8 + 8):
        rs = np.random.RandomState(5000 + case)
        n, m = int(rs.randint(1, 1100)), int(rs.randint(1, 1500))
        cfg = ["C2", "C3", "C4", "C5"][case % 4]
        r = synth.scheduling_round(cfg, case, n=n, m=m)
        share = [0.3, 0.8, 1.0, 1.6, 3.0][case % 5]            # rescales the memory fractions: how much can share
        r["x_on"][:, 0] = np.minimum(1.0, r["x_on"][:, 0] * share).astype(np.float32)
        r["x_off"][:, 0] = np.minimum(1.0, r["x_off"][:, 0] * share).astype(np.float32)
        if case % 7 == 0:
            r["x_on"][:, 0] = np.round(r["x_on"][:, 0] * 4) / np.float32(4)         # ties
        S = r["cfg"].scale
        ctx = mm.Context(n, m)
        ctx.set_option("fit_prefix_below", [101, 50, 0][case % 3])
        pred = ctx.predictor(dev_params(r["params"]), S)
        W = empty_matrix(n, m)
        r2c = torch.empty(n, dtype=torch.int32, device="cuda")
        u = torch.empty(n, dtype=torch.int64, device="cuda"); v = torch.empty(m, dtype=torch.int64, device="cuda")
        res = ctx.schedule_round(pred, dev(r["x_on"]), dev(r["x_off"]), W, r2c, u, v)
        Wg = W.cpu().numpy()[:, :m].copy()
        ctx.close()
        what = f"case {case}: {cfg} recipe, {n} x {m}, memory fractions x {share}"
        _, Wc = orc.score_pairs(r["x_on"], r["x_off"], r["params"], S, wide=False)
        assert ((Wg == INF) == (Wc == INF)).all(), what
        total = orc.max_weight_matching(Wg if n <= m else np.ascontiguousarray(Wg.T))[0]
        assert res.cert_ok == 1 and res.primal == total, what
        code, P, D = orc.check_certificate(Wg, r2c.cpu().numpy(), u.cpu().numpy(), v.cpu().numpy(), res.K)
        assert code == 0 and (P, D) == (res.primal, res.dual), what

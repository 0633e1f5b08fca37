"""GPU: the certificate check that allocates nothing against the one that uses context scratch.

Both evaluate the same proof on the same device buffers, so every field must agree exactly;
the second call on the same device takes a smaller problem (the shared array still holds the
first call's marks) and a third one a proof that must be rejected."""
import numpy as np
import pytest
import torch

import synth
from gpu_util import padded_matrix

pytestmark = pytest.mark.gpu


def _both(mm, binding, ctx, Wd, n, m, r2c, u, v, K, out):
    ref = ctx.check_certificate(Wd, n, m, r2c, u, v, K)
    out.fill_(0xAB)
    rc = binding.check_certificate_noalloc(Wd, n, m, r2c, u, v, K, out)
    assert rc == mm.OK, binding.strerror(rc)
    torch.cuda.synchronize()
    got = binding.read_certificate(out)
    for field in ("primal", "dual", "K", "min_reduced_cost", "matched", "cert_ok"):
        assert getattr(got, field) == getattr(ref, field), field
    return ref, got


def test_certificate_without_allocation_matches_the_context_one(orc):
    import paper_2303_13803_amd as mm
    from paper_2303_13803_amd import binding
    import ctypes
    out = torch.empty(ctypes.sizeof(binding.Certificate), dtype=torch.uint8, device="cuda")
    ctx = mm.Context(700, 1201)
    first = None
    for n, m, high, masked in [(700, 1201, 2 ** 24, 0.25), (257, 300, 255, 0.5)]:      # the second is smaller
        W = synth.uniform_matrix(77, n, m, high, masked)
        Wd = padded_matrix(W)
        r2c = torch.empty(n, dtype=torch.int32, device="cuda")
        u = torch.empty(n, dtype=torch.int64, device="cuda")
        v = torch.empty(m, dtype=torch.int64, device="cuda")
        res = ctx.solve_assignment(Wd, n, m, r2c, u, v)
        ref, got = _both(mm, binding, ctx, Wd, n, m, r2c, u, v, res.K, out)
        assert got.cert_ok == 1 and got.flags == 0 and got.primal == orc.max_weight_matching(W)[0]
        code, P, D = orc.check_certificate(W, r2c.cpu().numpy(), u.cpu().numpy(), v.cpu().numpy(), res.K)
        assert code == 0 and (P, D) == (got.primal, got.dual)
        if first is None:
            first = (Wd, n, m, r2c.clone(), u.clone(), v.clone(), res.K)
    # a proof that must fail, on the first (larger) problem again: one column used twice, one dual too small
    Wd, n, m, r2c, u, v, K = first
    matched = torch.nonzero(r2c >= 0).flatten()
    r2c[matched[1]] = r2c[matched[0]]
    u[matched[2]] -= 5 * K
    ref, got = _both(mm, binding, ctx, Wd, n, m, r2c, u, v, K, out)
    assert got.cert_ok == 0 and (got.flags & 1) and got.min_reduced_cost < 0
    ctx.close()


def test_sizes_beyond_the_static_array_are_refused():
    import paper_2303_13803_amd as mm
    from paper_2303_13803_amd import binding
    import ctypes
    out = torch.empty(ctypes.sizeof(binding.Certificate), dtype=torch.uint8, device="cuda")
    m = binding.NOALLOC_MAX_COLS + 4
    Wd = torch.zeros((1, m), dtype=torch.int32, device="cuda")
    r2c = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    u = torch.zeros(1, dtype=torch.int64, device="cuda")
    v = torch.zeros(m, dtype=torch.int64, device="cuda")
    assert binding.check_certificate_noalloc(Wd, 1, m, r2c, u, v, 2, out) == mm.ERR_SHAPE
    assert binding.check_certificate_noalloc(Wd, 1, m - 4, r2c, u, v, 0, out) == mm.ERR_ARG       # K < 1
    rc = binding.check_certificate_noalloc(Wd, 1, m - 4, r2c, u, v, 2, out)                       # the largest allowed
    assert rc == mm.OK
    torch.cuda.synchronize()
    got = binding.read_certificate(out)
    assert got.cert_ok == 1 and got.primal == 0 and got.dual == 0 and got.matched == 0

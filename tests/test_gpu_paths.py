"""GPU parity for the end of a run: bidders placed by shortest-augmenting-path searches.

The searches replace chains of bids, so the optimum (bit-exact against the exact CPU solver), the
validity of the matching and the host-verified duals are the whole contract; the cases force the
searches on from the first chain step, widen them to many bidders, and cut their waits short so
that they give up half-way and the chains take over again."""
import numpy as np
import pytest
import torch

import synth
from gpu_util import padded_matrix

pytestmark = pytest.mark.gpu
INF = synth.INFEASIBLE


@pytest.fixture(scope="module")
def mm():
    import paper_2303_13803_amd as mm
    import paper_2303_13803_amd.binding  # noqa: F401  (mm.binding: the bit names)
    return mm


def _solve_and_verify(ctx, orc, W, expect, fallbacks=0):
    """fallbacks: the bits mf_result must report (None: whatever), 0 for a solve nothing was forced to give up in."""
    n, m = W.shape
    r2c = torch.empty(n, dtype=torch.int32, device="cuda")
    u = torch.empty(n, dtype=torch.int64, device="cuda")
    v = torch.empty(m, dtype=torch.int64, device="cuda")
    res = ctx.solve_assignment(padded_matrix(W), n, m, r2c, u, v)
    code, P, D = orc.check_certificate(W, r2c.cpu().numpy(), u.cpu().numpy(), v.cpu().numpy(), res.K)
    assert code == 0 and res.cert_ok == 1
    assert (P, D) == (res.primal, res.dual)
    assert res.primal == expect
    if fallbacks is not None:
        assert res.fallbacks == fallbacks
    return res


def _cases():
    yield "uniform square", synth.uniform_matrix(41, 700, 700, 2 ** 20, 0.1)
    yield "uniform wide, reverse rounds", synth.uniform_matrix(42, 400, 900, 2 ** 24, 0.3)
    yield "more rows than columns", synth.uniform_matrix(43, 900, 350, 2 ** 20, 0.2)
    yield "few levels, nested neighbourhoods", synth.threshold_matrix(44, 500, 800, 256, 0.9)
    yield "rank one", synth.rank_one_matrix(45, 300, 450, 2 ** 20)[0]
    yield "planted", synth.planted_matrix(46, 300, 400, 2 ** 20)[0]
    yield "constant", np.full((200, 300), 77, np.int32)
    yield "single row", synth.uniform_matrix(47, 1, 50, 1000, 0.0)
    yield "nothing feasible", np.full((60, 70), INF, np.int32)
    W = synth.uniform_matrix(50, 1400, 1400, 2 ** 24, 0.1)          # rows that rest while epsilon is coarse
    faint = W[:120] != INF
    W[:120][faint] = W[:120][faint] >> 12
    yield "square with faint rows", W


def _optimum(orc, W):
    n, m = W.shape
    return orc.max_weight_matching(W if n <= m else np.ascontiguousarray(W.T))[0]


@pytest.mark.parametrize("options", [{"path_after": 0}, {"path_after": 0, "path_max": 64, "team_max": 0},
                                     {"path_after": 0, "path_pull": 1}, {"path_after": 0, "path_max": 64, "team_max": 0, "path_pull": 1},
                                     {"path_after": 20, "path_pull": 1, "path_width": 2},
                                     {"path_after": 0, "path_width": 1}, {"path_after": 40},
                                     {"team_wide": 64, "team_regroup": 16, "path_after": 30},
                                     {"team_wide": 24, "team_size": 4, "path_max": 0}])
def test_searches_reach_the_optimum(mm, orc, options):
    used = 0
    for name, W in _cases():
        ctx = mm.Context(*W.shape)
        for k, val in options.items():
            ctx.set_option(k, val)
        res = _solve_and_verify(ctx, orc, W, _optimum(orc, W))
        used += res.path_steps
        ctx.close()
    if options.get("path_max", 8) > 0:
        assert used > 0, "no search ran: the cases no longer exercise this path"


def test_scored_round_with_searches_only(mm, orc):
    r = synth.scheduling_round("C4", 3, n=1500, m=1500)
    W = orc.score_pairs(r["x_on"], r["x_off"], r["params"], r["cfg"].scale, wide=False)[1]
    ctx = mm.Context(1500, 1500)
    for pull in (0, 1):
        ctx.set_option("path_after", 0)
        ctx.set_option("path_pull", pull)
        ctx.set_option("team_wide", 0)                  # no teams between the chain kernel and the searches
        res = _solve_and_verify(ctx, orc, W, orc.max_weight_matching(W)[0])
        assert res.path_steps > 0 and res.team_bids == 0
    ctx.close()


@pytest.mark.parametrize("polls", [0, 3, 40])
def test_a_search_that_gives_up_hands_back_to_the_chains(mm, orc, polls):
    """The waits between the workgroups of a search are bounded; with a bound of a few polls they
    run out at arbitrary points.  Whatever was reached must still be a valid state: the chains
    finish the run and the result is the exact optimum."""
    W = synth.uniform_matrix(48, 800, 800, 2 ** 20, 0.1)
    expect = orc.max_weight_matching(W)[0]
    ctx = mm.Context(800, 800)
    ctx.set_option("path_after", 0)
    ctx.set_option("path_pull", polls % 2)                # one of the two ways a served tree's columns are labelled again
    ctx.set_option("path_spin_limit", polls)
    gave_up = 0
    for attempt in range(3):                              # every solve starts with its searches switched on again
        res = _solve_and_verify(ctx, orc, W, expect, fallbacks=None)
        assert res.fallbacks in (0, mm.binding.FALLBACK_SEARCHES)
        gave_up += res.fallbacks != 0
    if polls == 0:
        assert gave_up == 3                               # no wait at all: the first barrier of every solve runs out
    ctx.set_option("path_spin_limit", 1 << 22)
    res = _solve_and_verify(ctx, orc, W, expect)          # ... and reports nothing once the waits are long enough
    assert res.path_steps > 0
    ctx.close()


@pytest.mark.parametrize("chain_grid", [1, 8, 64])
def test_chain_kernel_with_fewer_workgroups_than_it_hands_back_at(mm, orc, chain_grid):
    """With so few workgroups every one of them hands its bidder back at its first step; the
    entries of the list nobody claimed must still reach the next kernel."""
    for name, W in [("uniform square", synth.uniform_matrix(51, 900, 900, 2 ** 20, 0.1)),
                    ("wide", synth.uniform_matrix(52, 500, 1300, 2 ** 24, 0.3)),
                    ("few levels", synth.threshold_matrix(53, 600, 900, 256, 0.9))]:
        ctx = mm.Context(*W.shape)
        ctx.set_option("chain_grid", chain_grid)
        _solve_and_verify(ctx, orc, W, _optimum(orc, W))
        ctx.close()


@pytest.mark.parametrize("options", [{"phase_stop": 0}, {"phase_stop": 8, "phase_keep": 1},
                                     {"phase_stop": 64, "phase_keep": 2, "phase_growth": 4, "path_after": 0},
                                     {"phase_stop": 1 << 20, "phase_keep": 1},
                                     {"phase_stop": 3, "phase_keep": 64},
                                     {"phase_tail_steps": 1, "phase_tail_from": 0, "phase_tail_sides": 3},
                                     {"phase_tail_steps": 8, "phase_tail_from": 0, "phase_tail_sides": 2, "phase_stop": 64},
                                     {"phase_tail_steps": 4, "phase_tail_from": 0, "phase_tail_sides": 1, "phase_keep": 1},
                                     {"phase_growth": 4, "phase_growth_rest": 0}, {"phase_growth": 3, "phase_growth_rest": 1 << 20},
                                     {"round_lag": 0}, {"round_lag": 1, "tail_max": 16},
                                     {"round_lag": 1, "tail_max": 0, "phase_stop": 64}])
def test_phases_that_end_early_leave_the_optimum_alone(mm, orc, options):
    """Phases at a coarse epsilon may stop with bidders unplaced (they only prepare prices); with
    more columns than rows the other side then runs from profits that cover the unplaced rows.
    Whatever the setting - every phase completed, only the last one, as many bidders left over as
    the library allows, chains of bids cut off after a few steps on either side - the last phase
    makes the result exactly optimal."""
    cases = list(_cases()) + [("one more column than rows", synth.uniform_matrix(48, 300, 301, 2 ** 24, 0.2)),
                              ("one more row than columns", synth.uniform_matrix(49, 301, 300, 2 ** 24, 0.2))]
    for name, W in cases:
        ctx = mm.Context(*W.shape)
        for k, val in options.items():
            ctx.set_option(k, val)
        _solve_and_verify(ctx, orc, W, _optimum(orc, W))
        ctx.close()


_BULK = {}


@pytest.mark.parametrize("options", [{}, {"bulk_shape": 0}, {"bulk_shape": 2, "bulk_share": 0},
                                     {"bulk_shape": 3, "bulk_share": 50}, {"bulk_shape": 4, "bulk_grid": 64},
                                     {"bulk_share": 100, "round_lag": 0}, {"bulk_share": 0, "bulk_grid": 8192}])
def test_workgroup_shapes_of_the_bidding_rounds(mm, orc, options):
    """Rounds with at least 2048 bidders choose among several workgroup shapes (lines in groups
    per wavefront when nearly every line bids, one line per workgroup otherwise); which one runs
    when changes the order in which bids land, never the optimum.  Two matrices just large enough
    for such rounds, the exact CPU solver run once for all settings."""
    if not _BULK:
        for name, W in [("square", synth.uniform_matrix(61, 2200, 2200, 2 ** 20, 0.2)),
                        ("wide, few levels", synth.threshold_matrix(62, 2100, 2600, 256, 0.8))]:
            _BULK[name] = (W, _optimum(orc, W))
    for name, (W, expect) in _BULK.items():
        ctx = mm.Context(*W.shape)
        for k, val in options.items():
            ctx.set_option(k, val)
        _solve_and_verify(ctx, orc, W, expect)
        ctx.close()

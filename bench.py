"""Benchmark: whole scheduling rounds (score every pair, then match) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C4] [--seed 1]

A step is one mf_schedule_round on a cluster-shaped synthetic round whose inputs
already sit in device memory.  Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_FP32_PEAK = 157.3e12      # MI355X dense fp32 matrix peak, flop/s
MFMA_FP16_PEAK = 2.5e15        # MI355X dense fp16 matrix peak, flop/s
SPLIT_PRODUCTS = 3             # fp16 matrix products the default scorer issues per product of two fp32 operands
HBM_PEAK = 8.0e12              # byte/s

# HBM bytes per launch from hardware counters (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by
# what the same counters read for a 1 GiB copy), valid for the named kernel at the named workload
# only.  Set an entry to None when its kernel changes after the counters were taken.
MEASURED_TRAFFIC = {
    ("C4", "pair_mlp_kernel"): 2.167e9,
    ("C4", "pair_mlp_kernel, fp32 products"): 2.058e9,
    ("C4", "round_kernel"): 1.614e9,
}


def cpu_baseline(r, Wg_block, sample_rows, full=None):
    """Times the CPU checker, as it stands, on a bounded sample of the same round.

    full = (W, row2col, u, v, K) as host arrays: also times the checker's O(nm) verification of the
    GPU's certificate on the whole matrix (the one part of the matching the CPU can do at this size)."""
    import numpy as np

    import oracle
    S = r["cfg"].scale
    rows = min(sample_rows, r["n"])
    t0 = time.perf_counter()
    oracle.score_pairs(r["x_on"][:rows], r["x_off"], r["params"], S, wide=False)
    t_score = time.perf_counter() - t0
    side = Wg_block.shape[0]
    t0 = time.perf_counter()
    oracle.max_weight_matching(np.ascontiguousarray(Wg_block))
    t_match = time.perf_counter() - t0
    t_cert = None
    if full is not None:
        t0 = time.perf_counter()
        code = oracle.check_certificate(*full)[0]
        t_cert = time.perf_counter() - t0
        assert code == 0, f"host certificate check failed with code {code}"
    return {"certificate_check_ms": None if t_cert is None else t_cert * 1e3,
            "value": rows * r["m"] / t_score, "unit": "pairs/s", "cores": oracle.threads(), "kind": "oracle",
            "sample": (f"float32 scorer on the first {rows} of {r['n']} online rows x all {r['m']} offline "
                       f"columns ({t_score:.2f} s, OpenMP over rows); exact matching timed separately on the "
                       f"leading {side}x{Wg_block.shape[1]} block of the scored matrix, 1 thread: "
                       f"{t_match * 1e3:.0f} ms (O(n^2 m): the full round does not finish); "
                       + (f"the GPU's optimality certificate for the whole matrix re-verified on the host in "
                          f"{t_cert * 1e3:.0f} ms; " if t_cert is not None else "")
                       + "value is the scoring rate alone, an upper bound on a CPU round"),
            "matching_block_ms": t_match * 1e3}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="C4")
    ap.add_argument("--seed", type=int, default=1)
    ap.add_argument("--cpu-rows", type=int, default=1280)
    ap.add_argument("--cpu-block", type=int, default=1536)
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--update-rounds", type=int, default=3,
                    help="also time this many follow-up rounds with --churn of the workloads replaced")
    ap.add_argument("--churn", type=float, default=0.02)
    ap.add_argument("--other-seeds", default="2,3,4,5,6,7,8,12",
                    help="also run one warm-up and two rounds on these input seeds and report the median "
                         "round time over all seeds ('' to skip)")
    ap.add_argument("--all-configs", default="C1,C2,C3,C5",
                    help="also run whole rounds of these configurations, each with its certificate checked on the "
                         "device and, with the CPU baseline on, again on the host ('' to skip)")
    ap.add_argument("--no-masked-matrix", dest="masked_matrix", action="store_false",
                    help="skip matching a caller-brought matrix with an arbitrary 90 percent mask")
    ap.add_argument("--types", type=int, default=3,
                    help="also time scoring with this many per-GPU-type predictors (0: skip)")
    ap.add_argument("--calib-mib", type=int, default=0,
                    help="also run a plain device copy of this many MiB (reference for hardware byte counters)")
    ap.add_argument("--no-fp32-products", dest="fp32_products", action="store_false",
                    help="skip the extra rounds with fp32 products in the scorer (option score_split = 0)")
    ap.add_argument("--no-sm-input", dest="sm_input", action="store_false",
                    help="skip timing the scorer with the pair-dependent SM input")
    ap.add_argument("--opt", action="append", default=[], help="solver option name=value (repeatable)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py measures one GPU: the scheduling round is a single-device kernel path "
              "(run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2303_13803_amd as mm
    import synth

    r = synth.scheduling_round(args.config, args.seed)
    cfg, n, m = r["cfg"], r["n"], r["m"]
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    ctx = mm.Context(n, m, device=0)
    params = {k: dev(v) for k, v in r["params"].items()}
    for kv in args.opt:
        name, value = kv.split("=")
        ctx.set_option(name, int(value))
    pred = ctx.predictor(params, cfg.scale)
    x_on, x_off = dev(r["x_on"]), dev(r["x_off"])
    ld = (m + 3) // 4 * 4
    W = torch.empty((n, ld), dtype=torch.int32, device="cuda")
    r2c = torch.empty(n, dtype=torch.int32, device="cuda")
    u = torch.empty(n, dtype=torch.int64, device="cuda")
    v = torch.empty(m, dtype=torch.int64, device="cuda")

    def step():
        res = ctx.schedule_round(pred, x_on, x_off, W, r2c, u, v)
        return res, ctx.last_timings()

    if args.calib_mib:
        src = torch.ones(args.calib_mib * 262144, dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    stages = []
    for _ in range(args.steps):
        stages.append(step())
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps
    res = stages[-1][0]
    assert all(s[0].cert_ok == 1 for s in stages)
    assert all(s[0].fallbacks == 0 for s in stages), "a bounded wait ran out: the timed rounds did not run as designed"
    avg = {k: float(np.mean([s[1][k] for s in stages])) for k in stages[0][1]}

    pair_ms = avg["pair_scoring_ms"]
    # hidden-layer MFMA flops one launch issues: pairs that cannot fit in memory get no MLP pass
    evaluated = avg["pairs_evaluated_fraction"]
    flops = 2.0 * cfg.H * cfg.H * n * m * evaluated
    achieved = flops / (pair_ms * 1e-3)
    bulk_launches = max(avg["bulk_bid_launches"], 1.0)
    bulk_bytes = avg["bulk_bid_bytes"] / bulk_launches
    bulk_ms = max(avg["bulk_bid_ms"] / bulk_launches, 1e-9)      # no bulk round at tiny sizes
    out = {
        "metric": "pairs scored/s + schedule_round latency (ms) at 20k x 20k on 1 MI355X",
        "value": n * m / (ms_per_step * 1e-3), "unit": "pairs/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 pieces of f32 operands with f32 accumulation (scoring, MFMA: two pieces per operand, three "
                 "products, scores as close to f64 as with f32 products) / i32 weights with exact integer duals (matching)",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {n} online x {m} offline, F={cfg.F}, MLP {2 * cfg.F}->{cfg.H}->{cfg.H}->1, "
                               f"S={cfg.scale:g}, {cfg.features} features, ~{cfg.masked} masked, seed {args.seed}; "
                               "value = n*m / time of one whole round (score + match + certificate)"},
        "schedule_round_ms": ms_per_step,
        "score_pairs_per_s": n * m / ((pair_ms + avg["projections_ms"]) * 1e-3),
        "stage_ms": {k: avg[k] for k in ("projections_ms", "pair_scoring_ms", "prepare_ms", "auction_ms",
                                         "duals_ms", "certificate_ms")},
        # the two whole-matrix passes after the auction, against the 4 n m bytes each has to read
        "scan_gbps": {"duals": 4.0 * n * m / (avg["duals_ms"] * 1e-3) / 1e9 if avg["duals_ms"] > 0 else None,
                      "certificate": 4.0 * n * m / (avg["certificate_ms"] * 1e-3) / 1e9 if avg["certificate_ms"] > 0 else None},
        "auction": {"phases": res.phases, "rounds": res.rounds, "bids": res.bids,
                    "bytes_scanned": res.bytes_scanned, "chain_bids": res.chain_bids, "chain_depth": res.chain_depth, "chain_retries": res.chain_retries, "team_bids": res.team_bids, "path_steps": res.path_steps, "path_scans": res.path_scans, "matched": res.matched,
                    "primal": res.primal, "cert_ok": res.cert_ok, "fallbacks": res.fallbacks},
        # The dominant kernel.  Its contraction runs on the fp16 matrix pipe, so the peak is that
        # pipe's; `achieved` counts the algorithmic flops (2 H^2 per scored pair), of which the kernel
        # issues SPLIT_PRODUCTS times as many in fp16 (`issued_frac`).
        "roofline": {"bound": "mfma", "kernel": "pair_mlp_kernel (fp16 pieces of fp32 operands, three products)",
                     "achieved": achieved / 1e12,
                     "peak": MFMA_FP16_PEAK / 1e12, "unit": "TFLOP/s", "frac": achieved / MFMA_FP16_PEAK,
                     "issued_frac": SPLIT_PRODUCTS * achieved / MFMA_FP16_PEAK,
                     "times_fp32_matrix_peak": achieved / MFMA_FP32_PEAK,
                     "pairs_evaluated_fraction": evaluated,
                     "traffic": MEASURED_TRAFFIC.get((cfg.name, "pair_mlp_kernel")),
                     "note": "frac counts one product per pair of fp32 operands against the fp16 matrix peak; the kernel "
                             "issues three fp16 products for it (issued_frac).  The same layer with fp32 products "
                             "(fp32_products.roofline) runs at 0.85 of the fp32 matrix peak and takes three times as long"},
        "roofline_bid_scan": {"bound": "hbm", "kernel": "round_kernel (first round of each phase: every row bids)",
                              "achieved": bulk_bytes / (bulk_ms * 1e-3) / 1e9, "peak": HBM_PEAK / 1e9,
                              "unit": "GB/s", "frac": bulk_bytes / (bulk_ms * 1e-3) / HBM_PEAK,
                              "bytes_per_launch": bulk_bytes, "ms_per_launch": bulk_ms,
                              "traffic": MEASURED_TRAFFIC.get((cfg.name, "round_kernel")),
                              # every weight byte any scan of the solve read, over the whole auction's time
                              "whole_solve_gbps": res.bytes_scanned / (avg["auction_ms"] * 1e-3) / 1e9},
        # the chain-following kernels take most of the auction's time but are bound by the latency of
        # dependent steps, not by bandwidth: reported as steps and microseconds per step
        "auction_tail": {"kernels": "chain_kernel + team_kernel (dependent bids), path_kernel (search super-steps)",
                         "bound": "latency", "sequential_steps": res.chain_depth, "bids": res.chain_bids,
                         "path_super_steps": res.path_steps, "path_row_scans": res.path_scans,
                         "chain_steps": res.chain_depth - res.path_steps},
    }
    # measured ceilings of this device next to the published peaks
    ceil = ctx.measure_ceilings(W)
    out["roofline"]["measured_ceiling"] = ceil["mfma_f16_tflops"]
    out["roofline"]["issued_frac_of_measured_ceiling"] = SPLIT_PRODUCTS * achieved / 1e12 / ceil["mfma_f16_tflops"]
    if args.fp32_products:
        # the same rounds with fp32 products in the scorer (option score_split = 0): the matrix instruction,
        # peak and roofline of the fp32 pipe
        ctx.set_option("score_split", 0)
        step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        plain = [step() for _ in range(max(2, args.steps // 2))]
        torch.cuda.synchronize()
        plain_ms = (time.perf_counter() - t0) * 1e3 / len(plain)
        ctx.set_option("score_split", 1)
        assert all(s[0].cert_ok == 1 and s[0].fallbacks == 0 for s in plain)
        plain_pair_ms = float(np.mean([s[1]["pair_scoring_ms"] for s in plain]))
        plain_achieved = flops / (plain_pair_ms * 1e-3)
        out["fp32_products"] = {"schedule_round_ms": plain_ms, "pair_scoring_ms": plain_pair_ms,
                                "value": n * m / (plain_ms * 1e-3), "unit": "pairs/s",
                                "roofline": {"bound": "mfma", "kernel": "pair_mlp_kernel (fp32 products, v_mfma_f32_32x32x2_f32)",
                                             "achieved": plain_achieved / 1e12, "peak": MFMA_FP32_PEAK / 1e12, "unit": "TFLOP/s",
                                             "frac": plain_achieved / MFMA_FP32_PEAK,
                                             "measured_ceiling": ceil["mfma_f32_tflops"],
                                             "frac_of_measured_ceiling": plain_achieved / 1e12 / ceil["mfma_f32_tflops"],
                                             "traffic": MEASURED_TRAFFIC.get((cfg.name, "pair_mlp_kernel, fp32 products"))}}
    out["roofline_bid_scan"]["measured_ceiling"] = ceil["read_gbps"]
    out["roofline_bid_scan"]["frac_of_measured_ceiling"] = bulk_bytes / (bulk_ms * 1e-3) / 1e9 / ceil["read_gbps"]
    if args.other_seeds:
        # the same round on other draws of the workload: per-seed round time and the median over seeds
        per_seed = {str(args.seed): ms_per_step}
        for sd in [int(x) for x in args.other_seeds.split(",") if x]:
            rs = synth.scheduling_round(args.config, sd)
            ps = ctx.predictor({k: dev(v) for k, v in rs["params"].items()}, cfg.scale)
            xo_s, xf_s = dev(rs["x_on"]), dev(rs["x_off"])
            ctx.schedule_round(ps, xo_s, xf_s, W, r2c, u, v)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(2):
                rr = ctx.schedule_round(ps, xo_s, xf_s, W, r2c, u, v)
                assert rr.cert_ok == 1 and rr.fallbacks == 0
            torch.cuda.synchronize()
            per_seed[str(sd)] = (time.perf_counter() - t0) * 1e3 / 2
            del rs, ps, xo_s, xf_s
        med = float(np.median(list(per_seed.values())))
        worst = max(per_seed, key=per_seed.get)
        # a scheduler interval has to budget for the slowest round, not the median one
        out["seeds"] = {"round_ms": per_seed, "median_round_ms": med, "max_round_ms": per_seed[worst],
                        "max_round_seed": int(worst), "max_over_median": per_seed[worst] / med}
    checks = {}
    if args.all_configs:
        # every other configuration: whole rounds, certificate on the device (and on the host below)
        out["all_configs"] = {}
        for name in [c for c in args.all_configs.split(",") if c and c != args.config]:
            rk = synth.scheduling_round(name, args.seed)
            ck, nk, mk = rk["cfg"], rk["n"], rk["m"]
            ctxk = mm.Context(nk, mk, device=0)
            pk = ctxk.predictor({k: dev(v) for k, v in rk["params"].items()}, ck.scale)
            xo_k, xf_k = dev(rk["x_on"]), dev(rk["x_off"])
            Wk = torch.empty((nk, (mk + 3) // 4 * 4), dtype=torch.int32, device="cuda")
            r2ck = torch.empty(nk, dtype=torch.int32, device="cuda")
            uk = torch.empty(nk, dtype=torch.int64, device="cuda"); vk = torch.empty(mk, dtype=torch.int64, device="cuda")
            ctxk.schedule_round(pk, xo_k, xf_k, Wk, r2ck, uk, vk)
            ms, last_k = [], None
            for _ in range(3):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                last_k = ctxk.schedule_round(pk, xo_k, xf_k, Wk, r2ck, uk, vk)
                torch.cuda.synchronize()
                ms.append((time.perf_counter() - t0) * 1e3)
                assert last_k.cert_ok == 1 and last_k.fallbacks == 0
            tk = ctxk.last_timings()
            out["all_configs"][name] = {"n": nk, "m": mk, "round_ms": float(np.median(ms)), "auction_ms": tk["auction_ms"],
                                        "pair_scoring_ms": tk["pair_scoring_ms"], "phases": last_k.phases,
                                        "matched": last_k.matched, "primal": last_k.primal, "cert_ok": last_k.cert_ok,
                                        "fallbacks": last_k.fallbacks,
                                        "pairs_evaluated_fraction": tk["pairs_evaluated_fraction"]}
            if not args.no_cpu:
                checks[name] = (np.ascontiguousarray(Wk[:, :mk].cpu().numpy()), r2ck.cpu().numpy(), uk.cpu().numpy(),
                                vk.cpu().numpy(), last_k.K)
            ctxk.close()
            del Wk, xo_k, xf_k, rk
    if args.update_rounds > 0:
        # follow-up rounds: a share of the online and offline workloads is replaced by fresh draws,
        # only their rows/columns are re-scored, then the matching is solved again (from zero prices
        # unless the warm-start option is set)
        xo, xf = r["x_on"].copy(), r["x_off"].copy()
        times, last = [], None
        for k in range(args.update_rounds):
            fresh = synth.scheduling_round(cfg, args.seed + 100 + k)
            rows = np.sort(synth.permutation(args.seed + k, n, 3)[:max(1, int(args.churn * n))]).astype(np.int32)
            cols = np.sort(synth.permutation(args.seed + k, m, 4)[:max(1, int(args.churn * m))]).astype(np.int32)
            xo[rows] = fresh["x_on"][rows]; xf[cols] = fresh["x_off"][cols]
            d_on, d_off, d_rows, d_cols = dev(xo), dev(xf), dev(rows), dev(cols)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            last = ctx.schedule_round_update(pred, d_on, d_off, d_rows, d_cols, W, r2c, u, v)
            torch.cuda.synchronize()
            times.append((time.perf_counter() - t0) * 1e3)
            assert last.cert_ok == 1
        tm = ctx.last_timings()
        out["next_round_update"] = {"churn": args.churn, "rounds": args.update_rounds, "ms_per_round": float(np.mean(times)),
                                    "ms_each": times, "auction_ms_last": tm["auction_ms"],
                                    "rescore_ms_last": tm["pair_scoring_ms"] + tm["projections_ms"],
                                    "phases_last": last.phases, "bids_last": last.bids,
                                    "sequential_steps_last": last.chain_depth}
    if args.masked_matrix:
        # a matrix the caller brings, one pair in ten feasible in no pattern: matched from per-row
        # edge lists (default) and, for comparison, from the rows themselves
        Wm = synth.device_masked_matrix(args.seed, n, m, int(cfg.scale), 10, pitch=ld)
        entry = {"feasible_share": 0.1, "n": n, "m": m}
        for label, lists_from in (("edge_lists", None), ("rows", 0)):
            if lists_from is not None:
                ctx.set_option("edge_lists_from", lists_from)
            ms = []
            for _ in range(3):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                rm_ = ctx.solve_assignment(Wm, n, m, r2c, u, v)
                torch.cuda.synchronize()
                ms.append((time.perf_counter() - t0) * 1e3)
                assert rm_.cert_ok == 1 and rm_.fallbacks == 0
            tm = ctx.last_timings()
            entry[label] = {"solve_ms": float(np.median(ms)), "auction_ms": tm["auction_ms"], "prepare_ms": tm["prepare_ms"],
                            "bytes_scanned": rm_.bytes_scanned, "phases": rm_.phases, "rounds": rm_.rounds,
                            "primal": rm_.primal, "cert_ok": rm_.cert_ok}
        ctx.set_option("edge_lists_from", 4096)
        assert entry["edge_lists"]["primal"] == entry["rows"]["primal"]
        out["masked_matrix"] = entry
        del Wm
    if args.types > 0:
        # one predictor per GPU type: same shapes, other weights; rows are scored by their type's
        plist = [{k: dev(v) for k, v in p.items()} for p in synth.typed_predictors(args.seed + 7, cfg.F, [cfg.H] * args.types)]
        tpreds = [ctx.predictor(p, cfg.scale) for p in plist]
        d_types = dev(synth.gpu_types(args.seed, n, args.types))
        W2 = torch.empty_like(W)
        ms = []
        for _ in range(3):
            ctx.score_pairs_typed(tpreds, d_types, x_on, x_off, W2)
            torch.cuda.synchronize()
            tm = ctx.last_timings()
            ms.append(tm["pair_scoring_ms"] + tm["projections_ms"])
        out["typed_scoring"] = {"gpu_types": args.types, "ms": float(np.median(ms)),
                                "pairs_per_s": n * m / (float(np.median(ms)) * 1e-3),
                                "pairs_evaluated_fraction": tm["pairs_evaluated_fraction"]}
        del W2
    if args.sm_input:
        # the pair-dependent SM share as a third predictor input (same network plus one layer-1 column)
        full = synth.with_sm_input(r["params"], args.seed + 3)
        sp = dict(params)
        sp["W1sm"] = dev(full["W1"][:, -1])
        spred = ctx.predictor(sp, cfg.scale, sm=(2, 3))
        W2 = torch.empty_like(W)
        ms = []
        for _ in range(3):
            ctx.score_pairs(spred, x_on, x_off, W2)
            torch.cuda.synchronize()
            tm = ctx.last_timings()
            ms.append(tm["pair_scoring_ms"] + tm["projections_ms"])
        out["sm_input_scoring"] = {"ms": float(np.median(ms)), "pairs_per_s": n * m / (float(np.median(ms)) * 1e-3),
                                   "pairs_evaluated_fraction": tm["pairs_evaluated_fraction"]}
        del W2
    if not args.no_cpu:
        blk = min(args.cpu_block, n)
        # the matrix and the certificate of the last full round on --seed (recomputed: later
        # sections reused the buffers)
        res = ctx.schedule_round(pred, x_on, x_off, W, r2c, u, v)
        Wh = W[:, :m].cpu().numpy()
        Wg_block = np.ascontiguousarray(Wh[:blk, :min(m, blk * (m // n))])
        out["cpu_baseline"] = cpu_baseline(r, Wg_block, args.cpu_rows,
                                           (np.ascontiguousarray(Wh), r2c.cpu().numpy(), u.cpu().numpy(),
                                            v.cpu().numpy(), res.K))
        # the other configurations' certificates, re-verified by the checker on the host
        import oracle
        verified = {}
        for name, full in checks.items():
            t0 = time.perf_counter()
            code = oracle.check_certificate(*full)[0]
            verified[name] = {"ok": code == 0, "ms": (time.perf_counter() - t0) * 1e3}
            assert code == 0, f"host certificate check of {name} failed with code {code}"
        out["cpu_baseline"]["certificates_verified_on_host"] = verified
    ctx.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()

#!/usr/bin/env python3
"""Benchmark: one step = one pass of the whole hot path (plan, unrank, semantic evaluation,
goal test, cost, compaction, ordering, top-k) over every query of the workload.

Prints ONE JSON line.  `value` is candidate programs resolved per second (valid or not, cost and
rank for the valid ones) by the library's default engine.  On this workload that is the
shared-prefix engine: the instructions that the candidates of a wavefront have in common are
applied once, so it carries out far fewer instruction applications than there are candidates.
The `roofline` object therefore prices the lane-operations that kernel really carried out
against the chip's 32-bit integer VALU rate (a small fraction: the kernel is bound by
bookkeeping and dependent lane exchanges, not by arithmetic), and `per_candidate_engine` reports
the engine that evaluates every candidate on its own, lane by lane, with its own roofline
fraction.  `cpu_baseline` times the plain CPU oracle on a bounded sample of the same candidates.
Queries of the batch whose reduction group, chunks, patterns, alphabet and size limit are equal are
evaluated once by the library (their costs stay their own): `config.queries_evaluated` says how many
were, and `every_query_evaluated` times the same batch with that switched off.
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# 32-bit integer lane-operations per second: 256 compute units x 128 lanes per clock x 2.4 GHz, the rate behind
# the published 157.3 TFLOP/s of fp32 vector arithmetic (one fused multiply-add = 2 flops per lane and clock).
# A stream of independent v_xor_b32 reaches about 0.8 of it (roofline.peak_measured, p2_measure_alu_peak).
ALU_PEAK_LANE_OPS = 256 * 128 * 2.4e9


def algorithmic_lane_ops(stats, n_chunks, key="member_visits"):
    """Lane-operations of instruction applications in the compact state form: every device taking part
    in an applied instruction has ceil(k/32) chunk-set words and ceil(R/32) mask words, and each word is
    read, tested against the rule's premise, folded into the group's result and written: 4 each.
    key = "member_visits": applications counted per candidate (what evaluating every candidate on its own
    executes); key = "members_evaluated": applications the engine really carried out."""
    words = -(-n_chunks // 32) + -(-stats["group_size"] // 32)
    return 4.0 * words * stats[key]


def measured_traffic(kernel):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 counter summary, or
    None when there is none or the kernel source has changed since the counters were taken."""
    path = os.path.join(ROOT, "profiles", "%s_cfg2_traffic.json" % kernel)
    src = os.path.join(ROOT, "paper_2110_10548_amd", "csrc",
                       {"k_eval_shared": "p2_shared.hip", "k_eval_regs": "p2_regs.hip", "k_eval_compact": "p2_compact.hip"}.get(kernel, "p2_literal.hip"))
    try:
        rec = json.load(open(path))
        if rec["source_sha256"] != hashlib.sha256(open(src, "rb").read()).hexdigest():
            return None
        return rec["hbm_bytes_per_launch"]
    except (OSError, KeyError, ValueError):
        return None


def cpu_baseline(queries, budget_s=15.0):
    """The oracle as it stands: flat, unpruned evaluation of a bounded sample of each query's
    candidate indices (the first S and S seeded-random ones; all of them where the space is smaller),
    OpenMP over all host cores this process may use."""
    import numpy as np
    from oracle import p2_oracle
    from paper_2110_10548_amd.workloads import SplitMix64
    cores = min(len(os.sched_getaffinity(0)), int(os.environ.get("OMP_NUM_THREADS", "1024")))
    S = 1_000_000
    total, t_all, t_one, n_one = 0, 0.0, 0.0, 0
    t_begin = time.time()
    for qi, q in enumerate(queries):
        oq = p2_oracle.Query(q["card"], q["axes"], q["placement"], q["reduce_axes"], bw=q["bw"], alpha=q["alpha"],
                             n_chunks=q.get("n_chunks", 0))
        N = oq.num_candidates(q["max_len"])
        if N <= 2 * S:
            idx = np.arange(N, dtype=np.uint64)
        else:
            rng = SplitMix64(1000 + qi)
            idx = np.concatenate([np.arange(S, dtype=np.uint64),
                                  np.array([rng.below(N) for _ in range(S)], dtype=np.uint64)])
        t0 = time.time()
        oq.eval_indices(q["max_len"], indices=idx, n_threads=cores)
        t_all += time.time() - t0
        total += len(idx)
        sub = idx[::16]
        t0 = time.time()
        oq.eval_indices(q["max_len"], indices=sub, n_threads=1)
        t_one += time.time() - t0
        n_one += len(sub)
        if time.time() - t_begin > 2 * budget_s:
            break
    # the oracle's enumeration by size with pruning (Sec. 3.5), single-threaded, over whole queries: the
    # CPU counterpart of an engine that settles candidates under an invalid prefix in bulk
    t_pruned, covered = 0.0, 0
    for q in queries:
        if time.time() - t_begin > 3 * budget_s:
            break
        oq = p2_oracle.Query(q["card"], q["axes"], q["placement"], q["reduce_axes"], bw=q["bw"], alpha=q["alpha"],
                             n_chunks=q.get("n_chunks", 0))
        t0 = time.time()
        oq.synthesize(q["max_len"], q.get("msg_bytes", ()))
        t_pruned += time.time() - t0
        covered += oq.num_candidates(q["max_len"])
    return {"value": total / t_all, "unit": "candidates/s", "cores": cores, "kind": "oracle",
            "value_1core": n_one / t_one,
            "pruned_enumeration_candidates_covered_per_s_1core": covered / t_pruned if t_pruned > 0 else None,
            "sample": "per query the first %d and %d SplitMix64-random candidate indices (the whole space where "
                      "smaller), flat unpruned evaluation from the init state; %d candidates in %.1f s" % (S, S, total, t_all)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, help="workload configuration 1..5 (2 is the benchmark)")
    ap.add_argument("--engine", type=int, default=0,
                    help="0 auto, 1 literal, 2 compact (state in LDS), 3 frontier, 4 small-group, 5 shared-prefix")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle leg")
    ap.add_argument("--no-compare", action="store_true", help="skip the leg that evaluates every query on its own (profiling runs)")
    ap.add_argument("--copy-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB (calibration of HBM byte counters under rocprofv3)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: candidate evaluation is embarrassingly parallel and the library "
              "runs on a single MI355X; --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2110_10548_amd import binding as B, workloads
    if not torch.cuda.is_available():
        print("no GPU visible: the evaluator has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    cfg = workloads.config(args.config)
    queries = workloads.expand(cfg, B.p2_enumerate_placements(cfg["card"], cfg["axes"]))
    msg = cfg["msg_bytes"]
    B.p2_set_profiling(True)

    if args.copy_mib > 0:
        src = torch.ones(args.copy_mib << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)                            # reads and writes copy_mib MiB each
        torch.cuda.synchronize()
        del src, dst
    def timed(engine, steps, warmup, flags=0):
        """K timed steps of the whole path with one engine: wall time, device times, results."""
        qs = [dict(q, engine=engine, flags=flags) for q in queries]
        batch = B.Batch(qs, msg)                  # argument marshalling only; every step replans on the host
        for _ in range(max(warmup, 1)):
            batch.run_raw()
        torch.cuda.synchronize()
        eval_ms, post_ms, launches = 0.0, 0.0, 0
        t0 = time.perf_counter()
        for _ in range(steps):
            batch.run_raw()                       # one p2_synthesize_batch call; returns after its stream sync
            prof = B.p2_get_profile()
            eval_ms += prof["eval_ms"]
            post_ms += prof["post_ms"]
            launches += prof["eval_launches"]
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        return {"dt": dt, "eval_ms": eval_ms, "post_ms": post_ms, "launches": launches, "results": batch.results(), "steps": steps}

    def summarise(run, key):
        """Throughput and the evaluation kernel's lane-operation rate; key selects which applications count."""
        results = run["results"]
        candidates = sum(r["stats"]["candidates"] for r in results)
        ops = sum(algorithmic_lane_ops(r["stats"], q["n_chunks"] or int(torch.tensor(q["card"]).prod()), key)
                  for q, r in zip(queries, results))
        launch_ms = run["eval_ms"] / max(run["launches"], 1)
        ops_per_launch = ops / (run["launches"] / run["steps"])
        return candidates, ops_per_launch, launch_ms, ops_per_launch / (launch_ms * 1e-3)

    peak_measured = B.p2_measure_alu_peak(5)        # independent v_xor_b32 stream, lane-operations per second
    KERNEL = {1: "k_eval_literal", 2: "k_eval_compact", 4: "k_eval_regs", 5: "k_eval_shared", 3: "k_front_classify"}
    run = timed(args.engine, args.steps, args.warmup)
    results = run["results"]
    dt = run["dt"]
    engines = sorted({r["stats"]["engine"] for r in results})
    kernel = KERNEL[max(engines, key=lambda e: sum(r["stats"]["candidates"] for r in results if r["stats"]["engine"] == e))]
    steps_exec = sum(r["stats"]["steps_executed"] for r in results)
    steps_eval = sum(r["stats"]["steps_evaluated"] for r in results)
    valid = sum(r["stats"]["valid"] for r in results)
    reruns = sum(r["stats"]["literal_reruns"] for r in results)
    candidates, ops_launch, launch_ms, achieved = summarise(run, "members_evaluated")
    _, flat_ops_launch, _, flat_rate = summarise(run, "member_visits")
    ms_per_step = dt / args.steps * 1e3
    eval_ms, post_ms = run["eval_ms"], run["post_ms"]

    out = {
        "metric": "candidate programs evaluated/sec (validity+cost)",
        "value": candidates / (dt / args.steps),
        "unit": "candidates/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32", "data": "synthetic",
        "config": {"workload": "%s: hierarchy %s, axes %s, all %d placements x reduce sets %s, max_len %d, %d message sizes"
                               % (cfg["name"], cfg["card"], cfg["axes"], len(queries) // max(len(cfg["reduce_sets"]) * len(cfg["n_chunks"]), 1),
                                  cfg["reduce_sets"], cfg["max_len"], len(msg)),
                   "queries": len(queries), "candidates_per_step": candidates, "valid_per_step": valid,
                   "steps_executed_per_step": steps_exec, "steps_evaluated_per_step": steps_eval,
                   "literal_reruns_per_step": reruns,
                   "engine": {0: "auto", 1: "literal", 2: "compact", 3: "frontier", 4: "small-group", 5: "shared-prefix"}[args.engine],
                   "engines_used": engines},
        "device_ms_per_step": {"evaluate": eval_ms / args.steps, "order_cost_topk": post_ms / args.steps},
        "evaluate_only_candidates_per_s": candidates / (eval_ms / args.steps * 1e-3),
        "steps_executed_per_s": steps_exec / (eval_ms / args.steps * 1e-3),
        "steps_evaluated_per_s": steps_eval / (eval_ms / args.steps * 1e-3),
        # lane-operations of the instruction applications the kernel carried out (shared ones once)
        "roofline": {"bound": "alu", "achieved": achieved / 1e12, "peak": ALU_PEAK_LANE_OPS / 1e12, "unit": "Tlane-op/s",
                     "frac": achieved / ALU_PEAK_LANE_OPS, "peak_measured": peak_measured / 1e12,
                     "traffic": measured_traffic(kernel) if args.config == 2 else None,
                     "kernel": kernel,
                     "launch_ms": launch_ms, "algorithmic_lane_ops_per_launch": ops_launch,
                     # the same launch priced with every candidate's applications counted on their own
                     "per_candidate_lane_ops_per_launch": flat_ops_launch,
                     "per_candidate_equivalent_frac": flat_rate / ALU_PEAK_LANE_OPS},
    }
    # Queries of the batch with the same reduction group, chunks, patterns, alphabet and size limit are evaluated
    # once (validity does not depend on the links or on where the placement puts the group); every query is still
    # costed on its own.  The same batch with that switched off, for comparison:
    out["config"]["queries_evaluated"] = sum(1 for r in results if r["stats"]["steps_evaluated"] > 0) if engines == [5] else None
    if args.engine == 0 and 3 not in engines and not args.no_compare:
        every = timed(args.engine, max(args.steps // 2, 2), 2, B.FLAG_EVALUATE_EVERY_QUERY)
        out["every_query_evaluated"] = {"value": candidates / (every["dt"] / every["steps"]), "unit": "candidates/s",
                                        "ms_per_step": every["dt"] / every["steps"] * 1e3, "steps": every["steps"],
                                        "device_ms_per_step": {"evaluate": every["eval_ms"] / every["steps"],
                                                               "order_cost_topk": every["post_ms"] / every["steps"]}}
    if 3 in engines:
        # the frontier engine's time is spread over many launches per query outside the evaluation events, and
        # its work is pruned enumeration, not candidates visited: no lane-operation rate is quoted for it
        for key in ("achieved", "frac", "launch_ms", "per_candidate_equivalent_frac"):
            out["roofline"][key] = None
    if 5 in engines and args.engine == 0 and candidates <= 1 << 30:
        # the engine that evaluates every candidate on its own, timed the same way (fewer steps)
        every_q = B.FLAG_EVALUATE_EVERY_QUERY           # (this leg is about the kernel: every candidate is visited)
        try:
            own, own_engine = timed(4, max(args.steps // 2, 2), 2, every_q), 4
        except B.P2Error:                          # more than 32 devices or chunks: the LDS-resident compact engine
            try:
                own, own_engine = timed(2, max(args.steps // 10, 1), 1, every_q), 2
            except B.P2Error:                      # too many candidates to visit one by one (config 5)
                own = None
    else:
        own = None
    if own is not None:
        c2, ops2, ms2, rate2 = summarise(own, "member_visits")
        out["per_candidate_engine"] = {
            "engine": {4: "small-group", 2: "compact"}[own_engine], "kernel": KERNEL[own_engine],
            "value": c2 / (own["dt"] / own["steps"]), "unit": "candidates/s",
            "ms_per_step": own["dt"] / own["steps"] * 1e3, "steps": own["steps"],
            "roofline": {"bound": "alu", "achieved": rate2 / 1e12, "peak": ALU_PEAK_LANE_OPS / 1e12, "unit": "Tlane-op/s",
                         "frac": rate2 / ALU_PEAK_LANE_OPS, "launch_ms": ms2, "algorithmic_lane_ops_per_launch": ops2,
                         "traffic": measured_traffic(KERNEL[own_engine]) if args.config == 2 else None}}
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(queries)
    print(json.dumps(out))


if __name__ == "__main__":
    main()

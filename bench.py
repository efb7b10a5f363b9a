#!/usr/bin/env python3
"""Benchmark: one step = one pass of the whole hot path (plan, unrank, semantic evaluation,
goal test, cost, compaction, ordering, top-k) over every query of the workload: one
p2_synthesize_batch call.

Prints ONE JSON line.  The default workload is configuration 5, the largest (512 devices, 512
queries, programs of up to six instructions): its candidate spaces (up to 2.65e11 programs per
query) are resolved by enumeration by program size with pruning (Sec. 3.5), the frontier engine.
`value` counts the candidate programs whose status (valid or not; cost and rank for the valid
ones) one step settles, per second, and counts a query's candidate space only where the library
evaluated that query itself: queries of the batch whose validity results are equal by construction
(same reduction group, chunks, patterns, alphabet, size limit) are enumerated once and only costed
on their own (`config.queries_evaluated` of `config.queries`; `value_all_queries` counts every query).

`roofline` prices the dominant kernel family of the step.  For the frontier engine that is the
classification of the states of valid prefixes against every instruction of the alphabet
(k_front_classify; prefixes that end in the same state share one classification:
`states_judged_per_step` of `prefixes_per_step`): its algorithmic work per judged state is 4
lane-operations (read, union, intersection / seen-twice, compare) per 32-bit word of the (chunk
set, mask) pairs of every device that a pattern of the alphabet visits, set against the chip's
32-bit integer vector rate (`per_prefix_equivalent_frac` prices the same time as if every prefix had
been judged on its own); the same words are read from LDS once per pattern (`roofline.lds`, against
256 bytes per clock and compute unit) and the state comes from device memory once (`roofline.hbm`).
`materialize` prices the kernel that builds the children of the judged states against HBM.  Times
are HIP-event times around every launch of the family on the stream it is launched on, taken inside
the timed steps (p2_get_profile; the timed steps bracket these two families only, p2_set_profiling(2):
event pairs around every group of the engine's small launches as well cost 7 % of a call, and are
taken in the one-at-a-time leg, whose device_ms_per_step has the full breakdown).  The library runs up to four enumerations of a batch side by
side, so those are times of kernels that share the chip, and an event pair on one stream also sees
the time its kernel waits for a turn behind the other streams' kernels, which a profiler's kernel
duration does not; `one_enumeration_at_a_time` gives the same objects for a few steps with the
enumerations one after the other (there the two agree), and `--one-at-a-time` times the whole run so.
For the flat engines (configurations 1-4 with the default engine) the roofline is the lane-operation
rate of the evaluation kernel, as `other_configs` reports per configuration.
`cpu_baseline` times the plain CPU oracle on a bounded sample of the same workload.
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
# local data share: 256 bytes per clock and compute unit with 128-bit reads (a read stream reaches 0.98 of it:
# roofline.lds.peak_measured, p2_measure_lds_peak)
LDS_PEAK_BYTES = 256 * 256 * 2.4e9
HBM_PEAK_BYTES = 8.0e12

ENGINE_NAMES = {0: "auto", 1: "literal", 2: "compact", 3: "frontier", 4: "small-group", 5: "shared-prefix"}
KERNEL = {1: "k_eval_literal", 2: "k_eval_compact", 4: "k_eval_regs", 5: "k_eval_shared", 3: "k_front_classify"}
KERNEL_SOURCE = {"k_eval_shared": "p2_shared.hip", "k_eval_regs": "p2_regs.hip", "k_eval_compact": "p2_compact.hip",
                 "k_front_classify": "p2_frontier.hip", "k_front_materialize": "p2_frontier.hip"}


def algorithmic_lane_ops(stats, n_chunks, key="member_visits"):
    """Lane-operations of instruction applications in the compact state form: every device taking part
    in an applied instruction has ceil(k/32) chunk-set words and ceil(R/32) mask words, and each word is
    read, tested against the rule's premise, folded into the group's result and written: 4 each.
    key = "member_visits": applications counted per candidate (what evaluating every candidate on its own
    executes); key = "members_evaluated": applications the engine really carried out."""
    words = -(-n_chunks // 32) + -(-stats["group_size"] // 32)
    return 4.0 * words * stats[key]


def measured_traffic(kernel, cfg_index):
    """HBM bytes per launch of a kernel family from the committed rocprofv3 counter summary, or None when
    there is none or the kernel source has changed since the counters were taken."""
    path = os.path.join(ROOT, "profiles", "%s_cfg%d_traffic.json" % (kernel, cfg_index))
    src = os.path.join(ROOT, "paper_2110_10548_amd", "csrc", KERNEL_SOURCE.get(kernel, "p2_literal.hip"))
    try:
        rec = json.load(open(path))
        if rec["source_sha256"] != hashlib.sha256(open(src, "rb").read()).hexdigest():
            return None
        return rec["hbm_bytes_per_launch"]
    except (OSError, KeyError, ValueError):
        return None


def oracle_build_flags():
    """The gcc command line the oracle library is built with (read from its build script)."""
    try:
        import re
        text = open(os.path.join(ROOT, "oracle", "build.py")).read()
        m = re.search(r'cmd = \[(.*?)\]', text, re.S)
        return " ".join(t for t in re.findall(r'"([^"]+)"', m.group(1)) if t != "-o") if m else None
    except OSError:
        return None


def cpu_baseline(queries, budget_s=12.0):
    """The oracle as it stands, on a bounded sample of the workload, OpenMP over the host cores this
    process may use: flat, unpruned evaluation of seeded-random candidate indices of queries spread
    over the batch, sized from a short probe so that it takes about budget_s; and, single-threaded,
    the oracle's own enumeration by size with pruning (Sec. 3.5) of whole queries, smallest spaces
    first, while the budget lasts."""
    import numpy as np
    from oracle import p2_oracle
    from paper_2110_10548_amd.workloads import SplitMix64
    cores = min(len(os.sched_getaffinity(0)), int(os.environ.get("OMP_NUM_THREADS", "1024")))

    def oracle_query(q):
        return p2_oracle.Query(q["card"], q["axes"], q["placement"], q["reduce_axes"], bw=q["bw"], alpha=q["alpha"],
                               n_chunks=q.get("n_chunks", 0))

    picks = list(range(0, len(queries), max(len(queries) // 8, 1)))[:8]
    oqs = [(qi, oracle_query(queries[qi])) for qi in picks]

    def sample(qi, oq, n):
        N = oq.num_candidates(queries[qi]["max_len"])
        if N <= n:
            return np.arange(N, dtype=np.uint64)
        rng = SplitMix64(1000 + qi)
        return np.array([rng.below(N) for _ in range(n)], dtype=np.uint64)

    # probe: a few candidates per picked query
    t0 = time.time()
    probe = 0
    for qi, oq in oqs:
        idx = sample(qi, oq, 4 * cores)
        oq.eval_indices(queries[qi]["max_len"], indices=idx, n_threads=cores)
        probe += len(idx)
    t_probe = max(time.time() - t0, 1e-6)
    per_query = int(min(max(budget_s / t_probe * 4 * cores, 4 * cores), 1_000_000))
    total, t_all = 0, 0.0
    for qi, oq in oqs:
        idx = sample(qi, oq, per_query)
        t0 = time.time()
        oq.eval_indices(queries[qi]["max_len"], indices=idx, n_threads=cores)
        t_all += time.time() - t0
        total += len(idx)
        if t_all > 2 * budget_s:
            break
    # pruned enumeration of whole queries, one core, smallest candidate spaces first
    order = sorted(range(len(queries)), key=lambda i: (oracle_query(queries[i]).num_candidates(queries[i]["max_len"]), i))
    t_pruned, covered, n_pruned, seen = 0.0, 0, 0, set()
    for i in order:
        q = queries[i]
        key = (tuple(map(tuple, q["placement"])), tuple(q["reduce_axes"]), q.get("n_chunks", 0))
        if key in seen:
            continue
        seen.add(key)
        if t_pruned > budget_s:
            break
        oq = oracle_query(q)
        t0 = time.time()
        oq.synthesize(q["max_len"], q.get("msg_bytes", ()))
        t_pruned += time.time() - t0
        covered += oq.num_candidates(q["max_len"])
        n_pruned += 1
        if oq.num_candidates(q["max_len"]) > 1_000_000:      # (one large space is enough: the next ones take minutes)
            break
    return {"value": total / t_all, "unit": "candidates/s", "cores": cores, "kind": "oracle",
            "nproc": os.cpu_count(), "build": oracle_build_flags(),
            "pruned_enumeration_candidates_covered_per_s_1core": covered / t_pruned if t_pruned > 0 else None,
            "sample": "flat unpruned evaluation from the init state of %d SplitMix64-random candidate indices of each of the "
                      "queries %s (%d candidates in %.1f s, %d threads); pruned enumeration of the %d distinct queries with the "
                      "smallest candidate spaces, 1 thread, %.1f s" % (per_query, picks, total, t_all, cores, n_pruned, t_pruned)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=5, help="workload configuration 1..5 (5, the largest, is the benchmark)")
    ap.add_argument("--engine", type=int, default=0,
                    help="0 auto, 1 literal, 2 compact (state in LDS), 3 frontier, 4 small-group, 5 shared-prefix")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle leg")
    ap.add_argument("--no-compare", action="store_true", help="skip the legs that run other engines or other configurations (profiling runs)")
    ap.add_argument("--one-at-a-time", action="store_true",
                    help="time the steps with the enumerations of a batch one after the other (P2_FLAG_ONE_ENUMERATION_AT_A_TIME): "
                         "every kernel then has the chip to itself, which is the setting in which an event time around a launch "
                         "and a profiler's kernel duration are the same thing")
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
    B.p2_set_profiling(True)

    if args.copy_mib > 0:
        src = torch.ones(args.copy_mib << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)                            # reads and writes copy_mib MiB each
        torch.cuda.synchronize()
        del src, dst

    PROFILE_SUMS = ("eval_ms", "post_ms", "eval_launches", "front_ms", "front_classify_ms", "front_literal_ms",
                    "front_materialize_ms", "front_group_ms", "front_entries", "front_classify_launches", "front_literal_launches", "front_materialize_launches",
                    "front_prefixes", "front_classify_state_bytes", "front_classify_lane_ops", "front_survivors",
                    "front_materialize_bytes")

    def load(cfg_index):
        cfg = workloads.config(cfg_index)
        return cfg, workloads.expand(cfg, B.p2_enumerate_placements(cfg["card"], cfg["axes"]))

    def timed(queries, msg, engine, steps, warmup, flags=0, every_span=True):
        """K timed steps of the whole path with one engine: wall time, device times, results.
        every_span=False: of the frontier engine's launches only the classification and the building of the
        children are bracketed by events (the two kernels the roofline objects are about): the event pairs around
        its many small launches cost several per cent of a call on a large batch."""
        B.p2_set_profiling(True if every_span else 2)
        qs = [dict(q, engine=engine, flags=flags) for q in queries]
        batch = B.Batch(qs, msg)                  # argument marshalling only; every step replans on the host
        for _ in range(max(warmup, 1)):
            batch.run_raw()
        torch.cuda.synchronize()
        acc = {k: 0.0 for k in PROFILE_SUMS}
        t0 = time.perf_counter()
        for _ in range(steps):
            batch.run_raw()                       # one p2_synthesize_batch call; returns after its stream sync
            prof = B.p2_get_profile()
            for k in PROFILE_SUMS:
                acc[k] += prof[k]
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        return dict(acc, dt=dt, results=batch.results(), steps=steps, queries=queries)

    def flat_summary(run, key):
        """Lane-operation rate of the flat engines' evaluation kernel; key selects which applications count."""
        results, queries = run["results"], run["queries"]
        ops = sum(algorithmic_lane_ops(r["stats"], q["n_chunks"] or int(torch.tensor(q["card"]).prod()), key)
                  for q, r in zip(queries, results))
        launches = max(run["eval_launches"], 1)
        launch_ms = run["eval_ms"] / launches
        ops_per_launch = ops / (launches / run["steps"])
        return ops_per_launch, launch_ms, ops_per_launch / (launch_ms * 1e-3)

    def report(run, cfg_index, engine_asked):
        """The figures of one timed run: throughput, device times, roofline of its dominant kernel family."""
        results, steps = run["results"], run["steps"]
        step_s = run["dt"] / steps
        own = [r for r in results if r["stats"]["evaluated_with"] < 0]
        candidates_all = sum(r["stats"]["candidates"] for r in results)
        candidates = sum(r["stats"]["candidates"] for r in own)
        engines = sorted({r["stats"]["engine"] for r in results})
        main_engine = max(engines, key=lambda e: sum(r["stats"]["candidates"] for r in own if r["stats"]["engine"] == e))
        out = {"value": candidates / step_s, "unit": "candidates/s", "value_all_queries": candidates_all / step_s,
               "ms_per_step": step_s * 1e3, "steps": steps,
               "queries": len(results), "queries_evaluated": len(own),
               "candidates_per_step": candidates, "candidates_per_step_all_queries": candidates_all,
               "valid_per_step": sum(r["stats"]["valid"] for r in results),
               "engine": ENGINE_NAMES[engine_asked], "engines_used": engines,
               "device_ms_per_step": {"evaluate": run["eval_ms"] / steps, "frontier": run["front_ms"] / steps,
                                      "order_cost_topk": run["post_ms"] / steps}}
        if main_engine == 3:
            cls_s = run["front_classify_ms"] * 1e-3
            n_launch = max(run["front_classify_launches"], 1)
            rate = run["front_classify_lane_ops"] / cls_s
            lds_rate = run["front_classify_lane_ops"] / cls_s           # 4 lane-operations per 4-byte word read from LDS
            hbm_rate = run["front_classify_state_bytes"] / cls_s
            mat_s = max(run["front_materialize_ms"] * 1e-3, 1e-12)
            out["states_judged_per_step"] = run["front_prefixes"] / steps
            out["prefixes_per_step"] = run["front_entries"] / steps
            out["states_judged_per_s"] = run["front_prefixes"] / cls_s
            out["device_ms_per_step"].update({"front_classify": run["front_classify_ms"] / steps,
                                              "front_materialize": run["front_materialize_ms"] / steps})
            if run["front_group_ms"] > 0.0:          # (the timed steps of the default run do not bracket these launches)
                out["device_ms_per_step"].update({"front_literal": run["front_literal_ms"] / steps,
                                                  "front_group_and_list": run["front_group_ms"] / steps})
            out["roofline"] = {
                "bound": "alu", "kernel": "k_front_classify", "achieved": rate / 1e12, "peak": ALU_PEAK_LANE_OPS / 1e12,
                "unit": "Tlane-op/s", "frac": rate / ALU_PEAK_LANE_OPS,
                "traffic": measured_traffic("k_front_classify", cfg_index),
                "launch_ms": run["front_classify_ms"] / n_launch, "launches_per_step": n_launch / steps,
                "algorithmic_lane_ops_per_launch": run["front_classify_lane_ops"] / n_launch,
                "algorithmic_hbm_bytes_per_launch": run["front_classify_state_bytes"] / n_launch,
                "lds": {"achieved": lds_rate / 1e9, "peak": LDS_PEAK_BYTES / 1e9, "unit": "GB/s", "frac": lds_rate / LDS_PEAK_BYTES},
                "hbm": {"achieved": hbm_rate / 1e9, "peak": HBM_PEAK_BYTES / 1e9, "unit": "GB/s", "frac": hbm_rate / HBM_PEAK_BYTES},
                "per_prefix_equivalent_frac": rate / ALU_PEAK_LANE_OPS * run["front_entries"] / max(run["front_prefixes"], 1.0),
                "share_of_device_time": run["front_classify_ms"] / max(run["front_ms"] + run["post_ms"] + run["eval_ms"], 1e-9)}
            n_mat = max(run["front_materialize_launches"], 1)
            out["materialize"] = {
                "bound": "hbm", "kernel": "k_front_materialize", "achieved": run["front_materialize_bytes"] / mat_s / 1e9,
                "peak": HBM_PEAK_BYTES / 1e9, "unit": "GB/s", "frac": run["front_materialize_bytes"] / mat_s / HBM_PEAK_BYTES,
                "traffic": measured_traffic("k_front_materialize", cfg_index),
                "launch_ms": run["front_materialize_ms"] / n_mat, "launches_per_step": n_mat / steps,
                "algorithmic_hbm_bytes_per_launch": run["front_materialize_bytes"] / n_mat,
                "children_per_step": run["front_survivors"] / steps}
        else:
            kernel = KERNEL[main_engine]
            ops_launch, launch_ms, achieved = flat_summary(run, "members_evaluated")
            flat_ops_launch, _, flat_rate = flat_summary(run, "member_visits")
            out["steps_executed_per_step"] = sum(r["stats"]["steps_executed"] for r in own)
            out["steps_evaluated_per_step"] = sum(r["stats"]["steps_evaluated"] for r in own)
            # lane-operations of the instruction applications the kernel carried out (shared ones once)
            out["roofline"] = {"bound": "alu", "kernel": kernel, "achieved": achieved / 1e12, "peak": ALU_PEAK_LANE_OPS / 1e12,
                               "unit": "Tlane-op/s", "frac": achieved / ALU_PEAK_LANE_OPS,
                               "traffic": measured_traffic(kernel, cfg_index),
                               "launch_ms": launch_ms, "algorithmic_lane_ops_per_launch": ops_launch,
                               # the same launch priced with every candidate's applications counted on their own
                               "per_candidate_lane_ops_per_launch": flat_ops_launch,
                               "per_candidate_equivalent_frac": flat_rate / ALU_PEAK_LANE_OPS}
        return out

    cfg, queries = load(args.config)
    msg = cfg["msg_bytes"]
    peak_measured = B.p2_measure_alu_peak(5)        # independent v_xor_b32 stream, lane-operations per second
    lds_measured = B.p2_measure_lds_peak(5)         # 128-bit LDS reads, bytes per second
    run = timed(queries, msg, args.engine, args.steps, args.warmup, B.FLAG_ONE_ENUMERATION_AT_A_TIME if args.one_at_a_time else 0,
                every_span=args.one_at_a_time)
    head = report(run, args.config, args.engine)
    placements = len({q["placement_index"] for q in queries})
    if cfg["placements"] == "all":
        what = "all %d placements x reduce sets %s x chunk counts %s" % (placements, cfg["reduce_sets"], cfg["n_chunks"])
    else:
        what = ("%d (placement, reduce-axis subset) draws with replacement, seed %d: %d of the %d placements, %d distinct queries"
                % (len(queries), cfg["seed"], placements, len(B.p2_enumerate_placements(cfg["card"], cfg["axes"])),
                   len({(q["placement_index"], tuple(q["reduce_axes"])) for q in queries})))
    out = {
        "metric": "candidate programs evaluated/sec (validity+cost)",
        "value": head["value"], "unit": "candidates/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32", "data": "synthetic",
        "config": {"workload": "%s: hierarchy %s, axes %s, %s, max_len %d, top-%d, %d message size(s)"
                               % (cfg["name"], cfg["card"], cfg["axes"], what, cfg["max_len"], cfg["topk"], len(msg)),
                   "queries": head["queries"], "queries_evaluated": head["queries_evaluated"],
                   "candidates_per_step": head["candidates_per_step"],
                   "candidates_per_step_all_queries": head["candidates_per_step_all_queries"],
                   "valid_per_step": head["valid_per_step"], "engine": head["engine"], "engines_used": head["engines_used"]},
        "value_all_queries": head["value_all_queries"],
        "device_ms_per_step": head["device_ms_per_step"],
        "roofline": dict(head["roofline"], peak_measured=peak_measured / 1e12),
    }
    if "lds" in out["roofline"]:
        out["roofline"]["lds"]["peak_measured"] = lds_measured / 1e9
    for key in ("materialize", "states_judged_per_step", "prefixes_per_step", "states_judged_per_s", "steps_executed_per_step",
                "steps_evaluated_per_step"):
        if key in head:
            out[key] = head[key]
    if args.one_at_a_time:
        out["config"]["enumerations"] = "one at a time"
    if 3 in head["engines_used"] and not args.no_compare and not args.one_at_a_time:
        # The timed steps run up to four enumerations side by side, so the event time of a launch there is the time of
        # a kernel that shares the chip.  The same batch with the enumerations one after the other, a few steps: what
        # the kernels reach with the chip to themselves.
        alone = report(timed(queries, msg, args.engine, max(args.steps // 5, 2), 1, B.FLAG_ONE_ENUMERATION_AT_A_TIME), args.config, args.engine)
        out["one_enumeration_at_a_time"] = {"ms_per_step": alone["ms_per_step"], "steps": alone["steps"],
                                            "device_ms_per_step": alone["device_ms_per_step"], "roofline": alone["roofline"],
                                            "materialize": alone["materialize"]}
        # (beside the timed figure, for a reader of the roofline object alone)
        out["roofline"]["frac_one_enumeration_at_a_time"] = alone["roofline"]["frac"]
        out["roofline"]["enumerations_side_by_side"] = 4

    if not args.no_compare:
        # the other configurations, a few steps each with the default engine, and where that is the shared-prefix
        # engine also the engine that evaluates every candidate on its own, lane by lane
        others = {}
        for ci in (1, 2, 3, 4, 5):
            if ci == args.config:
                continue
            c2, q2 = load(ci)
            steps2 = 3 if ci == 5 else 10
            r2 = report(timed(q2, c2["msg_bytes"], 0, steps2, 2), ci, 0)
            entry = {k: r2[k] for k in ("value", "unit", "value_all_queries", "ms_per_step", "steps", "queries", "queries_evaluated",
                                        "candidates_per_step", "valid_per_step", "engines_used", "device_ms_per_step", "roofline")}
            if r2["engines_used"] == [5] and r2["candidates_per_step"] <= 1 << 30:
                every_q = B.FLAG_EVALUATE_EVERY_QUERY           # (this leg is about the kernel: every candidate is visited)
                own, own_engine = None, None
                for eng, st in ((4, 5), (2, 2)):                # small-group engine; else the LDS-resident compact engine
                    try:
                        own, own_engine = timed(q2, c2["msg_bytes"], eng, st, 1, every_q), eng
                        break
                    except B.P2Error:
                        continue
                if own is not None:
                    ops2, ms2, rate2 = flat_summary(own, "member_visits")
                    c_all = sum(r["stats"]["candidates"] for r in own["results"])
                    entry["per_candidate_engine"] = {
                        "engine": ENGINE_NAMES[own_engine], "kernel": KERNEL[own_engine],
                        "value": c_all / (own["dt"] / own["steps"]), "unit": "candidates/s",
                        "ms_per_step": own["dt"] / own["steps"] * 1e3, "steps": own["steps"],
                        "roofline": {"bound": "alu", "achieved": rate2 / 1e12, "peak": ALU_PEAK_LANE_OPS / 1e12, "unit": "Tlane-op/s",
                                     "frac": rate2 / ALU_PEAK_LANE_OPS, "launch_ms": ms2, "algorithmic_lane_ops_per_launch": ops2,
                                     "traffic": measured_traffic(KERNEL[own_engine], ci)}}
            others[c2["name"]] = entry
        out["other_configs"] = others
        # flat evaluation outside the power-of-two fast paths: a hierarchy with levels of 3 and 6 (72 devices) and a
        # reduction group of 128 devices, every candidate visited by the LDS-resident compact engine
        paths = {}
        for name, card, bw, alpha in (("radix_3_4_6", [3, 4, 6], [25e9, 100e9, 300e9], [20e-6, 10e-6, 5e-6]),
                                      ("r128_compact", [2, 8, 8], [25e9, 100e9, 300e9], [20e-6, 10e-6, 5e-6])):
            devices = card[0] * card[1] * card[2]
            q = dict(card=card, bw=bw, alpha=alpha, axes=[devices], placement=[card], placement_index=0, reduce_axes=[0],
                     max_len=4, n_chunks=0, topk=0)
            try:
                r = timed([q], [float(1 << 26)], 2, 3, 1, B.FLAG_EVALUATE_EVERY_QUERY)
            except B.P2Error as e:
                paths[name] = {"error": str(e)}
                continue
            ops, launch_ms, rate = flat_summary(r, "member_visits")
            st = r["results"][0]["stats"]
            paths[name] = {"hierarchy": card, "devices": devices, "engine": ENGINE_NAMES[st["engine"]], "kernel": KERNEL[st["engine"]],
                           "candidates_per_step": st["candidates"], "valid_per_step": st["valid"],
                           "value": st["candidates"] / (r["dt"] / r["steps"]), "unit": "candidates/s",
                           "ms_per_step": r["dt"] / r["steps"] * 1e3, "steps": r["steps"],
                           "roofline": {"bound": "alu", "achieved": rate / 1e12, "peak": ALU_PEAK_LANE_OPS / 1e12, "unit": "Tlane-op/s",
                                        "frac": rate / ALU_PEAK_LANE_OPS, "launch_ms": launch_ms, "algorithmic_lane_ops_per_launch": ops}}
        out["other_paths"] = paths
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(queries)
    print(json.dumps(out))


if __name__ == "__main__":
    main()

"""Placement-level search, written out plainly on top of the oracle's per-placement synthesis.

TEST INFRASTRUCTURE (see p2_oracle.py): only tests, the smoke check and the benchmark's
CPU-baseline leg may import this module.

What it states (Sec. 4.1, Results 1 and 4 of the evaluation; Sec. 2.2 for the outer loop): the tool
goes through every parallelism matrix of a system, and for each of them through every requested
reduction; for one (matrix, reduction) pair it synthesizes all valid programs and simulates them.
The figures the paper compares are, per pair, the time of the single AllReduce over the whole
reduction group and the time of the best synthesized program; and a mapping has to be chosen with
all of a model's reductions in view, which is taken here as the weighted sum of the best times.
"""
import math

from . import p2_oracle as O

AR = 0


def search_placements(card, axes, reduce_sets, max_len, msg_bytes, bw=None, alpha=None, weights=None, n_chunks=0,
                      form_mask=7, op_mask=31, algo=0):
    """Returns {"placements": [...], "rows": {(p, s): {...}}, "total": [...], "order": [...]}.

    rows[(p, s)]: valid = number of valid programs, best_index / best_instr / best_cost = the valid
    program with the smallest (cost, index), allreduce_cost = the one-instruction program AllReduce
    over the whole reduction group (always valid).  A reduction over a single device needs no
    program: valid 0, best_instr [], both costs 0.
    total[p] = sum_s weights[s] * best_cost(p, s); order = placements by ascending (total, p)."""
    placements = O.enumerate_placements(card, axes)
    weights = list(weights) if weights is not None else [1.0] * len(reduce_sets)
    rows, total = {}, []
    for p, x in enumerate(placements):
        acc = 0.0
        for s, red in enumerate(reduce_sets):
            q = O.Query(card, axes, x, red, bw=bw, alpha=alpha, n_chunks=n_chunks, form_mask=form_mask, op_mask=op_mask,
                        algo=algo)
            if q.alphabet == 0:
                rows[(p, s)] = {"valid": 0, "best_index": None, "best_instr": [], "best_cost": 0.0, "allreduce_cost": 0.0}
                continue
            r = q.synthesize(max_len, [msg_bytes])
            best = None
            for i in range(len(r["index"])):
                key = (float(r["cost"][i, 0]), int(r["index"][i]))
                if best is None or key < best[0]:
                    best = (key, i)
            # the baseline is always InsideGroup on the root slice, whatever masks the query has
            base = O.Query(card, axes, x, red, bw=bw, alpha=alpha, n_chunks=n_chunks, form_mask=1, op_mask=1, algo=algo)
            ok, c_ar, _ = base.eval_program([AR], [msg_bytes])
            assert ok
            row = {"valid": len(r["index"]), "allreduce_cost": float(c_ar[0])}
            if best is None:
                row.update(best_index=None, best_instr=[], best_cost=math.inf)
            else:
                i = best[1]
                row.update(best_index=int(r["index"][i]), best_instr=[int(v) for v in r["instr"][i][:r["len"][i]]],
                           best_cost=float(r["cost"][i, 0]))
            rows[(p, s)] = row
            acc += weights[s] * row["best_cost"]
        total.append(acc)
    order = sorted(range(len(placements)), key=lambda p: (total[p], p))
    return {"placements": [[[int(v) for v in r] for r in x] for x in placements], "rows": rows, "total": total,
            "order": order}

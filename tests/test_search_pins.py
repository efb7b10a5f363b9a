"""Pins of the oracle's placement-level search (oracle/p2_search.py): the qualitative results the paper
states for its evaluation (Sec. 4.1-4.2), closed forms, and brute force over every candidate."""
import numpy as np
import pytest

AR = 0
N26 = float(2 ** 26)
CARD, AXES = [2, 4], [2, 4]                  # 2 nodes of 4 devices; placements [[1,2],[2,2]] and [[2,1],[1,4]]
BW, ALPHA = [25e9, 300e9], [20e-6, 5e-6]


@pytest.fixture(scope="module")
def S():
    from oracle import p2_search
    return p2_search


def test_reduction_inside_a_node_is_best_done_by_one_allreduce(S, oracle):
    # Sec. 4.2, Result 3: if the reduction axes fit in one node, the single AllReduce is the best program
    r = S.search_placements(CARD, AXES, [[0], [1]], 4, N26, bw=BW, alpha=ALPHA)
    assert r["placements"] == [[[1, 2], [2, 2]], [[2, 1], [1, 4]]]
    for key, g in (((0, 0), 2), ((1, 1), 4)):
        row = r["rows"][key]
        assert row["best_instr"] == [AR] and row["best_index"] == 0
        assert row["best_cost"] == row["allreduce_cost"] == pytest.approx(2 * (g - 1) * 5e-6 + 2 * (g - 1) / g * N26 / 300e9, rel=1e-14)


def test_reduction_across_nodes_prefers_a_topology_aware_program(S):
    # Sec. 4.2, Result 5; and Result 1: the same reduction costs very different times on different matrices
    r = S.search_placements(CARD, AXES, [[1]], 4, N26, bw=BW, alpha=ALPHA)
    across, inside = r["rows"][(0, 0)], r["rows"][(1, 0)]
    assert len(across["best_instr"]) > 1 and across["best_cost"] < across["allreduce_cost"]
    assert inside["allreduce_cost"] < across["best_cost"]            # placement matters more than the program
    assert r["order"] == [1, 0]
    # reducing the other axis turns the ranking around (the remark that B3 is the better matrix for the other reduction)
    assert S.search_placements(CARD, AXES, [[0]], 4, N26, bw=BW, alpha=ALPHA)["order"] == [0, 1]


def test_all_reductions_of_a_model_decide_together(S):
    # Sec. 4.1: a mapping is selected with every reduction in view -> weighted sum of the best times
    a = S.search_placements(CARD, AXES, [[0], [1]], 4, N26, bw=BW, alpha=ALPHA)
    for p in range(2):
        assert a["total"][p] == pytest.approx(a["rows"][(p, 0)]["best_cost"] + a["rows"][(p, 1)]["best_cost"], rel=1e-15)
    assert a["order"] == [0, 1]
    b = S.search_placements(CARD, AXES, [[0], [1]], 4, N26, bw=BW, alpha=ALPHA, weights=[0.01, 1.0])
    assert b["order"] == [1, 0]
    assert b["total"][1] == pytest.approx(0.01 * b["rows"][(1, 0)]["best_cost"] + b["rows"][(1, 1)]["best_cost"], rel=1e-15)


def test_reducing_every_axis_makes_all_placements_equal(S):
    r = S.search_placements([2, 2, 4], [4, 4], [[0, 1]], 3, N26, bw=[25e9, 100e9, 300e9], alpha=[20e-6, 10e-6, 5e-6])
    assert len(r["placements"]) > 2
    first = r["rows"][(0, 0)]
    for p in range(len(r["placements"])):
        row = r["rows"][(p, 0)]
        assert row["valid"] == first["valid"] and row["best_index"] == first["best_index"]
        assert row["best_cost"] == pytest.approx(first["best_cost"], rel=1e-14)
    if len(set(r["total"])) == 1:
        assert r["order"] == list(range(len(r["placements"])))


def test_best_program_against_every_candidate_on_its_own(S, oracle):
    r = S.search_placements(CARD, AXES, [[1]], 3, N26, bw=BW, alpha=ALPHA, algo=1)
    for p, x in enumerate(r["placements"]):
        q = oracle.Query(CARD, AXES, x, [1], bw=BW, alpha=ALPHA, algo=1)
        best, valid = None, 0
        for idx in range(q.num_candidates(3)):
            ok, cost, _ = q.eval_program(q.unrank(3, idx), [N26])
            if ok:
                valid += 1
                if best is None or (cost[0], idx) < best:
                    best = (float(cost[0]), idx)
        row = r["rows"][(p, 0)]
        assert (row["valid"], row["best_cost"], row["best_index"]) == (valid, best[0], best[1])


def test_single_device_reduction_needs_no_program(S):
    r = S.search_placements([2, 4], [1, 8], [[0], [1]], 3, N26, bw=BW, alpha=ALPHA)
    for p in range(len(r["placements"])):
        assert r["rows"][(p, 0)] == {"valid": 0, "best_index": None, "best_instr": [], "best_cost": 0.0, "allreduce_cost": 0.0}
        assert r["total"][p] == r["rows"][(p, 1)]["best_cost"] > 0.0

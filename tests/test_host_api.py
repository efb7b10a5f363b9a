"""CPU-side checks of the C-ABI library: it loads, exports every declared symbol, and its
host-only entry points (placements, pattern description, argument errors) agree with the oracle.
No kernel is launched here."""
import ctypes
import itertools
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2110_10548_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    binding.lib()
    return binding


def test_every_declared_symbol_is_exported(B):
    header = open(os.path.join(ROOT, "include", "p2.h")).read()
    declared = set(re.findall(r"\b(p2_[a-z_]+)\s*\(", header))
    declared -= {"p2_hierarchy", "p2_options", "p2_program", "p2_stats", "p2_query", "p2_search_row"}
    assert declared == set(B.EXPORTS)
    L = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert getattr(L, name) is not None
    assert ctypes.sizeof(B.p2_program) == 16


@pytest.mark.parametrize("card,axes", [([1, 2, 2, 4], [4, 4]), ([2, 4], [2, 4]), ([4, 2, 4], [4, 8]), ([2, 4, 8], [2, 4, 8]),
                                       ([4, 8, 8], [4, 8, 8]), ([2, 4, 8, 8], [2, 4, 8, 8]), ([6, 4], [3, 8]), ([4, 16], [8, 2, 4])])
def test_placements_match_oracle(B, oracle, card, axes):
    a, b = B.p2_enumerate_placements(card, axes), oracle.enumerate_placements(card, axes)
    assert a.shape == b.shape and (a == b).all()


@pytest.mark.parametrize("card,axes", [([2, 4], [2, 4]), ([4, 2, 4], [4, 8]), ([3, 2, 4], [6, 4]), ([2, 3, 2], [6, 2]),
                                       ([2, 2, 2, 2], [4, 4])])
def test_patterns_match_oracle(B, oracle, card, axes):
    for r in range(1, len(axes) + 1):
        for red in itertools.combinations(range(len(axes)), r):
            for fm in (7, 3, 5, 6, 4):
                for x in oracle.enumerate_placements(card, axes):
                    q = oracle.Query(card, axes, x, list(red), form_mask=fm)
                    assert B.p2_num_patterns(card, axes, x, list(red), form_mask=fm) == q.n_patterns
                    for pid in range(q.n_patterns):
                        d, o = B.p2_describe_pattern(card, axes, x, list(red), pid, form_mask=fm), q.pattern(pid)
                        assert (d["slice"], d["form"], d["form_level"]) == (o["slice"], o["form"], o["form_level"])
                        assert (d["group_of"] == o["group_of"]).all() and (d["rank"] == o["rank"]).all()


@pytest.mark.parametrize("kind", ["system", "column", "row", "reduction"])
@pytest.mark.parametrize("card,axes", [([2, 4], [2, 4]), ([4, 2, 4], [4, 8]), ([3, 2, 4], [6, 4]), ([2, 3, 2], [6, 2]),
                                       ([2, 2, 2, 2], [4, 4]), ([2, 6], [2, 3, 2])])
def test_patterns_of_the_other_hierarchies_match_oracle(B, oracle, card, axes, kind):
    """Sec. 3.4, hierarchies (a)-(c) and the uncollapsed reduction rows: same patterns in the same order, same
    groups on the full system, same ranks (the library numbers devices by synthesis level internally)."""
    for r in range(1, len(axes) + 1):
        for red in itertools.combinations(range(len(axes)), r):
            for fm in (7, 5):
                for x in oracle.enumerate_placements(card, axes):
                    q = oracle.Query(card, axes, x, list(red), form_mask=fm, hierarchy=kind)
                    assert B.p2_num_patterns(card, axes, x, list(red), form_mask=fm, hierarchy=kind) == q.n_patterns
                    for pid in range(q.n_patterns):
                        d = B.p2_describe_pattern(card, axes, x, list(red), pid, form_mask=fm, hierarchy=kind)
                        o = q.pattern(pid)
                        assert (d["slice"], d["form"], d["form_level"]) == (o["slice"], o["form"], o["form_level"])
                        assert (d["group_of"] == o["group_of"]).all() and (d["rank"] == o["rank"]).all()


def test_canonical_alphabet_is_L_squared(B):
    # L levels with factor > 1 give L*L distinct group sets
    for f in ([8], [2, 4], [2, 1, 4], [2, 2, 2], [2, 2, 2, 2], [2, 1, 2, 1, 2]):
        L = sum(1 for v in f if v > 1)
        assert B.p2_num_patterns(f, [int(np.prod(f))], [f], [0]) == L * L


def test_argument_errors(B):
    def code(fn, *a, **k):
        with pytest.raises(B.P2Error) as e:
            fn(*a, **k)
        return e.value.code
    assert code(B.p2_enumerate_placements, [2, 4], [3, 3]) == B.P2_EINVAL               # products differ
    assert code(B.p2_enumerate_placements, [2] * 9, [512]) == B.P2_EUNSUPPORTED         # 9 levels
    assert code(B.p2_describe_pattern, [2, 4], [2, 4], [[2, 1], [1, 4]], [0, 0], 0) == B.P2_EINVAL   # duplicate axis
    assert code(B.p2_describe_pattern, [2, 4], [2, 4], [[2, 1], [1, 4]], [2], 0) == B.P2_EINVAL      # axis out of range
    assert code(B.p2_describe_pattern, [2, 4], [2, 4], [[1, 2], [1, 4]], [0], 0) == B.P2_EINVAL      # violates Eq. (1)
    assert code(B.p2_describe_pattern, [2, 4], [2, 4], [[2, 1], [1, 4]], [0], 7) == B.P2_EINVAL      # no such pattern
    assert code(B.p2_describe_pattern, [4, 16, 16], [1024], [[4, 16, 16]], [0], 0) == B.P2_EUNSUPPORTED   # > 512 devices
    # planning errors come back before any device work
    assert code(B.p2_synthesize, [2, 4], [2, 4], [[2, 1], [1, 4]], [0], 0) == B.P2_EINVAL            # max_len < 1
    assert code(B.p2_synthesize, [2, 4], [2, 4], [[2, 1], [1, 4]], [0], 8) == B.P2_EUNSUPPORTED      # max_len > 7
    assert code(B.p2_synthesize, [2, 4], [2, 4], [[2, 1], [1, 4]], [], 3) == B.P2_EINVAL             # empty reduce set
    assert code(B.p2_synthesize, [2, 4], [2, 4], [[2, 1], [1, 4]], [0], 3, [1e6]) == B.P2_EINVAL     # costs without links
    assert code(B.p2_synthesize, [2, 4], [2, 4], [[2, 1], [1, 4]], [0], 3, max_row_classes=65) == B.P2_EINVAL
    assert code(B.p2_synthesize, [2, 4], [2, 4], [[2, 1], [1, 4]], [0], 3, max_row_classes=-1) == B.P2_EINVAL
    assert code(B.p2_synthesize, [2, 4], [2, 4], [[2, 1], [1, 4]], [0], 3, flags=4) == B.P2_EINVAL   # unknown flag
    assert code(B.p2_synthesize, [2, 4], [2, 4], [[2, 1], [1, 4]], [0], 3, hierarchy=5) == B.P2_EUNSUPPORTED   # no such hierarchy
    for engine in (2, 3, 4, 5):       # the other hierarchies of Sec. 3.4 run on the literal engine only
        assert code(B.p2_synthesize, [2, 4], [2, 4], [[2, 1], [1, 4]], [0], 3, hierarchy="row", engine=engine) == B.P2_EUNSUPPORTED
    assert code(B.p2_synthesize, [2, 4, 4], [2, 4, 4], [[2, 1, 1], [1, 4, 1], [1, 1, 4]], [0], 7, hierarchy="row") == B.P2_EUNSUPPORTED   # > 2^30
    # the placement search checks its arguments and counts the placements before any device work
    assert code(B.p2_search_placements, [2, 4], [3, 3], [[0]], 3, 1e6) == B.P2_EINVAL                # products differ
    assert code(B.p2_search_placements, [2, 4], [2, 4], [], 3, 1e6) == B.P2_EINVAL                   # no reduction
    assert code(B.p2_search_placements, [2, 4], [2, 4], [[]], 3, 1e6) == B.P2_EINVAL                 # empty reduction
    assert code(B.p2_search_placements, [2, 4], [2, 4], [[0]], 3, -1.0) == B.P2_EINVAL               # negative bytes
    assert code(B.p2_topk, [0.0], [0], -1) == B.P2_EINVAL
    assert code(B.p2_topk, [0.0], [0], 5000) == B.P2_EUNSUPPORTED
    assert b"" == b"" and isinstance(B.lib().p2_last_error(), bytes)


def test_workloads_are_seeded(B):
    from paper_2110_10548_amd import workloads
    a, b = workloads.config(3), workloads.config(3)
    assert a == b and all(10e9 <= v <= 400e9 for v in a["bw"])
    cfg = workloads.config(5)
    pls = B.p2_enumerate_placements(cfg["card"], cfg["axes"])
    q1, q2 = workloads.expand(cfg, pls), workloads.expand(cfg, pls)
    assert q1 == q2 and len(q1) == 512 and len(pls) == 227
    counts = [len(workloads.expand(workloads.config(i), B.p2_enumerate_placements(workloads.config(i)["card"],
                                                                                  workloads.config(i)["axes"])))
              for i in (1, 2, 3, 4)]
    assert counts == [2, 10, 84, 140]

"""Pins of the CPU oracle against what the paper prints and what the mathematics fixes.

Nothing here touches the GPU path.  Every expected value is the paper's (fixtures under
tests/golden/, each with its citation), a closed form, or a hand-worked number.
"""
import itertools
import math

import numpy as np
import pytest

from conftest import golden_lines

AR, RS, AG, RD, BC = range(5)
INSIDE, PARALLEL, MASTER = range(3)


# --------------------------------------------------------------------------- placements (Sec. 3.1)
def _prime_factors(v):
    out, p = {}, 2
    while v > 1:
        while v % p == 0:
            out[p] = out.get(p, 0) + 1
            v //= p
        p += 1
    return out


def _contingency(rows, cols):
    """Number of non-negative integer tables with the given row and column sums."""
    if len(rows) == 1:
        return 1 if rows[0] == sum(cols) else 0
    total = 0
    for first in itertools.product(*[range(c + 1) for c in cols]):
        if sum(first) == rows[0]:
            total += _contingency(rows[1:], [c - f for c, f in zip(cols, first)])
    return total


def _closed_form_count(card, axes):
    primes = set()
    for v in list(card) + list(axes):
        primes |= set(_prime_factors(v))
    n = 1
    for p in primes:
        n *= _contingency([_prime_factors(a).get(p, 0) for a in axes], [_prime_factors(h).get(p, 0) for h in card])
    return n


@pytest.mark.parametrize("card,axes", [([1, 2, 2, 4], [4, 4]), ([2, 4], [2, 4]), ([4, 2, 4], [4, 8]), ([2, 4, 8], [2, 4, 8]),
                                       ([4, 8, 8], [4, 8, 8]), ([2, 4, 8, 8], [2, 4, 8, 8]), ([6, 4], [3, 8]), ([3, 6], [2, 9]),
                                       ([4, 16], [8, 2, 4]), ([2, 3], [7])])
def test_placement_count_closed_form_and_constraints(oracle, card, axes):
    pls = oracle.enumerate_placements(card, axes)
    assert len(pls) == _closed_form_count(card, axes)
    for x in pls:
        assert (x >= 1).all()
        assert [int(v) for v in x.prod(axis=0)] == list(card)      # Eq. (1): column products
        assert [int(v) for v in x.prod(axis=1)] == list(axes)      # Eq. (2): row products
    flat = [tuple(x.flatten()) for x in pls]
    assert flat == sorted(set(flat))                               # distinct, lexicographic


def test_placement_examples_of_the_overview_figure(oracle):
    # Fig. "overview" (b), (c), (d): three placements of [4,4] on [1,2,2,4]
    got = {tuple(x.flatten()) for x in oracle.enumerate_placements([1, 2, 2, 4], [4, 4])}
    for m in ([[1, 2, 2, 1], [1, 1, 1, 4]], [[1, 2, 1, 2], [1, 1, 2, 2]], [[1, 1, 2, 2], [1, 2, 1, 2]]):
        assert tuple(np.array(m).flatten()) in got


def _parse_matrices(text):
    return [tuple(tuple(int(v) for v in row.split(",")) for row in m.strip().split("/")) for m in text.split(";")]


@pytest.mark.parametrize("row", golden_lines("paper_program_counts.txt"), ids=lambda r: "%s|%s|%s" % (r[0], r[1], r[2]))
def test_paper_placement_lists_and_program_counts(oracle, row):
    """Appendix A: complete matrix list per row, and the total number of synthesized programs
    at size limit 5.  The printed totals (6 ... 235) are reproduced by the InsideGroup and
    Parallel forms (3 programs for a one-level hierarchy, 47 for a two-level one)."""
    card = [int(v) for v in row[0].split(",")]
    axes = [int(v) for v in row[1].split(",")]
    reduce_axes = [int(v) for v in row[2].split(",")]
    total = int(row[3])
    printed = _parse_matrices(row[4])
    pls = oracle.enumerate_placements(card, axes)
    assert {tuple(tuple(int(v) for v in r) for r in x) for x in pls} == set(printed)
    got = 0
    for x in pls:
        q = oracle.Query(card, axes, x, reduce_axes, form_mask=3)
        got += len(q.synthesize(5)["index"])
    assert got == total


def test_saturation_at_size_limit_five(oracle):
    # Sec. 4.2 Result 2: a larger size limit "for most cases does not generate new programs"
    q = oracle.Query([4, 16], [64], [[4, 16]], [0], form_mask=3)
    assert len(q.synthesize(5)["index"]) == len(q.synthesize(6)["index"]) == 47


# --------------------------------------------------------------------------- rules (Sec. 3.2)
def _state(text, D=4, k=4):
    s = np.zeros((k, D), dtype=np.uint8)
    if text != "-":
        for part in text.split(";"):
            r, cols = part.split(":")
            for c in cols.split(","):
                s[int(r), int(c)] = 1
    return s


@pytest.mark.parametrize("row", golden_lines("collective_examples.txt"), ids=lambda r: r[0])
def test_worked_examples_of_the_semantics_figure(oracle, row):
    op = ["AllReduce", "ReduceScatter", "AllGather", "Reduce", "Broadcast"].index(row[0])
    st = np.zeros((4, 4, 4), dtype=np.uint8)
    st[0], st[1] = _state(row[1]), _state(row[2])
    st[2] = _state("1:2")       # bystanders keep whatever they hold
    ok, out = oracle.apply_collective(st, op, [0, 1])
    assert ok
    assert (out[0] == _state(row[3])).all()
    assert (out[1] == _state(row[4])).all()
    assert (out[2] == st[2]).all() and (out[3] == st[3]).all()


def test_device_state_figure_rows(oracle):
    # Fig. "A device state": rows 0,1,3 non-empty ("3 data chunks"), row 2 empty
    fig = _state("0:0,1;1:1,2;3:2,3")
    st = np.zeros((4, 4, 4), dtype=np.uint8)
    st[0] = fig
    st[1] = _state("2:0")                       # exactly the missing chunk
    ok, out = oracle.apply_collective(st, AG, [0, 1])
    assert ok and (out[0] == _state("0:0,1;1:1,2;2:0;3:2,3")).all() and (out[1] == out[0]).all()
    st[1] = _state("3:0")                       # overlaps chunk 3 -> rows not disjoint
    assert not oracle.apply_collective(st, AG, [0, 1])[0]
    assert not oracle.apply_collective(st, AR, [0, 1])[0]   # different chunk sets


def test_rule_premises(oracle):
    init = np.zeros((4, 4, 4), dtype=np.uint8)
    for d in range(4):
        init[d, :, d] = 1
    # same data twice: after AllReduce(0,1) another AllReduce(0,1) must fail (columns not disjoint)
    ok, s1 = oracle.apply_collective(init, AR, [0, 1])
    assert ok and not oracle.apply_collective(s1, AR, [0, 1])[0]
    # scatter: contiguous blocks in ascending row order, rank p gets block p
    ok, s2 = oracle.apply_collective(init, RS, [0, 1])
    assert ok
    assert (s2[0] == _state("0:0,1;1:0,1")).all() and (s2[1] == _state("2:0,1;3:0,1")).all()
    # Sec. 2.3: ReduceScatter(A0,A1) then AllReduce(A0,A1) mixes different chunks -> invalid
    assert not oracle.apply_collective(s2, AR, [0, 1])[0]
    # scatter error when the chunk count is not divisible by the group size
    three = np.zeros((3, 4, 3), dtype=np.uint8)
    for d in range(3):
        three[d, :, d] = 1
    assert not oracle.apply_collective(three, RS, [0, 1, 2])[0]
    assert oracle.apply_collective(three, AR, [0, 1, 2])[0]
    # Reduce puts the sum on the first device and clears the others
    ok, s3 = oracle.apply_collective(init, RD, [1, 3])
    assert ok and (s3[1] == _state("0:1,3;1:1,3;2:1,3;3:1,3")).all() and not s3[3].any()
    # Broadcast needs information increase: from the init state the root knows nothing more
    assert not oracle.apply_collective(init, BC, [0, 1])[0]
    ok, s4 = oracle.apply_collective(s3, BC, [1, 3])
    assert ok and (s4[3] == s4[1]).all() and (s4[1] == s3[1]).all()
    assert not oracle.apply_collective(s4, BC, [1, 3])[0]     # nothing left to tell
    # AllGather of an empty member is rejected (reading: every member holds something)
    assert not oracle.apply_collective(s3, AG, [1, 3])[0]
    # ReduceScatter + AllGather == AllReduce
    ok, s5 = oracle.apply_collective(s2, AG, [0, 1])
    assert ok and (s5 == s1).all()


# --------------------------------------------------------------------------- groups (Sec. 3.3)
def _dev(name):
    return "ABCD".index(name[0]) * 4 + int(name[1])


def test_group_table_of_the_paper(oracle):
    # system hierarchy used as the synthesis hierarchy: one axis of 16 over [1,2,2,4], reduced
    q = oracle.Query([1, 2, 2, 4], [16], [[1, 2, 2, 4]], [0])
    level = {"root": 0, "rack": 1, "server": 2, "CPU": 3, "GPU": 4}    # (root,1) is put in front
    assert q.synthesis_hierarchy() == [1, 1, 2, 2, 4]
    for slice_name, form_text, groups_text in golden_lines("group_table.txt"):
        want = sorted(sorted(_dev(n.strip()) for n in g.split(",")) for g in groups_text.split(";"))
        if form_text == "InsideGroup":
            got = q.groups_raw(level[slice_name], INSIDE)
        else:
            form = PARALLEL if form_text.startswith("Parallel") else MASTER
            got = q.groups_raw(level[slice_name], form, level[form_text[form_text.index("(") + 1:-1]])
        assert sorted(got) == want, (slice_name, form_text)


@pytest.mark.parametrize("f", [[2, 3, 2], [4, 2, 2, 2], [3, 1, 4]])
def test_parallel_group_size_and_count_lemma(oracle, f):
    # Appendix B, lemma "Parallel reduction": (x_i, Parallel(x_j)) has groups of size
    # x_{j+1}...x_i and x_0...x_j * x_{i+1}...x_n of them.  Levels here are e_0=root, e_1..e_n.
    q = oracle.Query(f, [math.prod(f)], [f], [0])
    x = [1] + f
    n = len(f)
    for i in range(1, n + 1):
        for j in range(0, i):
            size = math.prod(x[j + 1:i + 1])
            count = math.prod(x[:j + 1]) * math.prod(x[i + 1:])
            groups = q.groups_raw(i, PARALLEL, j)
            if size == 1:
                assert groups == []          # groups of one device are not generated
            else:
                assert len(groups) == count and all(len(g) == size for g in groups)
            master = q.groups_raw(i, MASTER, j)
            if size > 1:
                assert len(master) == math.prod(x[:j + 1]) and all(len(g) == size for g in master)
                assert all(g in groups for g in master)
        inside = q.groups_raw(i, INSIDE)
        size = math.prod(x[i + 1:])
        if size > 1:
            assert len(inside) == math.prod(x[:i + 1]) and all(len(g) == size for g in inside)


def test_synthesis_hierarchies_of_the_overview_table(oracle):
    # Table "Synthesis hierarchy"
    m = [[1, 1, 2, 2], [1, 2, 1, 2]]
    assert oracle.hierarchy_of_matrix(m, [1], "column") == [1, 1, 1, 2, 2, 1, 2, 2]
    assert oracle.hierarchy_of_matrix(m, [1], "row") == [1, 1, 2, 2, 1, 2, 1, 2]
    assert oracle.hierarchy_of_matrix(m, [1], "reduction") == [1, 2, 1, 2]
    m3 = [[1, 2, 3], [4, 5, 6], [7, 8, 9]]
    assert oracle.hierarchy_of_matrix(m3, [0, 2], "column") == [1, 4, 7, 2, 5, 8, 3, 6, 9]
    assert oracle.hierarchy_of_matrix(m3, [0, 2], "row") == [1, 2, 3, 4, 5, 6, 7, 8, 9]
    assert oracle.hierarchy_of_matrix(m3, [0, 2], "reduction") == [1, 2, 3, 7, 8, 9]
    assert oracle.hierarchy_of_matrix(m3, [0, 2], "collapsed") == [7, 16, 27]


# --------------------------------------------------------------------------- running example (Sec. 2)
@pytest.fixture()
def running(oracle):
    # Fig. "overview" (d): matrix [[1,1,2,2],[1,2,1,2]] on [1,2,2,4], reduce along parameter sharding (axis 1)
    q = oracle.Query([1, 2, 2, 4], [4, 4], [[1, 1, 2, 2], [1, 2, 1, 2]], [1])
    pats = {}
    for pid in range(q.n_patterns):
        g = q.groups(pid)
        if [0, 1] in g and [2, 3] in g:
            pats["local"] = pid                  # {A0,A1},{A2,A3},... (Sec. 2.4)
        elif [0, 8] in g and [1, 9] in g:
            pats["remote"] = pid                 # A0 with C0 (Sec. 2.3), every device
        elif [0, 8] in g:
            pats["roots"] = pid                  # root devices only
        elif [0, 1, 8, 9] in g:
            pats["all"] = pid
    return q, pats


def test_running_example_named_programs(running):
    q, p = running
    assert set(p) == {"local", "remote", "roots", "all"} and q.n_patterns == 4
    assert q.synthesis_hierarchy() == [1, 1, 2, 1, 2]
    # reduction groups: devices with the same data batch, e.g. A0,A1,C0,C1
    ran, st, goal = q.run_state([p["all"] * 5 + AR])
    assert goal and sorted(np.nonzero(st[0, 0])[0]) == [0, 1, 8, 9]
    valid = [
        [p["all"] * 5 + AR],                                               # Fig. reduction (a)
        [p["local"] * 5 + AR, p["remote"] * 5 + AR],                       # (b) AllReduce-AllReduce
        [p["local"] * 5 + RD, p["roots"] * 5 + AR, p["local"] * 5 + BC],   # (c) Reduce-AllReduce-Broadcast
        [p["local"] * 5 + RS, p["remote"] * 5 + AR, p["local"] * 5 + AG],  # RS-AR-AG (Sec. 4.2)
    ]
    for prog in valid:
        assert q.eval_program(prog)[0], prog
    # Fig. "Semantically invalid reduction"
    assert q.run_state([p["local"] * 5 + RS, p["local"] * 5 + AR])[0] == 1      # second step rejected
    assert q.run_state([p["remote"] * 5 + AR, p["remote"] * 5 + AR])[0] == 1    # A0,C0 reduced twice
    # every valid program is found by the synthesizer, and only once
    res = q.synthesize(5)
    progs = [tuple(res["instr"][i][:res["len"][i]]) for i in range(len(res["index"]))]
    assert len(set(progs)) == len(progs)
    for prog in valid:
        assert tuple(prog) in progs


def _level_cells(kind, l, m, n, red):
    """Factors x[i][j] of the parallelism matrix that level e_l (l >= 1) of a synthesis hierarchy owns."""
    if kind == "system":
        return [(i, l - 1) for i in range(m)]
    if kind == "column":
        return [((l - 1) % m, (l - 1) // m)]
    if kind == "row":
        return [((l - 1) // n, (l - 1) % n)]
    if kind == "reduction":
        return [(red[(l - 1) // n], (l - 1) % n)]
    return [(i, l - 1) for i in red]                             # collapsed: the reduction axes' factors of level l-1


@pytest.mark.parametrize("kind", ["system", "column", "row", "reduction", "collapsed"])
def test_valid_programs_obey_the_validity_lemmas(oracle, kind):
    """Appendix B, "Semantically valid reduction": in a valid program an instruction (x_i, Parallel(x_j))
    only varies levels x_{j+1..i} that are 1 or on the reduction axes, (x_i, InsideGroup) only such levels
    x_{i+1..n}, and (x_i, Master(x_j)) only such levels x_{j+1..n}.  Checked on every instruction of every
    valid program of every placement of the running system, under all five synthesis hierarchies.  The
    Master lemma has two parts: the levels the groups range over (j+1..i), which must hold, and the
    levels that pick "the first group" (i+1..n).  With one group per instance of x_j and per digit of the
    other axes' levels (the reading of Master taken here) the second part can fail under (a)-(c) for a
    step that happens to be harmless; those are the only exceptions allowed."""
    card, axes = [1, 2, 2, 4], [4, 4]
    m, n = len(axes), len(card)
    exceptions = 0
    for x in oracle.enumerate_placements(card, axes):
        for red in ([0], [1]):
            q = oracle.Query(card, axes, x, red, hierarchy=kind)
            top = len(q.synthesis_hierarchy()) - 1

            def fine(l):
                return all(x[i][j] == 1 or i in red for i, j in _level_cells(kind, l, m, n, red))

            r = q.synthesize(4)
            assert len(r["index"]) > 0 or kind == "system"
            for ins, ln in zip(r["instr"], r["len"]):
                for v in ins[:ln]:
                    p = q.pattern(int(v) // 5)
                    i, form, j = p["slice"], p["form"], p["form_level"]
                    if form == INSIDE:
                        assert all(fine(l) for l in range(i + 1, top + 1)), (x.tolist(), red, int(v))
                    elif form == PARALLEL:
                        assert all(fine(l) for l in range(j + 1, i + 1)), (x.tolist(), red, int(v))
                    else:
                        assert all(fine(l) for l in range(j + 1, i + 1)), (x.tolist(), red, int(v))
                        tail = all(fine(l) for l in range(i + 1, top + 1))
                        assert tail or kind in ("system", "column", "row"), (x.tolist(), red, int(v))
                        exceptions += 0 if tail else 1
    if kind in ("reduction", "collapsed"):
        assert exceptions == 0                                   # (d): nothing but reduction-axis factors below the root


# --------------------------------------------------------------------------- enumeration invariants
def test_unrank_order_and_flat_equals_pruned(oracle):
    q = oracle.Query([2, 4], [2, 4], [[1, 2], [2, 2]], [1])
    I = q.alphabet
    assert q.num_candidates(3) == I + I * I + I ** 3
    progs = [q.unrank(3, i) for i in range(q.num_candidates(3))]
    assert [len(p) for p in progs] == [1] * I + [2] * I * I + [3] * I ** 3
    for block in (progs[:I], progs[I:I + I * I], progs[I + I * I:]):
        assert block == sorted(block)                      # lexicographic, first instruction most significant
    res = q.synthesize(3)
    n, valid, steps = q.eval_indices(3, start=0, count=q.num_candidates(3))
    assert np.nonzero(valid)[0].tolist() == res["index"].tolist()
    for i, idx in enumerate(res["index"]):
        assert q.unrank(3, int(idx)) == res["instr"][i][:res["len"][i]].tolist()


def test_single_allreduce_over_the_reduce_axes_is_always_valid(oracle):
    for card, axes in (([2, 4], [2, 4]), ([4, 2, 4], [4, 8]), ([2, 3, 2], [6, 2])):
        for x in oracle.enumerate_placements(card, axes):
            for red in ([0], [1], [0, 1]):
                q = oracle.Query(card, axes, x, red)
                assert q.pattern(0)["slice"] == 0 and q.pattern(0)["form"] == INSIDE
                assert q.eval_program([AR])[0]
                # RS;AG and Reduce;Broadcast on the same pattern leave the same state
                _, s_ar, _ = q.run_state([AR])
                for pair in ([RS, AG], [RD, BC]):
                    ran, s2, goal = q.run_state(pair)
                    assert ran == 2 and goal and (s2 == s_ar).all()


def test_validity_depends_only_on_the_number_of_levels(oracle):
    sets = []
    for f in ([2, 2], [2, 4], [3, 2], [4, 3]):
        q = oracle.Query(f, [math.prod(f)], [f], [0])
        sets.append([tuple(r) for r in q.synthesize(4)["instr"].tolist()])
    assert all(s == sets[0] for s in sets) and len(sets[0]) == 1 + 4 + 30 + 51


def test_all_axes_reduced_is_placement_independent(oracle):
    card, axes = [2, 2, 4], [4, 4]
    msg = [2.0 ** 20, 2.0 ** 26]
    ref = None
    for x in oracle.enumerate_placements(card, axes):
        q = oracle.Query(card, axes, x, [0, 1], bw=[25e9, 100e9, 300e9], alpha=[20e-6, 10e-6, 5e-6])
        r = q.synthesize(4, msg)
        key = (r["index"].tolist(), r["cost"].tolist())
        ref = ref or key
        assert key == ref


def test_chunk_count_multiple_of_group_size_gives_same_programs(oracle):
    x = [[1, 2], [2, 2]]
    base = oracle.Query([2, 4], [2, 4], x, [1]).synthesize(4)["index"].tolist()       # k = D = 8
    for k in (4, 12, 16):
        assert oracle.Query([2, 4], [2, 4], x, [1], n_chunks=k).synthesize(4)["index"].tolist() == base
    fewer = oracle.Query([2, 4], [2, 4], x, [1], n_chunks=1).synthesize(4)
    assert len(fewer["index"]) < len(base)
    assert all(RS not in [c % 5 for c in row[:n]] for row, n in zip(fewer["instr"], fewer["len"]))


# --------------------------------------------------------------------------- cost (ring alpha-beta reading)
N26 = float(1 << 26)


def test_single_level_allreduce_is_the_textbook_ring(oracle):
    for g, bw, a in ((8, 300e9, 5e-6), (3, 10e9, 1e-6)):
        q = oracle.Query([g], [g], [[g]], [0], bw=[bw], alpha=[a])
        ok, cost, _ = q.eval_program([AR], [N26])
        assert ok and cost[0] == pytest.approx(2 * (g - 1) * a + 2 * (g - 1) / g * N26 / bw, rel=1e-14)


def test_hand_worked_two_level_costs(oracle):
    # [2 nodes x 4 GPUs], NIC 25 GB/s / 20 us, in-node 300 GB/s / 5 us, one axis of 8, 64 MiB, k = 8
    q = oracle.Query([2, 4], [8], [[2, 4]], [0], bw=[25e9, 300e9], alpha=[20e-6, 5e-6])
    pats = {}
    for pid in range(q.n_patterns):
        g = q.groups(pid)
        pats["all" if len(g[0]) == 8 else "node" if g[0] == [0, 1, 2, 3] else "pairs" if len(g) == 4 else "roots"] = pid
    assert sorted(pats.values()) == [0, 1, 2, 3]
    n = N26
    # one AllReduce over 8: 14 steps across nodes; each node uplink carries 2*7/8*n
    want_a = 14 * 20e-6 + (2 * 7 / 8 * n) / 25e9
    # RS in node (3 steps, 3/4 n per GPU port); AR over pairs on n/4 bytes: 4 groups share each NIC
    # -> n bytes through it; AG in node moves 3/4 n again
    local = 3 * 5e-6 + (3 / 4 * n) / 300e9
    want_b = local + (2 * 20e-6 + (4 * (2 * 1 / 2 * n / 4)) / 25e9) + local
    # Reduce to the node root (n bytes into its port), AR between the two roots (n through each NIC),
    # Broadcast back
    red = 3 * 5e-6 + n / 300e9
    want_c = red + (2 * 20e-6 + (2 * 1 / 2 * n) / 25e9) + red
    for prog, want in (([pats["all"] * 5 + AR], want_a),
                       ([pats["node"] * 5 + RS, pats["pairs"] * 5 + AR, pats["node"] * 5 + AG], want_b),
                       ([pats["node"] * 5 + RD, pats["roots"] * 5 + AR, pats["node"] * 5 + BC], want_c)):
        ok, cost, _ = q.eval_program(prog, [n])
        assert ok and cost[0] == pytest.approx(want, rel=1e-13), prog
    assert want_b < want_c < want_a      # Sec. 4.2 Result 5: topology-aware programs win across nodes


def test_cost_identities_and_independence(oracle):
    card, axes, x = [2, 2, 4], [4, 4], [[1, 2, 2], [2, 1, 2]]
    bw, al = [25e9, 100e9, 300e9], [20e-6, 10e-6, 5e-6]
    q = oracle.Query(card, axes, x, [0], bw=bw, alpha=al)
    q0 = oracle.Query(card, axes, x, [0], bw=bw, alpha=[0, 0, 0])
    q2 = oracle.Query(card, axes, x, [0], bw=[1e9, 7e9, 3e9], alpha=[1e-3, 0, 2e-6])
    msg = [2.0 ** 20, 2.0 ** 21, 2.0 ** 30]
    r, r0, r2 = q.synthesize(4, msg), q0.synthesize(4, msg), q2.synthesize(4, msg)
    assert r["index"].tolist() == r0["index"].tolist() == r2["index"].tolist()     # validity ignores the links
    assert np.allclose(r0["cost"][:, 1], 2 * r0["cost"][:, 0], rtol=1e-14)         # linear in bytes when alpha = 0
    assert np.allclose(r0["cost"][:, 2], 1024 * r0["cost"][:, 0], rtol=1e-14)
    assert (r["cost"] > r0["cost"]).all()
    # RS;AG on a pattern costs what AR on it costs, per pattern and per message size (the ring figures add
    # up: (g-1) + (g-1) steps on the same links, (g-1)/g n bytes twice through the same uplinks).  Where the
    # one-instruction program is not a whole reduction the three are compared as prefixes of valid programs.
    found = 0
    for pid in range(q.n_patterns):
        ran_ar, s_ar, _ = q.run_state([pid * 5 + AR])
        ran_2, s_2, _ = q.run_state([pid * 5 + RS, pid * 5 + AG])
        assert ran_ar == 1 and ran_2 == 2 and (s_2 == s_ar).all()
        # a valid program that starts with AR on this pattern, and the same with RS;AG in its place
        for ins, ln, c_ar in zip(r["instr"], r["len"], r["cost"]):
            if int(ins[0]) != pid * 5 + AR or ln > 3:
                continue
            tail = [int(v) for v in ins[1:ln]]
            ok2, c2, _ = q.eval_program([pid * 5 + RS, pid * 5 + AG] + tail, msg)
            ok1, c1, _ = q.eval_program([pid * 5 + AR] + tail, msg)
            assert ok1 and ok2 and np.allclose(c1, c_ar, rtol=1e-15) and np.allclose(c2, c1, rtol=1e-13), (pid, tail)
            found += 1
    assert found >= q.n_patterns


def _pattern_named(q, **want):
    """Pattern id by its groups: n_groups, group size, and optionally a group that must be present."""
    for pid in range(q.n_patterns):
        g = q.groups(pid)
        if len(g) == want["n_groups"] and len(g[0]) == want["size"] and ("has" not in want or want["has"] in g):
            return pid
    raise AssertionError(want)


def test_hand_worked_three_level_costs_with_replicas(oracle):
    """Config 2's system [4 nodes x 2 sockets x 4 GPUs] (25 / 100 / 300 GB/s, 20 / 10 / 5 us), matrix
    [[1,2,2],[4,1,2]], 64 MiB per device, k = 32.  Device (c0, c1, c2): c0 = digit of axis 1, c1 = digit of
    axis 0, c2 = 2 * (digit of axis 0) + (digit of axis 1).  Every uplink load below is written out by hand,
    the groups of the other axis' replicas included; ring and tree."""
    card, axes, x = [4, 2, 4], [4, 8], [[1, 2, 2], [4, 1, 2]]
    bw, al = [25e9, 100e9, 300e9], [20e-6, 10e-6, 5e-6]
    n = N26
    dev = lambda c0, c1, c2: (c0 * 2 + c1) * 4 + c2
    for algo in (0, 1):
        # ---- reduce axis 0 (4 devices per reduction group: c1 and the high bit of c2; 8 replicas)
        q = oracle.Query(card, axes, x, [0], bw=bw, alpha=al, algo=algo)
        inner = _pattern_named(q, n_groups=16, size=2, has=[dev(0, 0, 0), dev(0, 0, 2)])     # same socket
        outer = _pattern_named(q, n_groups=16, size=2, has=[dev(0, 0, 0), dev(0, 1, 0)])     # across the sockets of a node
        whole = _pattern_named(q, n_groups=8, size=4)
        # ReduceScatter in the socket: 1 step, n/2 bytes through each GPU port
        t_rs = 1 * 5e-6 + (n / 2) / 300e9
        # AllReduce across sockets on the n/2 bytes each device kept: every socket holds 4 devices, each in a
        # group of its own (2 of this reduction group's halves x 2 replicas of the other axis), so 4 groups
        # share the socket's uplink; ring: 2 steps, 2 * 1/2 * n/2 bytes per group; tree: 2 steps, 2 * n/2
        per_group = (2 * (1 / 2) * (n / 2)) if algo == 0 else (2 * (n / 2))
        t_ar = 2 * 10e-6 + max(4 * per_group / 100e9, per_group / 300e9)
        # AllGather in the socket: n bytes afterwards, 1 step, n/2 through each port
        t_ag = 1 * 5e-6 + (n / 2) / 300e9
        ok, cost, _ = q.eval_program([inner * 5 + RS, outer * 5 + AR, inner * 5 + AG], [n])
        assert ok and cost[0] == pytest.approx(t_rs + t_ar + t_ag, rel=1e-13)
        # one AllReduce over the 4 devices: 2 of its members in each socket, and the socket also holds the
        # other replica's 2 members: 2 groups through the socket uplink; nothing leaves the node
        steps, per_group = (6, 2 * (3 / 4) * n) if algo == 0 else (4, 2 * n)
        ok, cost, _ = q.eval_program([whole * 5 + AR], [n])
        assert ok and cost[0] == pytest.approx(steps * 10e-6 + max(2 * per_group / 100e9, per_group / 300e9), rel=1e-13)

        # ---- reduce axis 1 (8 devices per reduction group: c0 and the low bit of c2; 4 replicas)
        q = oracle.Query(card, axes, x, [1], bw=bw, alpha=al, algo=algo)
        pair = _pattern_named(q, n_groups=16, size=2, has=[dev(0, 0, 0), dev(0, 0, 1)])       # same socket
        roots = _pattern_named(q, n_groups=4, size=4, has=[dev(0, 0, 0), dev(1, 0, 0), dev(2, 0, 0), dev(3, 0, 0)])
        # Reduce onto the pair's first device: 1 step, n bytes into its port; Broadcast back the same
        t_rd = 1 * 5e-6 + n / 300e9
        # AllReduce between the 4 nodes' roots: a node holds 4 roots (2 sockets x 2 replicas), each of a group
        # of its own, so its network uplink carries 4 groups; a socket's uplink carries 2
        steps, per_group = (6, 2 * (3 / 4) * n) if algo == 0 else (4, 2 * n)
        t_ar = steps * 20e-6 + max(4 * per_group / 25e9, 2 * per_group / 100e9, per_group / 300e9)
        ok, cost, _ = q.eval_program([pair * 5 + RD, roots * 5 + AR, pair * 5 + BC], [n])
        assert ok and cost[0] == pytest.approx(t_rd + t_ar + t_rd, rel=1e-13)


def test_rs_ag_costs_the_same_as_ar_when_both_complete(oracle):
    q = oracle.Query([2, 4], [8], [[2, 4]], [0], bw=[25e9, 300e9], alpha=[20e-6, 5e-6])
    msg = [N26, 3.0e6]
    ok1, c1, _ = q.eval_program([AR], msg)
    ok2, c2, _ = q.eval_program([RS, AG], msg)
    assert ok1 and ok2 and np.allclose(c1, c2, rtol=1e-14)


def test_tree_model_closed_forms_and_what_it_leaves_alone(oracle):
    # Sec. 4 runs both of the library's AllReduce algorithms; the tree one is the two-tree scheme
    # of its reference: up and down a binary tree, the whole message through every device twice.
    for g, bw, a in ((8, 300e9, 5e-6), (5, 10e9, 1e-6), (2, 7e9, 3e-6)):
        q = oracle.Query([g], [g], [[g]], [0], bw=[bw], alpha=[a], algo=1)
        ok, cost, _ = q.eval_program([AR], [N26])
        assert ok and cost[0] == pytest.approx(2 * math.ceil(math.log2(g)) * a + 2 * N26 / bw, rel=1e-14)
    # two levels by hand: [2 nodes x 4 GPUs], AllReduce over all 8: 2*3 tree steps over the network,
    # 2n through each node's uplink; the hierarchical program only changes in its AllReduce step
    q = oracle.Query([2, 4], [8], [[2, 4]], [0], bw=[25e9, 300e9], alpha=[20e-6, 5e-6], algo=1)
    r = oracle.Query([2, 4], [8], [[2, 4]], [0], bw=[25e9, 300e9], alpha=[20e-6, 5e-6])
    n = N26
    ok, cost, _ = q.eval_program([AR], [n])
    assert ok and cost[0] == pytest.approx(6 * 20e-6 + 2 * n / 25e9, rel=1e-13)
    node = next(pid for pid in range(q.n_patterns) if q.groups(pid)[0] == [0, 1, 2, 3])
    pairs = next(pid for pid in range(q.n_patterns) if len(q.groups(pid)) == 4)
    local = 3 * 5e-6 + (3 / 4 * n) / 300e9
    prog = [node * 5 + RS, pairs * 5 + AR, node * 5 + AG]
    ok, cost, _ = q.eval_program(prog, [n])
    assert ok and cost[0] == pytest.approx(local + (2 * 20e-6 + 4 * (2 * n / 4) / 25e9) + local, rel=1e-13)
    # the model touches AllReduce steps only, and never validity
    a, b = q.synthesize(4, [n]), r.synthesize(4, [n])
    assert a["index"].tolist() == b["index"].tolist()
    for idx, instr, ln, ca, cb in zip(a["index"], a["instr"], a["len"], a["cost"][:, 0], b["cost"][:, 0]):
        has_ar = any(int(v) % 5 == AR for v in instr[:ln])
        assert (ca != cb) if has_ar else (ca == cb), (idx, instr[:ln])
    with pytest.raises(ValueError):
        oracle.Query([2], [2], [[2]], [0], algo=2)


# --------------------------------------------------------------------------- synthesis hierarchies (Sec. 3.4)
def _lowered(q, max_len):
    """Valid programs as the paper's lowered form: a sequence of (device groups, collective)."""
    r = q.synthesize(max_len)
    groups = {pid: frozenset(tuple(g) for g in q.groups(pid)) for pid in range(q.n_patterns)}
    return {tuple((groups[int(v) // 5], int(v) % 5) for v in ins[:ln]) for ins, ln in zip(r["instr"], r["len"])}


def _replicated(program, q, reduce_axis, matrix):
    """Every instruction's groups repeated over the digits of the non-reduction axes (what lowering does
    to a pattern of hierarchy (d))."""
    n = len(matrix[0])
    other = [i for i in range(len(matrix)) if i != reduce_axis]
    coords = {}
    for d in range(q.D):
        rest, c = d, []
        for j in reversed(range(n)):
            hj = 1
            for row in matrix:
                hj *= row[j]
            c.append(rest % hj)
            rest //= hj
        c.reverse()
        dig = {}
        for j in range(n):
            v = c[j]
            for i in reversed(range(len(matrix))):
                dig[(i, j)] = v % matrix[i][j]
                v //= matrix[i][j]
        coords[d] = dig
    key_of = {d: (tuple(coords[d][(reduce_axis, j)] for j in range(n)),
                  tuple(coords[d][(i, j)] for i in other for j in range(n))) for d in range(q.D)}
    dev_of = {v: d for d, v in key_of.items()}
    replicas = sorted({k[1] for k in key_of.values()})
    out = []
    for groups, op in program:
        rep = set()
        for g in groups:
            for r in replicas:
                rep.add(tuple(sorted(dev_of[(key_of[d][0], r)] for d in g)))
        out.append((frozenset(rep), op))
    return tuple(out)


@pytest.mark.parametrize("matrix,axis", [([[1, 1, 2, 2], [1, 2, 1, 2]], 1), ([[1, 1, 2, 2], [1, 2, 1, 2]], 0),
                                         ([[1, 2, 1, 2], [1, 1, 2, 2]], 0), ([[1, 2, 2, 1], [1, 1, 1, 4]], 0)])
def test_expressive_power_of_the_synthesis_hierarchies(oracle, matrix, axis):
    """Sec. 3.4, Theorem (d) >= (c) >= (b) >= (a), on the running system with one reduction axis: every
    valid lowered program of the weaker hierarchy is a lowered program of the stronger one.  One caveat,
    which the proof sketch passes over: in (a)-(c) a Master instruction keeps only the groups whose later
    digits are zero, and those digits may belong to a non-reduction axis, so the instruction names the
    groups of some replicas only (which ones depends on the order of the levels).  Such programs are
    compared after their groups are repeated over all replicas, which is what lowering does to every
    pattern of (d); where no digit of another axis follows the reduction row nothing needs repeating.
    (This bears on the Master reading: with one group in the whole system instead of one per replica,
    (d) could not express the Master programs of (c) when the reduction row comes last.)"""
    card, axes = [1, 2, 2, 4], [4, 4]
    low = {kind: _lowered(oracle.Query(card, axes, matrix, [axis], hierarchy=kind), 4)
           for kind in ("system", "column", "row", "reduction", "collapsed")}
    assert low["reduction"] == low["collapsed"]                  # one axis: nothing to collapse
    qd = oracle.Query(card, axes, matrix, [axis])
    lifted = {kind: {_replicated(p, qd, axis, matrix) for p in low[kind]} for kind in low}
    assert lifted["collapsed"] == low["collapsed"]               # (d) is replicated already
    assert lifted["system"] <= lifted["column"] <= lifted["row"] <= low["collapsed"]
    if axis == len(matrix) - 1:                                  # the reduction row is the last one
        assert low["row"] <= low["collapsed"]
    # and (c) is not as expressive as (d) (the counterexample after Case 1 of the theorem's third part)
    if matrix == [[1, 1, 2, 2], [1, 2, 1, 2]] and axis == 0:
        assert not low["collapsed"] <= lifted["row"]


def test_hierarchy_kinds_of_the_overview_table_drive_the_patterns(oracle):
    x = [[1, 1, 2, 2], [1, 2, 1, 2]]
    want = {"system": [1, 1, 2, 2, 4], "column": [1, 1, 1, 1, 2, 2, 1, 2, 2], "row": [1, 1, 1, 2, 2, 1, 2, 1, 2],
            "reduction": [1, 1, 2, 1, 2], "collapsed": [1, 1, 2, 1, 2]}
    for kind, f in want.items():
        q = oracle.Query([1, 2, 2, 4], [4, 4], x, [1], hierarchy=kind)
        assert q.synthesis_hierarchy() == f                      # root level in front
        nonunit = sum(1 for v in f if v > 1)
        assert q.n_patterns == nonunit * nonunit                 # canonical alphabet: L^2 patterns


# --------------------------------------------------------------------------- top-k
def test_topk_against_lexsort(oracle):
    rng = np.random.default_rng(7)
    for n, k in ((1, 1), (10, 3), (1000, 10), (1000, 2000), (50, 50)):
        cost = np.round(rng.random(n), 2)            # many ties
        index = rng.permutation(n).astype(np.uint64)
        want = np.lexsort((index, cost))[:k]
        assert oracle.topk(cost, index, k).tolist() == want.tolist()
    with pytest.raises(ValueError):
        oracle.topk([1.0, float("nan")], [0, 1], 1)

"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Bar: valid program lists bit-exact (index, length, instruction codes); costs within 1e-9 relative.
"""
import numpy as np
import pytest

from paper_2110_10548_amd import workloads

pytestmark = pytest.mark.gpu

RTOL = 1e-9


@pytest.fixture(scope="module")
def B():
    from paper_2110_10548_amd import binding
    binding.lib()
    return binding


def oracle_result(oracle, q, msg, form_mask=7, op_mask=31):
    oq = oracle.Query(q["card"], q["axes"], q["placement"], q["reduce_axes"], bw=q.get("bw"), alpha=q.get("alpha"),
                      n_chunks=q.get("n_chunks", 0), form_mask=form_mask, op_mask=op_mask, algo=q.get("algo", 0),
                      hierarchy=q.get("hierarchy", "collapsed"))
    return oq, oq.synthesize(q["max_len"], msg)


def assert_same(res, ora, n_msg):
    progs = res["programs"]
    assert progs["index"].tolist() == ora["index"].tolist()
    assert progs["len"].tolist() == ora["len"].tolist()
    assert (progs["instr"] == ora["instr"][:, :7]).all()
    if n_msg:
        assert res["cost"].shape == ora["cost"].shape
        assert np.allclose(res["cost"], ora["cost"], rtol=RTOL, atol=0.0)


def in_threads(fn, items, workers=None):
    """fn over items on host threads (the oracle's C routines run outside the interpreter lock)."""
    import os
    from concurrent.futures import ThreadPoolExecutor
    workers = workers or max(1, min(16, len(os.sched_getaffinity(0))))
    with ThreadPoolExecutor(max_workers=workers) as pool:
        return list(pool.map(fn, items))


def oracle_query(oracle, q):
    return oracle.Query(q["card"], q["axes"], q["placement"], q["reduce_axes"], bw=q.get("bw"), alpha=q.get("alpha"),
                        n_chunks=q.get("n_chunks", 0), algo=q.get("algo", 0))


def check_listed_programs(oracle, q, res, rows, msg, probe_unlisted=()):
    """Rows of a result against the oracle one by one: the listed program is the unranked index, valid, at the
    oracle's cost; indices in probe_unlisted are invalid."""
    oq = oracle_query(oracle, q)
    progs = res["programs"]
    for i in rows:
        instr = progs["instr"][i][:progs["len"][i]].tolist()
        assert oq.unrank(q["max_len"], int(progs["index"][i])) == instr
        ok, cost, _ = oq.eval_program(instr, msg)
        assert ok and np.allclose(cost, res["cost"][i], rtol=RTOL, atol=0.0), (q["placement"], q["reduce_axes"], instr)
    if len(probe_unlisted):
        nvalid, _, _ = oq.eval_indices(q["max_len"], indices=list(probe_unlisted), n_threads=1)
        assert nvalid == 0
    return True


def check_shortlist(top, full, n_msg, k):
    """A query's shortlist (run with topk = k) against its own full list (run with topk = 0): for every message
    size the k smallest (cost, index) pairs in that order, programs and all their costs copied unchanged."""
    idx, cost = full["programs"]["index"], full["cost"]
    kk = min(k, len(idx))
    assert len(top["programs"]) == kk * n_msg
    pos_of = {int(ix): i for i, ix in enumerate(idx)}
    for m in range(n_msg):
        want = np.lexsort((idx, cost[:, m]))[:kk]
        got = top["programs"][m * kk:(m + 1) * kk]
        assert got["index"].tolist() == idx[want].tolist()
        rows = [pos_of[int(ix)] for ix in got["index"]]
        assert (got["instr"] == full["programs"]["instr"][rows]).all() and (got["len"] == full["programs"]["len"][rows]).all()
        assert (top["cost"][m * kk:(m + 1) * kk] == cost[rows]).all()


def queries_of(cfg_id, B):
    cfg = workloads.config(cfg_id)
    pls = B.p2_enumerate_placements(cfg["card"], cfg["axes"])
    return cfg, workloads.expand(cfg, pls)


@pytest.mark.parametrize("engine", [1, 0, 2, 4, 3], ids=["literal", "auto", "compact", "small", "frontier"])
def test_config1_every_query(B, oracle, engine):
    cfg, queries = queries_of(1, B)
    assert len(queries) == 2
    for q in queries:
        q["engine"] = engine
    results = B.p2_synthesize_batch(queries, cfg["msg_bytes"])
    for q, res in zip(queries, results):
        oq, ora = oracle_result(oracle, q, cfg["msg_bytes"])
        assert res["stats"]["candidates"] == oq.num_candidates(q["max_len"])
        assert_same(res, ora, len(cfg["msg_bytes"]))
        # steps executed == what flat, unpruned evaluation of every index executes
        _, _, steps = oq.eval_indices(q["max_len"], start=0, count=oq.num_candidates(q["max_len"]))
        if engine == 3:      # pruned enumeration: only valid prefixes are extended
            assert res["stats"]["engine"] == 3 and 0 < res["stats"]["steps_executed"] < steps
        else:
            assert res["stats"]["steps_executed"] == steps


@pytest.mark.parametrize("engine", [1, 0, 2, 4, 3], ids=["literal", "auto", "compact", "small", "frontier"])
def test_config2_every_query(B, oracle, engine):
    cfg, queries = queries_of(2, B)
    assert len(queries) == 10
    for q in queries:
        q["engine"] = engine
    results = B.p2_synthesize_batch(queries, cfg["msg_bytes"])
    cache = {}
    for q, res in zip(queries, results):
        key = (tuple(map(tuple, q["placement"])), tuple(q["reduce_axes"]))
        oq, ora = oracle_result(oracle, q, cfg["msg_bytes"])
        cache[key] = ora
        assert_same(res, ora, len(cfg["msg_bytes"]))
    # reducing over all axes: the same programs and costs whatever the placement
    full = [r for q, r in zip(queries, results) if q["reduce_axes"] == [0, 1]]
    for r in full[1:]:
        assert r["programs"]["index"].tolist() == full[0]["programs"]["index"].tolist()
        assert np.allclose(r["cost"], full[0]["cost"], rtol=1e-12)


def test_single_query_entry_point_and_sizing(B, oracle):
    cfg, queries = queries_of(1, B)
    q = queries[0]
    res = B.p2_synthesize(q["card"], q["axes"], q["placement"], q["reduce_axes"], q["max_len"], cfg["msg_bytes"],
                          bw=q["bw"], alpha=q["alpha"])
    _, ora = oracle_result(oracle, q, cfg["msg_bytes"])
    assert_same(res, ora, 1)
    assert res["candidates"] == res["stats"]["candidates"]
    with pytest.raises(B.P2Error) as e:
        B.p2_synthesize(q["card"], q["axes"], q["placement"], q["reduce_axes"], q["max_len"], cfg["msg_bytes"],
                        bw=q["bw"], alpha=q["alpha"], cap=1)
    assert e.value.code == B.P2_ENOSPC


@pytest.mark.parametrize("card,axes,red,max_len,k", [
    ([3, 2, 2], [6, 2], [0], 4, 0),          # radix 3: groups are not bit-fields
    ([2, 3, 2], [2, 6], [1], 4, 0),
    ([2, 2, 3], [4, 3], [0, 1], 3, 0),
    ([2, 4], [8], [0], 4, 3),                # chunk counts that break ReduceScatter
    ([2, 4], [8], [0], 4, 1),
    ([2, 2, 2], [8], [0], 4, 16),
    ([5], [5], [0], 4, 0),
    ([2, 4, 8], [2, 4, 8], [1], 4, 0),
])
@pytest.mark.parametrize("engine", [1, 0, 2, 4, 3], ids=["literal", "auto", "compact", "small", "frontier"])
def test_ragged_shapes_every_placement(B, oracle, card, axes, red, max_len, k, engine):
    bw = [11e9 * (j + 1) for j in range(len(card))]
    alpha = [7e-6 / (j + 1) for j in range(len(card))]
    msg = [1.0e6, 3.0e8]
    queries = [dict(card=card, axes=axes, placement=pl, reduce_axes=red, max_len=max_len, bw=bw, alpha=alpha,
                    n_chunks=k, engine=engine) for pl in B.p2_enumerate_placements(card, axes).tolist()]
    try:
        results = B.p2_synthesize_batch(queries, msg)
    except B.P2Error as e:
        if engine == 4 and e.code == B.P2_EUNSUPPORTED:
            pytest.skip("groups that are not bit-fields of the device number: outside the small-group engine")
        raise
    for q, res in zip(queries, results):
        _, ora = oracle_result(oracle, q, msg)
        assert_same(res, ora, 2)


@pytest.mark.parametrize("seed", [20211020, 7])
def test_random_queries_every_engine(B, oracle, seed):
    """Seeded random small systems, placements, reduce sets, chunk counts, grammar masks and cost models:
    every engine that accepts a query returns the oracle's list and costs."""
    queries = workloads.random_queries(seed, 150)
    msg = [float(1 << 22), 3.0e8]
    ran = {e: 0 for e in (0, 1, 2, 3, 4, 5)}
    for q in queries:
        probe = oracle.Query(q["card"], q["axes"], q["placement"], q["reduce_axes"], form_mask=q["form_mask"],
                             op_mask=q["op_mask"])
        q["max_len"] = 1
        while q["max_len"] < 5 and probe.alphabet > 0 and probe.num_candidates(q["max_len"] + 1) <= 200_000:
            q["max_len"] += 1
        _, ora = oracle_result(oracle, q, msg, form_mask=q["form_mask"], op_mask=q["op_mask"])
        for engine in ran:
            try:
                res = B.p2_synthesize_batch([dict(q, engine=engine)], msg)[0]
            except B.P2Error as e:
                assert e.code == B.P2_EUNSUPPORTED and engine in (4, 5), (engine, q)
                continue
            ran[engine] += 1
            assert res["stats"]["candidates"] == (probe.num_candidates(q["max_len"]) if probe.alphabet else 0), (engine, q)
            try:
                assert_same(res, ora, len(msg))
            except AssertionError:
                print("engine", engine, "query", q)
                raise
    assert min(ran[e] for e in (0, 1, 2, 3)) == len(queries) and ran[4] > 10 and ran[5] > 10, ran


def test_small_group_engine_selection(B, oracle):
    """AUTO evaluates reduction groups of at most 32 devices with power-of-two patterns on the shared-prefix
    engine (engine 5 in the stats); it and the small-group engine (4) can also be asked for, and refuse
    hierarchies they cannot hold."""
    cfg, queries = queries_of(2, B)
    for engine in (4, 5):
        for q, res in zip(queries, B.p2_synthesize_batch([dict(q, engine=engine) for q in queries], cfg["msg_bytes"])):
            assert res["stats"]["engine"] == engine
            _, ora = oracle_result(oracle, q, cfg["msg_bytes"])
            assert_same(res, ora, len(cfg["msg_bytes"]))
    auto = B.p2_synthesize_batch(queries[:2], cfg["msg_bytes"])
    assert [r["stats"]["engine"] for r in auto] == [5, 5]
    odd = dict(card=[2, 3], axes=[6], placement=[[2, 3]], reduce_axes=[0], max_len=3, bw=[1e10, 1e11], alpha=[1e-5, 1e-6])
    assert B.p2_synthesize_batch([odd], [1e6])[0]["stats"]["engine"] == 2          # groups of 3: compact engine
    for engine in (4, 5):
        with pytest.raises(B.P2Error) as ei:
            B.p2_synthesize_batch([dict(odd, engine=engine)], [1e6])
        assert ei.value.code == B.P2_EUNSUPPORTED


@pytest.mark.parametrize("engine", [1, 2, 5], ids=["literal", "compact", "shared"])
def test_tree_cost_model(B, oracle, engine):
    """algo = 1 (tree AllReduce): every cost kernel against the oracle, ring and tree queries in one batch."""
    cfg, queries = queries_of(2, B)
    mixed = []
    for i, q in enumerate(queries):
        mixed.append(dict(q, engine=engine, algo=1))
        if i % 3 == 0:
            mixed.append(dict(q, engine=engine, algo=0))
    cfg3 = workloads.config(3)
    pl3 = B.p2_enumerate_placements(cfg3["card"], cfg3["axes"])
    q3 = [q for q in workloads.expand(cfg3, pl3) if q["reduce_axes"] == [1, 2]][:2]      # 32 devices, 64 chunks
    mixed += [dict(q, engine=engine if engine != 1 else 0, algo=1, max_len=4) for q in q3]
    results = B.p2_synthesize_batch(mixed, cfg["msg_bytes"])
    differs = 0
    for q, res in zip(mixed, results):
        _, ora = oracle_result(oracle, q, cfg["msg_bytes"])
        assert_same(res, ora, len(cfg["msg_bytes"]))
        if q["algo"] == 1:
            _, ring = oracle_result(oracle, dict(q, algo=0), cfg["msg_bytes"])
            differs += int((ring["cost"] != ora["cost"]).any())
    assert differs > 0
    with pytest.raises(B.P2Error) as e:
        B.p2_synthesize_batch([dict(queries[0], algo=2)], cfg["msg_bytes"])
    assert e.value.code == B.P2_EUNSUPPORTED


def _check_search(got, want):
    assert got["placements"] == want["placements"]
    assert set(got["rows"]) == set(want["rows"])
    for key, w in want["rows"].items():
        g = got["rows"][key]
        assert g["valid"] == w["valid"], key
        assert np.isclose(g["best_cost"], w["best_cost"], rtol=RTOL, atol=0.0), key
        assert np.isclose(g["allreduce_cost"], w["allreduce_cost"], rtol=RTOL, atol=0.0), key
        assert len(g["best_instr"]) > 0 or w["best_index"] is None
    assert np.allclose(got["total"], want["total"], rtol=RTOL, atol=0.0)
    # ranking: ascending in the library's own totals; placements whose totals tie to within rounding may swap
    tot = got["total"]
    assert sorted(got["order"]) == list(range(len(tot)))
    assert [(tot[p], p) for p in got["order"]] == sorted((tot[p], p) for p in range(len(tot)))
    assert np.allclose([want["total"][p] for p in got["order"]], [want["total"][p] for p in want["order"]], rtol=RTOL, atol=0.0)
    return got


@pytest.mark.parametrize("cfg_id,algo", [(1, 0), (2, 0), (2, 1)])
def test_placement_search(B, oracle, cfg_id, algo):
    """Every placement x every reduce set in one call, against the oracle's plain loop (Sec. 4.1)."""
    from oracle import p2_search
    cfg = workloads.config(cfg_id)
    msg = cfg["msg_bytes"][0]
    kw = dict(bw=cfg["bw"], alpha=cfg["alpha"], algo=algo, weights=[1.0, 0.25][:len(cfg["reduce_sets"])])
    got = B.p2_search_placements(cfg["card"], cfg["axes"], cfg["reduce_sets"], cfg["max_len"], msg, **kw)
    want = p2_search.search_placements(cfg["card"], cfg["axes"], cfg["reduce_sets"], cfg["max_len"], msg, **kw)
    _check_search(got, want)
    # the best program is a valid one with that cost, and the cheapest up to ties within rounding
    for (p, s), g in got["rows"].items():
        oq = oracle.Query(cfg["card"], cfg["axes"], want["placements"][p], cfg["reduce_sets"][s], bw=cfg["bw"],
                          alpha=cfg["alpha"], algo=algo)
        ok, cost, _ = oq.eval_program(g["best_instr"], [msg])
        assert ok and np.isclose(cost[0], g["best_cost"], rtol=RTOL, atol=0.0)
        w = want["rows"][(p, s)]
        if g["best_index"] != w["best_index"]:
            assert np.isclose(w["best_cost"], g["best_cost"], rtol=RTOL, atol=0.0)


def test_placement_search_single_device_reduction_and_sizing(B):
    from oracle import p2_search
    args = ([2, 4], [1, 8], [[0], [1]], 3, float(2 ** 26))
    kw = dict(bw=[25e9, 300e9], alpha=[20e-6, 5e-6])
    got = _check_search(B.p2_search_placements(*args, **kw), p2_search.search_placements(*args, **kw))
    assert all(got["rows"][(p, 0)]["best_instr"] == [] and got["rows"][(p, 0)]["best_cost"] == 0.0
               for p in range(len(got["placements"])))


KINDS = ["system", "column", "row", "reduction"]


@pytest.mark.parametrize("kind", KINDS)
def test_other_synthesis_hierarchies(B, oracle, kind):
    """Sec. 3.4, hierarchies (a)-(c) and the reduction rows before collapsing, on the full system: valid lists
    and costs against the oracle, every placement and reduction of small systems (powers of two and not), ring
    and tree, in one batch with queries of the tool's own hierarchy."""
    msg = [2.0 ** 20, 2.0 ** 28]
    queries = []
    for card, axes, max_len in (([2, 4], [2, 4], 3), ([1, 2, 2, 4], [4, 4], 3), ([2, 3, 2], [6, 2], 3), ([2, 6], [2, 3, 2], 2)):
        links = dict(bw=[12.5e9, 50e9, 150e9, 300e9][:len(card)], alpha=[2e-5, 1e-5, 5e-6, 2e-6][:len(card)])
        reds = [[i] for i in range(len(axes))] + [list(range(len(axes)))]
        for n, x in enumerate(B.p2_enumerate_placements(card, axes).tolist()):
            for red in reds:
                queries.append(dict(card=card, axes=axes, placement=x, reduce_axes=red, max_len=max_len, hierarchy=kind,
                                    algo=n % 2, **links))
                if n % 4 == 0:
                    queries.append(dict(queries[-1], hierarchy="collapsed"))
    results = B.p2_synthesize_batch(queries, msg)
    n_valid = 0
    for q, res in zip(queries, results):
        oq, ora = oracle_result(oracle, q, msg)
        assert_same(res, ora, len(msg))
        assert res["stats"]["n_patterns"] == oq.n_patterns and res["stats"]["engine"] in (1, 2, 5)
        n_valid += len(ora["index"]) if q["hierarchy"] == kind else 0
    assert n_valid > 100
    for engine in (2, 3, 4, 5):
        with pytest.raises(B.P2Error) as e:
            B.p2_synthesize_batch([dict(queries[0], engine=engine)], msg)
        assert e.value.code == B.P2_EUNSUPPORTED


def test_random_queries_other_hierarchies(B, oracle):
    """Seeded random small systems under every other hierarchy of Sec. 3.4, with the random grammar masks, chunk
    counts and cost models of the generator: lists and costs against the oracle."""
    msg = [float(1 << 22), 3.0e8]
    n = 0
    for q in workloads.random_queries(77, 40, max_devices=32):
        for kind in KINDS:
            probe = oracle.Query(q["card"], q["axes"], q["placement"], q["reduce_axes"], form_mask=q["form_mask"],
                                 op_mask=q["op_mask"], hierarchy=kind)
            max_len = 1
            while max_len < 4 and probe.alphabet > 0 and probe.num_candidates(max_len + 1) <= 60_000:
                max_len += 1
            qk = dict(q, max_len=max_len, hierarchy=kind)
            _, ora = oracle_result(oracle, qk, msg, form_mask=q["form_mask"], op_mask=q["op_mask"])
            assert_same(B.p2_synthesize_batch([qk], msg)[0], ora, len(msg))
            n += len(ora["index"])
    assert n > 1000


@pytest.mark.parametrize("card,axes,placement,red,max_len", [
    ([6, 4, 6], [24, 6], [[6, 4, 1], [1, 1, 6]], [1], 3),             # 144 devices: 5 words per mask
    ([4, 3, 8], [8, 12, 1], [[2, 1, 4], [2, 3, 2], [1, 1, 1]], [0], 2),   # 96 devices: 3 words
    ([2, 8, 8], [2, 64], [[2, 1, 1], [1, 8, 8]], [1], 2),             # 128 devices: 4 words
])
def test_other_hierarchies_above_64_devices(B, oracle, card, axes, placement, red, max_len):
    """Sec. 3.4, hierarchies (a)-(c) on systems whose device masks take several words, a power of two or not:
    the per-device goals (several reduction groups inside the copy) against the oracle."""
    msg = [2.0 ** 22, 3.0e8]
    links = dict(bw=[12.5e9, 50e9, 150e9][:len(card)], alpha=[2e-5, 1e-5, 5e-6][:len(card)])
    n = 0
    for kind in KINDS:
        for algo in (0, 1):
            q = dict(card=card, axes=axes, placement=placement, reduce_axes=red, max_len=max_len, hierarchy=kind, algo=algo,
                     **links)
            _, ora = oracle_result(oracle, q, msg)
            assert_same(B.p2_synthesize_batch([q], msg)[0], ora, len(msg))
            n += len(ora["index"])
    assert n >= 8


def test_literal_states_of_different_shapes_in_one_batch(B, oracle):
    """Two queries of the literal engine with masks of the same width, one with many devices and one chunk,
    one with fewer devices and many chunks: each state fits in LDS, a state of the larger device count and the
    larger chunk count together would not.  They share their launches."""
    msg = [2.0 ** 22, 3.0e8]
    links = dict(bw=[12.5e9, 50e9, 150e9], alpha=[2e-5, 1e-5, 5e-6])
    queries = [dict(card=[4, 8, 8], axes=[256], placement=[[4, 8, 8]], reduce_axes=[0], n_chunks=1, max_len=2, engine=1, **links),
               dict(card=[6, 4, 6], axes=[144], placement=[[6, 4, 6]], reduce_axes=[0], n_chunks=16, max_len=2, engine=1, **links),
               dict(card=[6, 4, 6], axes=[144], placement=[[6, 4, 6]], reduce_axes=[0], n_chunks=16, max_len=2, engine=2, **links)]
    n = 0
    for q, res in zip(queries, B.p2_synthesize_batch(queries, msg)):
        _, ora = oracle_result(oracle, q, msg)
        assert_same(res, ora, len(msg))
        n += len(ora["index"])
    assert n >= 6


@pytest.mark.parametrize("seed", [17, 170])
def test_mixed_batches(B, oracle, seed):
    """One batch of seeded random queries of every kind at once: up to 512 devices, the tool's hierarchy and the
    others of Sec. 3.4, forced engines, and repeats of a query that differ in links, cost model or shortlist
    length (their validity is shared, their costs are their own), in shuffled order; each against the oracle."""
    msg = [float(1 << 20), float(1 << 26), 3.0e8]
    rng = workloads.SplitMix64(seed * 7 + 1)
    batch = []
    for q in workloads.random_queries(seed, 30, max_devices=512):
        devices = int(np.prod(q["card"]))
        kind = ["collapsed", "collapsed", "collapsed", "system", "column", "row", "reduction"][rng.below(7)]
        limit = min(200_000 if devices <= 64 else 20_000, 200_000 if kind == "collapsed" else 30_000)
        probe = oracle.Query(q["card"], q["axes"], q["placement"], q["reduce_axes"], form_mask=q["form_mask"],
                             op_mask=q["op_mask"], hierarchy=kind)
        max_len = 1
        while max_len < 5 and probe.alphabet > 0 and probe.num_candidates(max_len + 1) <= limit:
            max_len += 1
        q = dict(q, max_len=max_len, hierarchy=kind)
        batch.append(q)
        for _ in range(rng.below(4)):
            d = dict(q)
            if rng.below(2):
                d["bw"] = [b * (1 + rng.below(5)) for b in q["bw"]]
            if rng.below(2):
                d["alpha"] = [a * (1 + rng.below(3)) for a in q["alpha"]]
            if rng.below(2):
                d["algo"] = 1 - q.get("algo", 0)
            if rng.below(3) == 0:
                d["topk"] = 1 + rng.below(6)
            if kind == "collapsed" and rng.below(3) == 0:
                d["engine"] = [0, 1, 2, 3][rng.below(4)]
            batch.append(d)
    for i in range(len(batch) - 1, 0, -1):
        j = rng.below(i + 1)
        batch[i], batch[j] = batch[j], batch[i]
    results = B.p2_synthesize_batch(batch, msg)
    n_valid = 0
    for q, res in zip(batch, results):
        _, ora = oracle_result(oracle, q, msg, form_mask=q["form_mask"], op_mask=q["op_mask"])
        n_valid += len(ora["index"])
        k = q.get("topk", 0)
        if k == 0:
            assert_same(res, ora, len(msg))
            continue
        kk = min(k, len(ora["index"]))
        assert len(res["programs"]) == kk * len(msg)
        pos_of = {int(ix): i for i, ix in enumerate(ora["index"])}
        for m in range(len(msg)):
            got = res["programs"]["index"][m * kk:(m + 1) * kk].tolist()
            rows = [pos_of[ix] for ix in got]
            assert len(set(got)) == kk
            assert np.allclose(res["cost"][m * kk:(m + 1) * kk], ora["cost"][rows], rtol=RTOL, atol=0.0)
            assert np.allclose(np.sort(ora["cost"][rows, m]), np.sort(ora["cost"][:, m])[:kk], rtol=RTOL, atol=0.0)
    assert len(batch) > 50 and n_valid > 300


def _lowered_programs(B, q, res):
    """Programs as sequences of (device groups on the full system, collective)."""
    groups = {}
    for pid in range(res["stats"]["n_patterns"]):
        d = B.p2_describe_pattern(q["card"], q["axes"], q["placement"], q["reduce_axes"], pid, hierarchy=q["hierarchy"],
                                  form_mask=q.get("form_mask", 7))
        by = {}
        for dev, g in enumerate(d["group_of"].tolist()):
            if g >= 0:
                by.setdefault(g, []).append(dev)
        groups[pid] = frozenset(tuple(v) for v in by.values())
    return {tuple((groups[int(v) // 5], int(v) % 5) for v in p["instr"][:p["len"]]) for p in res["programs"]}


@pytest.mark.parametrize("matrix,axis", [([[1, 1, 2, 2], [1, 2, 1, 2]], 1), ([[1, 2, 1, 2], [1, 1, 2, 2]], 0)])
def test_expressive_power_of_the_hierarchies_on_the_gpu(B, oracle, matrix, axis):
    """Sec. 3.4, Theorem: on the running system, with the reduction row placed so that no digit of another
    axis follows it in hierarchy (c), every lowered program of (a) is one of (b), of (b) one of (c), of (c) one
    of (d); all five hierarchies through the library, the program sets equal to the oracle's."""
    card, axes = [1, 2, 2, 4], [4, 4]
    kinds = KINDS + ["collapsed"]
    queries = [dict(card=card, axes=axes, placement=matrix, reduce_axes=[axis], max_len=4, hierarchy=k) for k in kinds]
    low = {}
    for q, res in zip(queries, B.p2_synthesize_batch(queries)):
        _, ora = oracle_result(oracle, q, [])
        assert_same(res, ora, 0)
        low[q["hierarchy"]] = _lowered_programs(B, q, res)
    assert low["reduction"] == low["collapsed"] and len(low["column"]) > 0 and len(low["row"]) > len(low["column"])
    if axis == len(matrix) - 1:
        assert low["system"] <= low["column"] <= low["row"] <= low["collapsed"]
    else:
        # Master groups of (a)-(c) exist in some copies only; without them the chain holds as it stands
        def no_master(kind):
            q = dict(queries[kinds.index(kind)], form_mask=3)
            return _lowered_programs(B, q, B.p2_synthesize_batch([q])[0])
        assert no_master("system") <= no_master("column") <= no_master("row") <= no_master("collapsed")


@pytest.mark.parametrize("form_mask,op_mask", [(3, 31), (5, 31), (7, 0b01101), (7, 0b11001), (4, 31)])
def test_grammar_masks(B, oracle, form_mask, op_mask):
    q = dict(card=[2, 2, 2], axes=[8], placement=[[2, 2, 2]], reduce_axes=[0], max_len=4, bw=[1e9, 2e9, 3e9],
             alpha=[1e-6, 2e-6, 3e-6], form_mask=form_mask, op_mask=op_mask)
    res = B.p2_synthesize_batch([q], [1e7])[0]
    _, ora = oracle_result(oracle, q, [1e7], form_mask=form_mask, op_mask=op_mask)
    assert_same(res, ora, 1)


def test_paper_counts_on_the_gpu(B):
    # Appendix A: 47 programs for a two-level hierarchy, 3 for a one-level one (InsideGroup + Parallel)
    r = B.p2_synthesize([4, 16], [64], [[4, 16]], [0], 5, form_mask=3)
    assert len(r["programs"]) == 47
    r = B.p2_synthesize([4, 16], [4, 16], [[4, 1], [1, 16]], [0], 5, form_mask=3)
    assert len(r["programs"]) == 3


def test_topk_in_synthesize(B, oracle):
    cfg, queries = queries_of(2, B)
    q = dict(queries[1], topk=10)       # first placement, reduce over both axes
    msg = cfg["msg_bytes"]
    res = B.p2_synthesize_batch([q], msg)[0]
    _, ora = oracle_result(oracle, q, msg)
    n = len(ora["index"])
    kk = min(10, n)
    assert len(res["programs"]) == kk * len(msg)
    pos_of = {int(ix): i for i, ix in enumerate(ora["index"])}
    for m in range(len(msg)):
        want = oracle.topk(ora["cost"][:, m], ora["index"], 10)
        got = res["programs"]["index"][m * kk:(m + 1) * kk].tolist()
        gcost = res["cost"][m * kk:(m + 1) * kk]
        rows = [pos_of[ix] for ix in got]                       # every listed program is a valid one
        assert len(set(got)) == kk
        assert np.allclose(gcost, ora["cost"][rows], rtol=RTOL, atol=0.0)
        # ordered by (cost, index) in the kernel's own arithmetic
        keys = list(zip(gcost[:, m].tolist(), got))
        assert keys == sorted(keys)
        # and it is a cheapest-k set: programs whose oracle costs tie to within rounding may swap,
        # nothing else may differ from the oracle's shortlist
        assert np.allclose(np.sort(ora["cost"][rows, m]), ora["cost"][want, m], rtol=RTOL, atol=0.0)
        exact_ties = np.isclose(ora["cost"][:, m][None, want], ora["cost"][:, m][want, None], rtol=RTOL).sum() > kk
        if not exact_ties:
            assert got == ora["index"][want].tolist()


@pytest.mark.parametrize("n,k", [(1, 1), (7, 10), (64, 64), (1000, 10), (100003, 10), (100003, 1024), (5000, 1000)])
def test_topk_kernel(B, oracle, n, k):
    rng = np.random.default_rng(n * 31 + k)
    cost = np.round(rng.random(n), 3) if n > 100 else rng.random(n)      # ties in the big cases
    index = rng.permutation(n).astype(np.uint64)
    assert B.p2_topk(cost, index, k).tolist() == oracle.topk(cost, index, k).tolist()


def test_topk_device_pointers_and_nan(B, oracle):
    import torch
    n, k = 50000, 10
    rng = np.random.default_rng(5)
    cost = rng.random((n, 3))
    index = rng.permutation(n).astype(np.int64)
    dc = torch.from_numpy(cost).cuda()
    di = torch.from_numpy(index).cuda()
    out = torch.empty(k, dtype=torch.int64, device="cuda")
    torch.cuda.synchronize()
    for m in range(3):
        B.p2_topk_device(dc.data_ptr() + 8 * m, 3, di.data_ptr(), n, k, out.data_ptr())
        assert out.cpu().numpy().tolist() == oracle.topk(cost[:, m], index.astype(np.uint64), k).tolist()
    bad = cost[:, 0].copy()
    bad[123] = np.nan
    with pytest.raises(B.P2Error) as e:
        B.p2_topk(bad, index.astype(np.uint64), k)
    assert e.value.code == B.P2_EINVAL


def test_empty_and_degenerate(B):
    # a reduce axis of size 1: nothing to reduce, no instruction exists, no candidate
    r = B.p2_synthesize([2, 2], [1, 4], [[1, 1], [2, 2]], [0], 3)
    assert r["candidates"] == 0 and len(r["programs"]) == 0
    assert B.p2_topk(np.zeros(0), np.zeros(0, dtype=np.uint64), 5).tolist() == []


def test_measured_alu_ceiling(B):
    """The derived ceiling (256 CUs x 128 lanes per clock x 2.4 GHz) bounds what an instruction stream reaches,
    and the stream comes within a factor of two of it."""
    nominal = 256 * 128 * 2.4e9
    got = B.p2_measure_alu_peak(3)
    assert 0.5 * nominal < got <= 1.02 * nominal, got


def test_measured_lds_ceiling(B):
    """The derived ceiling of the local data share (256 CUs x 256 bytes per clock for 128-bit reads x 2.4 GHz) bounds
    what a stream of such reads reaches, and the stream comes within a factor of three of it."""
    nominal = 256 * 256 * 2.4e9
    got = B.p2_measure_lds_peak(3)
    print("LDS read stream: %.1f TB/s of %.1f" % (got / 1e12, nominal / 1e12))
    assert nominal / 3 < got <= 1.02 * nominal, got


def test_caller_stream_and_host_threads(B, oracle):
    """The call runs on the caller's HIP stream (after work already queued there), and calls from
    different host threads use their own device scratch."""
    import threading
    import torch
    cfg, queries = queries_of(2, B)
    msg = cfg["msg_bytes"]
    want = B.p2_synthesize_batch(queries, msg)
    stream = torch.cuda.Stream()                      # default priority
    with torch.cuda.stream(stream):
        x = torch.ones(1 << 20, device="cuda")
        for _ in range(20):
            x = x * 1.0001
        got = B.p2_synthesize_batch(queries, msg, stream=stream.cuda_stream)
    stream.synchronize()
    for g, w in zip(got, want):
        assert g["programs"]["index"].tolist() == w["programs"]["index"].tolist()
        assert (g["cost"] == w["cost"]).all()

    out, errors = {}, []

    def worker(tag, engine):
        try:
            qs = [dict(q, engine=engine) for q in queries]
            out[tag] = [B.p2_synthesize_batch(qs, msg) for _ in range(3)]
        except Exception as e:                        # noqa: BLE001 - reported below
            errors.append((tag, repr(e)))
    threads = [threading.Thread(target=worker, args=(t, e)) for t, e in (("a", 0), ("b", 4), ("c", 2))]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    for tag in ("a", "b", "c"):
        for res in out[tag]:
            for g, w in zip(res, want):
                assert g["programs"]["index"].tolist() == w["programs"]["index"].tolist()
                assert np.allclose(g["cost"], w["cost"], rtol=RTOL, atol=0.0)
    # (the three threads have ended and given their device caches back; this thread does so on request and
    # its next call allocates afresh)
    free_before = torch.cuda.mem_get_info()[0]
    B.p2_release_thread()
    assert torch.cuda.mem_get_info()[0] >= free_before
    again = B.p2_synthesize_batch(queries, msg)
    for g, w in zip(again, want):
        assert g["programs"]["index"].tolist() == w["programs"]["index"].tolist()
        assert (g["cost"] == w["cost"]).all()


# --------------------------------------------------------------------------- full-size configurations 3 and 4
def _levels(q):
    f = [1] * len(q["card"])
    for a in q["reduce_axes"]:
        f = [x * y for x, y in zip(f, q["placement"][a])]
    return sum(1 for v in f if v > 1)


def test_config3_every_query(B, oracle):
    """64 devices, 64-bit masks, every placement x every non-empty reduce-axis subset, length <= 5 (up to
    1.9e8 candidates per query): the 84 queries as one batch, every one of them compared with the oracle
    element by element (lists and costs; the oracle enumerates the 32 three-level queries in about a second
    each, on host threads)."""
    cfg, queries = queries_of(3, B)
    assert len(queries) == 84
    assert sorted(_levels(q) for q in queries) == [1] * 20 + [2] * 32 + [3] * 32
    results = B.p2_synthesize_batch(queries, cfg["msg_bytes"])
    oracles = in_threads(lambda q: oracle_result(oracle, q, cfg["msg_bytes"])[1], queries)
    for q, res, ora in zip(queries, results, oracles):
        assert res["stats"]["valid"] == {1: 3, 2: 110, 3: 2549}[_levels(q)] == len(ora["index"])
        assert_same(res, ora, 1)


@pytest.mark.parametrize("engine", [5, 2], ids=["shared", "compact"])
def test_alphabet_above_one_wavefront(B, oracle, engine):
    """Four non-unit levels give 16 patterns x 5 rules = 80 instructions, more than the 64 lanes of a
    wavefront: the shared-prefix engine walks a group's candidates in two passes."""
    q = dict(card=[2, 2, 2, 2], axes=[2, 2, 2, 2], placement=[[2, 1, 1, 1], [1, 2, 1, 1], [1, 1, 2, 1], [1, 1, 1, 2]],
             reduce_axes=[0, 1, 2, 3], max_len=3, bw=[10e9, 40e9, 100e9, 300e9], alpha=[20e-6, 10e-6, 5e-6, 2e-6], engine=engine)
    msg = [1.0e6, 2.5e8]
    res = B.p2_synthesize_batch([q], msg)[0]
    assert res["stats"]["alphabet"] == 80 and res["stats"]["engine"] == engine
    oq, ora = oracle_result(oracle, q, msg)
    assert_same(res, ora, 2)
    _, _, steps = oq.eval_indices(q["max_len"], start=0, count=oq.num_candidates(q["max_len"]))
    assert res["stats"]["steps_executed"] == steps


@pytest.mark.parametrize("classes", [1, 3])
def test_handed_over_groups_beyond_the_class_limit(B, oracle, classes):
    """The groups that the shared-prefix engine hands over are evaluated on classes of equal rows; an entry that
    needs more classes than the state holds falls back to the full literal state.  With power-of-two groups
    the real limit (64) is never reached, so the limit is lowered here: stems and groups then take the
    fallback at the first ReduceScatter (limit 1) or at a later one (limit 3), and the results stay the same.
    The frontier engine keeps its literal prefixes the same way and sends those beyond the limit to the kernel
    that rebuilds the full literal state."""
    cfg, queries = queries_of(2, B)
    cfg3 = workloads.config(3)
    pl3 = B.p2_enumerate_placements(cfg3["card"], cfg3["axes"])
    q3 = [dict(q, max_len=4) for q in workloads.expand(cfg3, pl3) if q["reduce_axes"] == [1, 2]][:2]   # 32 devices, 64 chunks
    batch = [dict(q, engine=5) for q in queries + q3]
    batch += [dict(q, engine=3) for q in queries[::9] + q3[:1]]      # the frontier engine's literal prefixes as well
    limited = B.p2_synthesize_batch([dict(q, max_row_classes=classes) for q in batch], cfg["msg_bytes"])
    usual = B.p2_synthesize_batch(batch, cfg["msg_bytes"])
    handed = 0
    for q, res, ref in zip(batch, limited, usual):
        _, ora = oracle_result(oracle, q, cfg["msg_bytes"])
        assert_same(res, ora, len(cfg["msg_bytes"]))
        for key in ("steps_executed", "member_visits", "literal_reruns", "valid"):
            assert res["stats"][key] == ref["stats"][key]
        handed += res["stats"]["literal_reruns"] if q["engine"] == 5 else 0
    assert handed > 0


@pytest.mark.parametrize("card,axes,k,algo", [([2, 8, 8], [128], 512, 0), ([3, 8, 8], [192], 384, 1), ([4, 8, 8], [256], 256, 0),
                                              ([2, 4, 8, 8], [2, 256], 256, 0)])
def test_costs_of_large_reduction_groups(B, oracle, card, axes, k, algo):
    """Reduction groups of 128 to 256 devices (one of them not a power of two) with many chunks: only a few such
    states fit in LDS beside each other, so their programs are costed one per wavefront (k_cost_wide), every
    collective and form among them; lists and costs against the oracle."""
    links = dict(bw=[12.5e9, 50e9, 150e9, 300e9][:len(card)], alpha=[2e-5, 1e-5, 5e-6, 2e-6][:len(card)])
    msg = [2.0 ** 20, 2.0 ** 30]
    x = [list(card)] if len(axes) == 1 else [[2, 1, 1, 1], [1, 4, 8, 8]]
    q = dict(card=card, axes=axes, placement=x, reduce_axes=[len(axes) - 1], max_len=3, n_chunks=k, algo=algo, engine=2, **links)
    res = B.p2_synthesize_batch([q], msg)[0]
    _, ora = oracle_result(oracle, q, msg)
    assert_same(res, ora, len(msg))
    ops = {int(v) % 5 for p in res["programs"] for v in p["instr"][:p["len"]]}
    assert ops == {0, 1, 2, 3, 4} and len(res["programs"]) > 20


@pytest.mark.parametrize("engine", [0, 2, 4, 1], ids=["auto", "compact", "small", "literal"])
def test_equal_queries_are_evaluated_once(B, oracle, engine):
    """Queries of a batch with the same reduction group, chunks, patterns, alphabet and size limit share one
    evaluation (validity does not depend on the links or on where the placement puts the group); lists, costs and
    per-candidate step counts are those of every query evaluated on its own (P2_FLAG_EVALUATE_EVERY_QUERY)."""
    cfg, queries = queries_of(2 if engine != 1 else 1, B)
    batch = [dict(q, engine=engine) for q in queries]
    shared = B.p2_synthesize_batch(batch, cfg["msg_bytes"])
    alone = B.p2_synthesize_batch([dict(q, flags=B.FLAG_EVALUATE_EVERY_QUERY) for q in batch], cfg["msg_bytes"])
    for q, a, b in zip(batch, shared, alone):
        _, ora = oracle_result(oracle, q, cfg["msg_bytes"])
        assert_same(a, ora, len(cfg["msg_bytes"]))
        assert_same(b, ora, len(cfg["msg_bytes"]))
        for key in ("steps_executed", "member_visits", "valid", "literal_reruns", "candidates"):
            assert a["stats"][key] == b["stats"][key]
    if engine == 0:      # the shared-prefix engine reports what it carried out per query: nothing for a repeated one
        assert sum(1 for r in shared if r["stats"]["steps_evaluated"] == 0) >= len(batch) // 2
        assert all(r["stats"]["steps_evaluated"] > 0 for r in alone)


def test_config3_compact_engine_matches_default(B, oracle):
    """The default engine on configuration 3 is the shared-prefix engine (64 devices, power-of-two levels);
    the LDS-resident compact engine, which evaluates every candidate in a lane of its own, gives the same
    lists, costs and per-candidate step counts."""
    cfg, queries = queries_of(3, B)
    mine = [q for q in queries if _levels(q) == 2][:4] + [dict(q, max_len=4) for q in queries if _levels(q) == 3][:3]
    auto = B.p2_synthesize_batch(mine, cfg["msg_bytes"])
    flat = B.p2_synthesize_batch([dict(q, engine=2) for q in mine], cfg["msg_bytes"])
    for a, b in zip(auto, flat):
        assert a["stats"]["engine"] == 5 and b["stats"]["engine"] == 2
        assert a["programs"]["index"].tolist() == b["programs"]["index"].tolist()
        assert np.allclose(a["cost"], b["cost"], rtol=RTOL)
        assert a["stats"]["steps_executed"] == b["stats"]["steps_executed"]
        assert a["stats"]["steps_evaluated"] < b["stats"]["steps_evaluated"] == b["stats"]["steps_executed"]
    _, ora = oracle_result(oracle, mine[0], cfg["msg_bytes"])
    assert_same(auto[0], ora, 1)


def test_config3_literal_engine_small_queries(B, oracle):
    cfg, queries = queries_of(3, B)
    mine = [dict(q, engine=1) for q in queries if _levels(q) == 1][:6] + \
           [dict(q, engine=1, max_len=4) for q in queries if _levels(q) == 2][:3]
    for q, res in zip(mine, B.p2_synthesize_batch(mine, cfg["msg_bytes"])):
        assert res["stats"]["engine"] == 1
        assert_same(res, oracle_result(oracle, q, cfg["msg_bytes"])[1], 1)


def test_config4_every_query(B, oracle):
    """256 devices, reduction groups of 64, chunk counts 1 / 8 / 64 / 256, top-10: the 140 queries as the
    configuration states them (one batch, shortlists of 10) and once more with full lists.
    Full lists against the oracle element by element for k = 1, 8 and 64 on every placement and for k = 256 on
    three placements (the oracle needs half a minute for one of those); the other k = 256 lists must equal
    the k = 64 ones (k a multiple of the group size) and have 300 sampled programs and 2 000 unlisted indices
    checked one by one on three further placements.  Every shortlist against its query's full list."""
    cfg, queries = queries_of(4, B)
    msg = cfg["msg_bytes"]
    assert len(queries) == 140
    levels = [_levels(q) for q in queries]
    assert levels.count(2) == 16 and levels.count(3) == 124
    top = B.p2_synthesize_batch(queries, msg)
    full = B.p2_synthesize_batch([dict(q, topk=0) for q in queries], msg)
    for q, t, f in zip(queries, top, full):
        check_shortlist(t, f, len(msg), 10)
    big = [i for i, q in enumerate(queries) if q["n_chunks"] == 256 and levels[i] == 3]
    whole = [i for i, q in enumerate(queries) if q["n_chunks"] != 256 or levels[i] == 2] + big[::13][:3]
    # the long oracle runs first, so that the threads end together
    whole.sort(key=lambda i: -queries[i]["n_chunks"] * levels[i])
    oracles = in_threads(lambda i: oracle_result(oracle, queries[i], msg)[1], whole)
    for i, ora in zip(whole, oracles):
        assert_same(full[i], ora, 1)
        if queries[i]["n_chunks"] >= 64:       # (fewer chunks than devices in the group: scatters drop out by divisibility)
            assert len(ora["index"]) == {3: 2549, 2: 110}[levels[i]]
    by_pl = {(q["placement_index"], q["n_chunks"]): i for i, q in enumerate(queries)}
    for i in big:
        j = by_pl[(queries[i]["placement_index"], 64)]
        assert full[i]["programs"]["index"].tolist() == full[j]["programs"]["index"].tolist()
        assert (full[i]["programs"]["instr"] == full[j]["programs"]["instr"]).all()
    rng = np.random.default_rng(4)
    jobs = []
    for i in [b for b in big if b not in whole][::9][:3]:
        q, res = queries[i], full[i]
        listed = set(res["programs"]["index"].tolist())
        N = full[i]["stats"]["candidates"]
        pick = rng.choice(len(res["programs"]), size=300, replace=False)
        probe = [int(v) for v in rng.integers(0, N, size=2000) if int(v) not in listed]
        # neighbours of valid programs are the likeliest false negatives
        probe += [int(ix) + d for ix in res["programs"]["index"][pick[:100]] for d in (-1, 1) if int(ix) + d not in listed and 0 <= int(ix) + d < N]
        for part in range(15):
            jobs.append((q, res, pick[part::15].tolist(), probe[part::15]))
    assert len(jobs) == 45
    assert all(in_threads(lambda j: check_listed_programs(oracle, j[0], j[1], j[2], msg, j[3]), jobs))


# --------------------------------------------------------------------------- configuration 5
def test_config5_every_query(B, oracle):
    """512 devices, size limit 6, 512 random (placement, reduce-axis subset) queries, top-10: the whole
    configuration as it is stated (one batch, shortlists of 10) and once more with full lists (13.7 M programs).
    On all 512 queries: valid counts (one to four levels: 3, 110, 6 794 and 83 920, the oracle's own counts on
    small systems with as many levels), ascending indices, equal lists for queries that are the same
    (placement, reduction), the shortlist against the query's own full list, and every entry of every
    shortlist valid for the oracle at the oracle's cost.  The oracle works on literal 512 x 512 x 512-bit
    states, so beyond that it checks outputs one by one, on host threads: for one query of every
    (group size, levels) class 100 listed programs (unranked program, validity, cost) and the unlisted
    neighbours of their indices; no program of the sample may be cheaper than the tenth of the shortlist."""
    cfg, queries = queries_of(5, B)
    msg = cfg["msg_bytes"]
    assert len(queries) == 512
    top = B.p2_synthesize_batch(queries, msg)
    full = B.p2_synthesize_batch([dict(q, topk=0) for q in queries], msg)
    count_of = {1: 3, 2: 110, 4: 83920}
    count_of[3] = len(oracle.Query([2, 2, 2], [8], [[2, 2, 2]], [0]).synthesize(6)["index"])
    assert count_of[3] == 6794
    assert len(oracle.Query([2, 2, 2, 2], [16], [[2, 2, 2, 2]], [0]).synthesize(6)["index"]) == count_of[4]
    twins, classes = {}, {}
    for n, (q, t, f) in enumerate(zip(queries, top, full)):
        L = _levels(q)
        if L == 0:
            assert f["stats"]["candidates"] == 0 and len(f["programs"]) == 0 and len(t["programs"]) == 0
            continue
        assert f["stats"]["valid"] == t["stats"]["valid"] == count_of[L] == len(f["programs"])
        assert (np.diff(f["programs"]["index"].astype(np.int64)) > 0).all()
        check_shortlist(t, f, 1, 10)
        key = (tuple(map(tuple, q["placement"])), tuple(q["reduce_axes"]))
        if key in twins:
            o = full[twins[key]]
            assert (f["programs"] == o["programs"]).all() and (f["cost"] == o["cost"]).all()
        twins.setdefault(key, n)
        classes.setdefault((f["stats"]["group_size"], L), n)
    assert len(classes) == 20 and {L for _, L in classes} == {1, 2, 3, 4} and max(R for R, _ in classes) == 512
    rng = np.random.default_rng(5)
    jobs = []
    for n in sorted(twins.values()):                       # the shortlist of every distinct query
        jobs += [(queries[n], top[n], [i], []) for i in range(len(top[n]["programs"]))]
    sampled = {}
    for (R, L), n in sorted(classes.items(), key=lambda kv: -kv[0][0]):     # the slow ones first
        q, f, t = queries[n], full[n], top[n]
        listed = set(f["programs"]["index"].tolist())
        pick = rng.choice(len(f["programs"]), size=min(100, len(f["programs"])), replace=False)
        sampled[n] = pick
        near = [int(ix) + d for ix in f["programs"]["index"][pick] for d in (-1, 1)
                if int(ix) + d not in listed and 0 <= int(ix) + d < f["stats"]["candidates"]]
        for i in pick:
            jobs.append((q, f, [int(i)], []))
        for part in range(0, len(near), 8):
            jobs.append((q, f, [], near[part:part + 8]))
    import time
    t0 = time.time()
    assert all(in_threads(lambda j: check_listed_programs(oracle, j[0], j[1], j[2], msg, j[3]), jobs))
    print("config 5: %d oracle jobs (%d programs, %d unlisted indices) in %.1f s" % (
        len(jobs), sum(len(j[2]) for j in jobs), sum(len(j[3]) for j in jobs), time.time() - t0), flush=True)
    for n, pick in sampled.items():
        tenth = top[n]["cost"][-1, 0]
        listed = set(top[n]["programs"]["index"].tolist())
        for i in pick:
            assert full[n]["cost"][i, 0] >= tenth or int(full[n]["programs"]["index"][i]) in listed


# --------------------------------------------------------------------------- frontier engine (enumeration by size, Sec. 3.5)
def test_frontier_four_levels_size_limit_six(B, oracle):
    """Four hierarchy levels, size limit 6: 2.65e11 candidates, far beyond index-by-index evaluation.
    On 16 devices the oracle's own pruned enumeration gives the whole list (83 920 programs)."""
    q = dict(card=[2, 2, 2, 2], axes=[16], placement=[[2, 2, 2, 2]], reduce_axes=[0], max_len=6,
             bw=[10e9, 40e9, 100e9, 300e9], alpha=[20e-6, 10e-6, 5e-6, 2e-6], engine=3)
    msg = [float(1 << 26)]
    res = B.p2_synthesize_batch([q], msg)[0]
    assert res["stats"]["candidates"] == sum(80 ** l for l in range(1, 7))
    oq, ora = oracle_result(oracle, q, msg)
    assert len(ora["index"]) == 83920
    assert_same(res, ora, 1)
    # pruning: far fewer steps than candidates
    assert res["stats"]["steps_executed"] < 1e8


@pytest.mark.parametrize("pairs", [1, 2, 3, 4], ids=["one-pair", "two-pairs", "two-pairs-handed-over", "literal-only"])
def test_frontier_state_forms(B, oracle, pairs):
    """The frontier engine keeps a prefix as up to two (chunk set, mask) pairs per device.  The same lists and
    costs must come out with one pair (what needs two goes to the literal kernels), with every two-pair prefix
    handed to the literal kernels for classification (the path of prefixes whose groups are not aligned), and
    with no pair states at all (every prefix literal, every program costed by re-running it)."""
    cfg, queries = queries_of(2, B)
    msg = cfg["msg_bytes"]
    batch = [dict(q, engine=3, frontier_pairs=pairs) for q in queries]
    four = dict(card=[2, 2, 2, 2], axes=[16], placement=[[2, 2, 2, 2]], reduce_axes=[0], max_len=5 if pairs != 4 else 4,
                bw=[10e9, 40e9, 100e9, 300e9], alpha=[20e-6, 10e-6, 5e-6, 2e-6], engine=3, frontier_pairs=pairs)
    odd = dict(card=[3, 2, 2], axes=[6, 2], placement=[[3, 2, 1], [1, 1, 2]], reduce_axes=[0], max_len=4, n_chunks=12,
               bw=[10e9, 40e9, 100e9], alpha=[20e-6, 10e-6, 5e-6], engine=3, frontier_pairs=pairs)
    batch += [four, dict(four, bw=[40e9, 10e9, 300e9, 100e9], algo=1), odd]
    results = B.p2_synthesize_batch(batch, msg)
    reruns = 0
    for q, res in zip(batch, results):
        _, ora = oracle_result(oracle, q, msg)
        assert_same(res, ora, len(msg))
        assert res["stats"]["engine"] == 3
        reruns += res["stats"]["literal_reruns"]
    # the two-pair form holds every prefix of these queries but a handful at five instructions
    assert (reruns > 0) == (pairs != 2) or reruns < 200


def test_enumerations_side_by_side_or_one_after_the_other(B, oracle):
    """A batch's enumerations run on several streams at once (a host thread each); with
    FLAG_ONE_ENUMERATION_AT_A_TIME they run one after the other.  Same lists, same costs, to the bit; the
    oracle agrees on every query."""
    cfg, queries = queries_of(3, B)
    msg = cfg["msg_bytes"]
    mine = [q for q in queries if _levels(q) == 3][:6] + [q for q in queries if _levels(q) == 2][:6] + [q for q in queries if _levels(q) == 1][:3]
    # different placements and reduce sets give different (R, patterns): several enumerations in the batch
    together = B.p2_synthesize_batch([dict(q, engine=3) for q in mine], msg)
    alone = B.p2_synthesize_batch([dict(q, engine=3, flags=B.FLAG_ONE_ENUMERATION_AT_A_TIME) for q in mine], msg)
    assert len({r["stats"]["evaluated_with"] for r in together}) > 1
    assert sum(1 for r in together if r["stats"]["evaluated_with"] < 0) >= 3
    for q, a, b in zip(mine, together, alone):
        assert a["programs"]["index"].tolist() == b["programs"]["index"].tolist()
        assert (a["programs"]["instr"] == b["programs"]["instr"]).all()
        assert (a["cost"] == b["cost"]).all()
        assert a["stats"]["steps_executed"] == b["stats"]["steps_executed"]
        _, ora = oracle_result(oracle, q, msg)
        assert_same(a, ora, len(msg))


def test_profiling_levels_of_the_frontier_engine(B):
    """p2_set_profiling(1) brackets every group of the frontier engine's launches with an event pair,
    p2_set_profiling(2) only its classification and the building of children; the results do not depend
    on either, and what the states-judged figures count is the same."""
    cfg, queries = queries_of(3, B)
    msg = cfg["msg_bytes"]
    mine = [dict(q, engine=3) for q in queries if _levels(q) == 3][:4]
    try:
        B.p2_set_profiling(False)
        plain = B.p2_synthesize_batch(mine, msg)
        B.p2_set_profiling(True)
        full = B.p2_synthesize_batch(mine, msg)
        p_full = B.p2_get_profile()
        B.p2_set_profiling(2)
        light = B.p2_synthesize_batch(mine, msg)
        p_light = B.p2_get_profile()
    finally:
        B.p2_set_profiling(False)
    for a, b, c in zip(plain, full, light):
        assert a["programs"]["index"].tolist() == b["programs"]["index"].tolist() == c["programs"]["index"].tolist()
        assert (a["cost"] == b["cost"]).all() and (a["cost"] == c["cost"]).all()
    assert p_full["front_classify_ms"] > 0 and p_full["front_materialize_ms"] > 0 and p_full["front_group_ms"] > 0
    assert p_light["front_classify_ms"] > 0 and p_light["front_materialize_ms"] > 0
    assert p_light["front_group_ms"] == 0 and p_light["front_literal_ms"] == 0
    for key in ("front_classify_launches", "front_materialize_launches", "front_prefixes", "front_entries", "front_classify_lane_ops"):
        assert p_full[key] == p_light[key] and p_full[key] > 0
    # at the size limit only the states from which an instruction can still end at the goal are walked:
    # fewer lane-operations than every judged state's planes times the alphabet's members would give
    assert p_full["front_classify_state_bytes"] > 0


def test_frontier_matches_flat_engine_on_config3_sample(B):
    cfg, queries = queries_of(3, B)
    mine = [q for q in queries if _levels(q) == 3][:4] + [q for q in queries if _levels(q) == 2][:4]
    flat = B.p2_synthesize_batch([dict(q, engine=0) for q in mine], cfg["msg_bytes"])
    front = B.p2_synthesize_batch([dict(q, engine=3) for q in mine], cfg["msg_bytes"])
    for a, b in zip(flat, front):
        assert a["programs"]["index"].tolist() == b["programs"]["index"].tolist()
        assert (a["programs"]["instr"] == b["programs"]["instr"]).all()
        assert np.allclose(a["cost"], b["cost"], rtol=1e-12)
        assert b["stats"]["engine"] == 3 and b["stats"]["steps_executed"] < a["stats"]["steps_executed"]

"""Seeded synthetic workloads: the five (system, axes, reduce sets, limits) configurations.

This module only *describes inputs*.  It holds none of the method's arithmetic: no
placement enumeration, no grouping, no semantics, no cost.  Both the CPU oracle's
tests and the GPU path's callers read their inputs from here, so that they see
identical numbers.  A workload is turned into a list of queries by `expand`, which is
handed the placement list by whoever enumerated it.

The paper's own workloads are (hierarchy, axes, reduce axes, size limit, bytes) tuples
(Sec. 4: systems [2|4,16] and [2|4,8], size limit 5, 2^29 x nodes floats); these have
the same shape, with link figures in the range of the ones Sec. 5 lists.
"""
from itertools import combinations

MASK64 = (1 << 64) - 1


class SplitMix64:
    """SplitMix64 (Steele, Lea, Flood 2014): the stated generator for every random input."""

    def __init__(self, seed: int):
        self.state = seed & MASK64

    def next_u64(self) -> int:
        self.state = (self.state + 0x9E3779B97F4A7C15) & MASK64
        z = self.state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK64
        return z ^ (z >> 31)

    def uniform(self, lo: float = 0.0, hi: float = 1.0) -> float:
        return lo + (hi - lo) * ((self.next_u64() >> 11) * (1.0 / (1 << 53)))

    def below(self, n: int) -> int:
        return self.next_u64() % n


def _subsets(n):
    out = []
    for r in range(1, n + 1):
        out += [list(c) for c in combinations(range(n), r)]
    return out


def config(i: int) -> dict:
    """Configuration i in 1..5.  Arrays are outermost hardware level first."""
    if i == 1:
        return dict(name="cfg1", card=[2, 4], bw=[25e9, 300e9], alpha=[20e-6, 5e-6], axes=[2, 4],
                    reduce_sets=[[1]], max_len=3, n_chunks=[0], msg_bytes=[float(1 << 26)], topk=0,
                    placements="all")
    if i == 2:
        return dict(name="cfg2", card=[4, 2, 4], bw=[25e9, 100e9, 300e9], alpha=[20e-6, 10e-6, 5e-6], axes=[4, 8],
                    reduce_sets=[[0], [0, 1]], max_len=4, n_chunks=[0],
                    msg_bytes=[float(1 << e) for e in range(20, 31)], topk=0, placements="all")
    if i == 3:
        rng = SplitMix64(3)
        bw = [rng.uniform(10e9, 400e9) for _ in range(3)]
        return dict(name="cfg3", card=[2, 4, 8], bw=bw, alpha=[20e-6, 10e-6, 5e-6], axes=[2, 4, 8],
                    reduce_sets=_subsets(3), max_len=5, n_chunks=[0], msg_bytes=[float(1 << 26)], topk=0,
                    placements="all")
    if i == 4:
        return dict(name="cfg4", card=[4, 8, 8], bw=[25e9, 100e9, 300e9], alpha=[20e-6, 10e-6, 5e-6], axes=[4, 8, 8],
                    reduce_sets=[[1, 2]], max_len=5, n_chunks=[1, 8, 64, 256], msg_bytes=[float(1 << 26)], topk=10,
                    placements="all")
    if i == 5:
        rng = SplitMix64(5)
        bw = [rng.uniform(10e9, 400e9) for _ in range(4)]
        alpha = [rng.uniform(1e-6, 30e-6) for _ in range(4)]
        return dict(name="cfg5", card=[2, 4, 8, 8], bw=bw, alpha=alpha, axes=[2, 4, 8, 8],
                    reduce_sets="random", max_len=6, n_chunks=[0], msg_bytes=[float(1 << 26)], topk=10,
                    placements=512, seed=5)
    raise ValueError(i)


def expand(cfg: dict, placements) -> list:
    """List of queries of a configuration, given its enumerated placement list
    (a sequence of [n_axes][n_levels] integer matrices in lexicographic order)."""
    placements = [[[int(v) for v in row] for row in pl] for pl in placements]
    queries = []
    base = dict(card=cfg["card"], bw=cfg["bw"], alpha=cfg["alpha"], axes=cfg["axes"], max_len=cfg["max_len"],
                msg_bytes=cfg["msg_bytes"], topk=cfg["topk"])
    if cfg["placements"] == "all":
        for pi, pl in enumerate(placements):
            for rs in cfg["reduce_sets"]:
                for k in cfg["n_chunks"]:
                    queries.append(dict(base, placement=pl, placement_index=pi, reduce_axes=list(rs), n_chunks=k))
    else:
        rng = SplitMix64(cfg["seed"] + 1000)
        subsets = _subsets(len(cfg["axes"]))
        for _ in range(cfg["placements"]):
            pi = rng.below(len(placements))
            rs = subsets[rng.below(len(subsets))]
            queries.append(dict(base, placement=placements[pi], placement_index=pi, reduce_axes=list(rs),
                                n_chunks=cfg["n_chunks"][0]))
    return queries


def random_queries(seed: int, count: int, max_devices: int = 64) -> list:
    """Seeded random small queries for parity sweeps: 1-4 hardware levels with cardinalities from
    {1, 2, 3, 4, 6, 8} (at most max_devices devices), 1-3 axes given by a random split of every level's
    cardinality (which is a placement), a random non-empty reduce set, chunk counts around the
    reduction-group size, random grammar masks, link parameters and cost model.  max_len is left to
    the caller (it depends on the alphabet)."""
    rng = SplitMix64(seed)
    out = []
    while len(out) < count:
        n = 1 + rng.below(4)
        card = [[1, 2, 3, 4, 6, 8][rng.below(6)] for _ in range(n)]
        devices = 1
        for c in card:
            devices *= c
        if devices < 2 or devices > max_devices:
            continue
        m = 1 + rng.below(3)
        placement = [[1] * n for _ in range(m)]
        for j, c in enumerate(card):
            rest = c
            for i in range(m - 1):
                divisors = [d for d in range(1, rest + 1) if rest % d == 0]
                placement[i][j] = divisors[rng.below(len(divisors))]
                rest //= placement[i][j]
            placement[m - 1][j] = rest
        axes = []
        for row in placement:
            size = 1
            for v in row:
                size *= v
            axes.append(size)
        subsets = _subsets(m)
        reduce_axes = subsets[rng.below(len(subsets))]
        group = 1
        for a in reduce_axes:
            group *= axes[a]
        chunks = [0, 0, group, 1, 2, 2 * group, 12, 3 * group][rng.below(8)]
        if chunks > 128:
            chunks = group
        form_mask = [7, 7, 7, 3, 5, 6, 1][rng.below(7)]
        op_mask = 31 if rng.below(3) else 1 + rng.below(31)
        out.append(dict(card=card, axes=axes, placement=placement, reduce_axes=list(reduce_axes), n_chunks=chunks,
                        form_mask=form_mask, op_mask=op_mask, algo=rng.below(2),
                        bw=[rng.uniform(10e9, 400e9) for _ in range(n)],
                        alpha=[rng.uniform(1e-6, 30e-6) for _ in range(n)]))
    return out

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

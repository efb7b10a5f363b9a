"""ctypes wrapper around oracle/p2_oracle.c.

TEST INFRASTRUCTURE: a plain CPU statement of what the P^2 synthesizer
(arXiv 2110.10548, Sec. 3 and 5) computes.  Only tests, the smoke check and the
benchmark's CPU-baseline leg may import this module.  It contains argument
marshalling only; every rule lives in the C file.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

OPS = ("AllReduce", "ReduceScatter", "AllGather", "Reduce", "Broadcast")
FORMS = ("InsideGroup", "Parallel", "Master")
MAXLEN = 8

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        i32p, f64p, u64p, u8p, i64p = (C.POINTER(C.c_int32), C.POINTER(C.c_double), C.POINTER(C.c_uint64),
                                       C.POINTER(C.c_uint8), C.POINTER(C.c_int64))
        L.p2o_enumerate_placements.restype = C.c_int64
        L.p2o_enumerate_placements.argtypes = [C.c_int, i32p, C.c_int, i32p, i32p, C.c_int64]
        L.p2o_query_create.restype = C.c_void_p
        L.p2o_query_create.argtypes = [C.c_int, i32p, f64p, f64p, C.c_int, i32p, i32p, C.c_int, i32p,
                                       C.c_int, C.c_uint32, C.c_uint32]
        L.p2o_query_create_kind.restype = C.c_void_p
        L.p2o_query_create_kind.argtypes = L.p2o_query_create.argtypes + [C.c_int]
        L.p2o_synthesis_levels.restype = C.c_int
        L.p2o_synthesis_levels.argtypes = [C.c_void_p]
        L.p2o_query_free.argtypes = [C.c_void_p]
        L.p2o_set_algo.restype = C.c_int
        L.p2o_set_algo.argtypes = [C.c_void_p, C.c_int]
        for name in ("p2o_num_devices", "p2o_num_chunks", "p2o_num_patterns", "p2o_alphabet_size"):
            getattr(L, name).restype = C.c_int
            getattr(L, name).argtypes = [C.c_void_p]
        L.p2o_synthesis_hierarchy.argtypes = [C.c_void_p, i32p]
        L.p2o_pattern_info.restype = C.c_int
        L.p2o_pattern_info.argtypes = [C.c_void_p, C.c_int, i32p, i32p, i32p, i32p, i32p]
        L.p2o_groups_raw.restype = C.c_int
        L.p2o_groups_raw.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, i32p, i32p]
        L.p2o_hierarchy_of_matrix.restype = C.c_int
        L.p2o_hierarchy_of_matrix.argtypes = [C.c_int, C.c_int, i32p, i32p, C.c_int, i64p]
        L.p2o_num_candidates.restype = C.c_uint64
        L.p2o_num_candidates.argtypes = [C.c_void_p, C.c_int]
        L.p2o_unrank.restype = C.c_int
        L.p2o_unrank.argtypes = [C.c_void_p, C.c_int, C.c_uint64, u8p]
        L.p2o_eval_program.restype = C.c_int
        L.p2o_eval_program.argtypes = [C.c_void_p, u8p, C.c_int, C.c_int, f64p, f64p, i32p]
        L.p2o_eval_indices.restype = C.c_int64
        L.p2o_eval_indices.argtypes = [C.c_void_p, C.c_int, u64p, C.c_uint64, C.c_int64, u8p, i64p, C.c_int]
        L.p2o_synthesize.restype = C.c_int64
        L.p2o_synthesize.argtypes = [C.c_void_p, C.c_int, C.c_int, f64p, u64p, u8p, u8p, f64p, C.c_int64, i64p]
        L.p2o_apply_collective_raw.restype = C.c_int
        L.p2o_apply_collective_raw.argtypes = [C.c_int, C.c_int, u8p, C.c_int, i32p, C.c_int]
        L.p2o_run_program_state.restype = C.c_int
        L.p2o_run_program_state.argtypes = [C.c_void_p, u8p, C.c_int, u8p, i32p]
        L.p2o_topk.restype = C.c_int64
        L.p2o_topk.argtypes = [f64p, u64p, C.c_int64, C.c_int, i64p]
        _lib = L
    return _lib


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t))


def _i32(x):
    return np.ascontiguousarray(np.asarray(x, dtype=np.int32))


def _f64(x):
    return np.ascontiguousarray(np.asarray(x, dtype=np.float64))


def enumerate_placements(card, axes):
    card, axes = _i32(card), _i32(axes)
    n = lib().p2o_enumerate_placements(len(card), _p(card, C.c_int32), len(axes), _p(axes, C.c_int32), None, 0)
    if n < 0:
        raise ValueError("bad arguments")
    out = np.zeros((max(n, 1), len(axes), len(card)), dtype=np.int32)
    lib().p2o_enumerate_placements(len(card), _p(card, C.c_int32), len(axes), _p(axes, C.c_int32),
                                   _p(out, C.c_int32), n)
    return out[:n]


class Query:
    """System + placement + reduction axes (+ chunk count and grammar masks)."""

    def __init__(self, card, axes, placement, reduce_axes, bw=None, alpha=None, n_chunks=0, form_mask=7, op_mask=31,
                 algo=0, hierarchy="collapsed"):
        card, axes = _i32(card), _i32(axes)
        placement = _i32(placement).reshape(len(axes), len(card))
        reduce_axes = _i32(reduce_axes)
        bw = _f64(bw if bw is not None else [1.0] * len(card))
        alpha = _f64(alpha if alpha is not None else [0.0] * len(card))
        # synthesis hierarchy (Sec. 3.4): the tool's own choice is "collapsed" = (d)
        kind = {"column": 0, "row": 1, "reduction": 2, "collapsed": 3, "system": 4}[hierarchy]
        self._h = lib().p2o_query_create_kind(len(card), _p(card, C.c_int32), _p(bw, C.c_double), _p(alpha, C.c_double),
                                              len(axes), _p(axes, C.c_int32), _p(placement, C.c_int32),
                                              len(reduce_axes), _p(reduce_axes, C.c_int32), n_chunks, form_mask, op_mask,
                                              kind)
        if not self._h:
            raise ValueError("invalid query")
        if lib().p2o_set_algo(self._h, algo) != 0:      # 0 ring, 1 tree (AllReduce only)
            raise ValueError("unknown cost model")
        self.n_levels = len(card)
        self.D = lib().p2o_num_devices(self._h)
        self.k = lib().p2o_num_chunks(self._h)
        self.n_patterns = lib().p2o_num_patterns(self._h)
        self.alphabet = lib().p2o_alphabet_size(self._h)

    def __del__(self):
        if getattr(self, "_h", None):
            lib().p2o_query_free(self._h)
            self._h = None

    def synthesis_hierarchy(self):
        out = np.zeros(lib().p2o_synthesis_levels(self._h) + 1, dtype=np.int32)
        lib().p2o_synthesis_hierarchy(self._h, _p(out, C.c_int32))
        return out.tolist()

    def pattern(self, pid):
        s, f, fl = C.c_int32(), C.c_int32(), C.c_int32()
        g = np.zeros(self.D, dtype=np.int32)
        r = np.zeros(self.D, dtype=np.int32)
        ng = lib().p2o_pattern_info(self._h, pid, C.byref(s), C.byref(f), C.byref(fl), _p(g, C.c_int32), _p(r, C.c_int32))
        if ng < 0:
            raise IndexError(pid)
        return {"slice": s.value, "form": f.value, "form_level": fl.value, "n_groups": ng, "group_of": g, "rank": r}

    def groups(self, pid):
        info = self.pattern(pid)
        out = [[] for _ in range(info["n_groups"])]
        for d in range(self.D):
            if info["group_of"][d] >= 0:
                out[info["group_of"][d]].append(d)
        return out

    def groups_raw(self, slice_level, form, form_level=-1):
        """Groups of one (slice, form) pair before dedupe, as lists of device ids."""
        g = np.zeros(self.D, dtype=np.int32)
        r = np.zeros(self.D, dtype=np.int32)
        ng = lib().p2o_groups_raw(self._h, slice_level, form, form_level, _p(g, C.c_int32), _p(r, C.c_int32))
        if ng < 0:
            raise ValueError("bad slice/form")
        out = [[] for _ in range(ng)]
        for d in range(self.D):
            if g[d] >= 0:
                assert r[d] == len(out[g[d]])
                out[g[d]].append(d)
        return out

    def num_candidates(self, max_len):
        return int(lib().p2o_num_candidates(self._h, max_len))

    def unrank(self, max_len, index):
        buf = np.zeros(MAXLEN, dtype=np.uint8)
        n = lib().p2o_unrank(self._h, max_len, index, _p(buf, C.c_uint8))
        if n < 0:
            raise IndexError(index)
        return buf[:n].tolist()

    def eval_program(self, instr, msg_bytes=()):
        instr = np.ascontiguousarray(np.asarray(instr, dtype=np.uint8))
        msg = _f64(list(msg_bytes))
        cost = np.zeros(max(len(msg), 1), dtype=np.float64)
        ran = C.c_int32()
        ok = lib().p2o_eval_program(self._h, _p(instr, C.c_uint8), len(instr), len(msg), _p(msg, C.c_double),
                                    _p(cost, C.c_double), C.byref(ran))
        return bool(ok), cost[:len(msg)].copy(), ran.value

    def eval_indices(self, max_len, indices=None, start=0, count=0, n_threads=1):
        if indices is not None:
            indices = np.ascontiguousarray(np.asarray(indices, dtype=np.uint64))
            count = len(indices)
            ip = _p(indices, C.c_uint64)
        else:
            ip = None
        valid = np.zeros(max(count, 1), dtype=np.uint8)
        steps = C.c_int64()
        n = lib().p2o_eval_indices(self._h, max_len, ip, start, count, _p(valid, C.c_uint8), C.byref(steps), n_threads)
        return int(n), valid[:count], steps.value

    def synthesize(self, max_len, msg_bytes=(), cap=1 << 20):
        msg = _f64(list(msg_bytes))
        idx = np.zeros(cap, dtype=np.uint64)
        ln = np.zeros(cap, dtype=np.uint8)
        ins = np.zeros((cap, MAXLEN), dtype=np.uint8)
        cost = np.zeros((cap, max(len(msg), 1)), dtype=np.float64)
        tried = C.c_int64()
        n = lib().p2o_synthesize(self._h, max_len, len(msg), _p(msg, C.c_double), _p(idx, C.c_uint64), _p(ln, C.c_uint8),
                                 _p(ins, C.c_uint8), _p(cost, C.c_double), cap, C.byref(tried))
        if n < 0 or n > cap:
            raise RuntimeError("synthesize failed or cap too small: %d" % n)
        return {"index": idx[:n].copy(), "len": ln[:n].copy(), "instr": ins[:n].copy(),
                "cost": cost[:n, :len(msg)].copy(), "steps_tried": tried.value}

    def run_state(self, instr):
        instr = np.ascontiguousarray(np.asarray(instr, dtype=np.uint8))
        st = np.zeros((self.D, self.k, self.D), dtype=np.uint8)
        goal = C.c_int32()
        ran = lib().p2o_run_program_state(self._h, _p(instr, C.c_uint8), len(instr), _p(st, C.c_uint8), C.byref(goal))
        return ran, st, bool(goal.value)


def hierarchy_of_matrix(matrix, reduce_axes, kind):
    """kind: 'column', 'row', 'reduction', 'collapsed' (Sec. 2.4)."""
    x = _i32(matrix)
    m, n = x.shape
    red = np.zeros(m, dtype=np.int32)
    red[list(reduce_axes)] = 1
    out = np.zeros(m * n, dtype=np.int64)
    c = lib().p2o_hierarchy_of_matrix(m, n, _p(x, C.c_int32), _p(red, C.c_int32),
                                      {"column": 0, "row": 1, "reduction": 2, "collapsed": 3}[kind], _p(out, C.c_int64))
    return out[:c].tolist()


def apply_collective(state, op, members):
    """state: bool array [D][k][D]; returns (ok, new_state)."""
    st = np.ascontiguousarray(np.asarray(state, dtype=np.uint8)).copy()
    D, k, D2 = st.shape
    assert D == D2
    mem = _i32(members)
    ok = lib().p2o_apply_collective_raw(D, k, _p(st, C.c_uint8), op, _p(mem, C.c_int32), len(mem))
    if ok < 0:
        raise ValueError("bad arguments")
    return bool(ok), st


def topk(cost, index, k):
    cost = _f64(cost)
    index = np.ascontiguousarray(np.asarray(index, dtype=np.uint64))
    out = np.zeros(max(min(k, len(cost)), 1), dtype=np.int64)
    n = lib().p2o_topk(_p(cost, C.c_double), _p(index, C.c_uint64), len(cost), k, _p(out, C.c_int64))
    if n < 0:
        raise ValueError("NaN cost or bad arguments")
    return out[:n].copy()

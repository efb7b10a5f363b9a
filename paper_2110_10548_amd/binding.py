"""Thin ctypes binding of libp2.so: same names as include/p2.h, argument marshalling only.

Every step of the evaluation runs inside the library's kernels.  Importing this module
fails loudly if the library has not been built (python paper_2110_10548_amd/build.py,
or __graft_entry__.build()).
"""
import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("P2_LIB_PATH", os.path.join(HERE, "libp2.so"))

P2_OK, P2_EINVAL, P2_ENOSPC, P2_EUNSUPPORTED, P2_EDEVICE = 0, -1, -2, -3, -4
ENGINE_AUTO, ENGINE_LITERAL, ENGINE_COMPACT, ENGINE_FRONTIER, ENGINE_SMALL, ENGINE_SHARED = 0, 1, 2, 3, 4, 5
OPS = ("AllReduce", "ReduceScatter", "AllGather", "Reduce", "Broadcast")
FORMS = ("InsideGroup", "Parallel", "Master")


class P2Error(RuntimeError):
    def __init__(self, code, text):
        super().__init__("p2 error %d: %s" % (code, text))
        self.code = code


class p2_hierarchy(C.Structure):
    _fields_ = [("n_levels", C.c_int32), ("card", C.POINTER(C.c_int32)),
                ("bw_bytes_per_s", C.POINTER(C.c_double)), ("alpha_s", C.POINTER(C.c_double))]


class p2_options(C.Structure):
    _fields_ = [("n_chunks", C.c_int32), ("form_mask", C.c_uint32), ("op_mask", C.c_uint32), ("algo", C.c_int32),
                ("topk", C.c_int32), ("engine", C.c_int32), ("hierarchy", C.c_int32), ("flags", C.c_uint32),
                ("max_row_classes", C.c_int32), ("frontier_pairs", C.c_int32), ("hip_stream", C.c_void_p)]


class p2_program(C.Structure):
    _fields_ = [("index", C.c_uint64), ("len", C.c_uint8), ("instr", C.c_uint8 * 7)]


class p2_stats(C.Structure):
    _fields_ = [("candidates", C.c_uint64), ("steps_executed", C.c_uint64), ("literal_reruns", C.c_uint64),
                ("member_visits", C.c_uint64), ("valid", C.c_int64), ("group_size", C.c_int32), ("n_patterns", C.c_int32), ("alphabet", C.c_int32),
                ("engine", C.c_int32), ("steps_evaluated", C.c_uint64), ("members_evaluated", C.c_uint64),
                ("evaluated_with", C.c_int32), ("reserved0", C.c_int32)]


class p2_profile(C.Structure):
    _fields_ = [("eval_ms", C.c_float), ("post_ms", C.c_float), ("eval_launches", C.c_int32), ("post_launches", C.c_int32),
                ("host_plan_ms", C.c_float), ("host_total_ms", C.c_float),
                ("front_ms", C.c_float), ("front_classify_ms", C.c_float), ("front_literal_ms", C.c_float),
                ("front_materialize_ms", C.c_float), ("front_classify_launches", C.c_int32),
                ("front_literal_launches", C.c_int32), ("front_materialize_launches", C.c_int32), ("front_group_ms", C.c_float),
                ("front_prefixes", C.c_double), ("front_classify_state_bytes", C.c_double),
                ("front_classify_lane_ops", C.c_double), ("front_survivors", C.c_double),
                ("front_materialize_bytes", C.c_double), ("front_entries", C.c_double)]


class p2_search_row(C.Structure):
    _fields_ = [("best", p2_program), ("best_cost", C.c_double), ("allreduce_cost", C.c_double), ("valid", C.c_uint64),
                ("candidates", C.c_uint64)]


class p2_query(C.Structure):
    _fields_ = [("h", C.POINTER(p2_hierarchy)), ("axes", C.POINTER(C.c_int32)), ("n_axes", C.c_int32),
                ("placement", C.POINTER(C.c_int32)), ("reduce_axes", C.POINTER(C.c_int32)), ("n_reduce", C.c_int32),
                ("max_len", C.c_int32), ("opt", C.POINTER(p2_options))]


PROGRAM_DTYPE = np.dtype([("index", np.uint64), ("len", np.uint8), ("instr", np.uint8, (7,))])
assert PROGRAM_DTYPE.itemsize == C.sizeof(p2_program) == 16

EXPORTS = ("p2_enumerate_placements", "p2_synthesize", "p2_synthesize_batch", "p2_describe_pattern", "p2_topk",
           "p2_topk_device", "p2_topk_device_noalloc", "p2_last_error", "p2_set_profiling", "p2_get_profile", "p2_search_placements", "p2_measure_alu_peak", "p2_measure_lds_peak", "p2_release_thread")

_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libp2.so is not built: run `python paper_2110_10548_amd/build.py` "
                              "(there is no CPU fallback for the evaluator)")
        # torch ships its own HIP runtime under the same soname as the system one; loading torch
        # first makes the library and torch share one runtime, so torch's device pointers and
        # streams are valid inside the library.
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        i32p, f64p, u64p, i64p = C.POINTER(C.c_int32), C.POINTER(C.c_double), C.POINTER(C.c_uint64), C.POINTER(C.c_int64)
        L.p2_last_error.restype = C.c_char_p
        L.p2_enumerate_placements.restype = C.c_int32
        L.p2_enumerate_placements.argtypes = [C.POINTER(p2_hierarchy), i32p, C.c_int32, i32p, C.c_int64, i64p]
        L.p2_synthesize.restype = C.c_int32
        L.p2_synthesize.argtypes = [C.POINTER(p2_hierarchy), i32p, C.c_int32, i32p, i32p, C.c_int32, C.c_int32, f64p,
                                    C.c_int32, C.POINTER(p2_options), C.c_void_p, f64p, C.c_int64, i64p, u64p,
                                    C.POINTER(p2_stats)]
        L.p2_synthesize_batch.restype = C.c_int32
        L.p2_synthesize_batch.argtypes = [C.POINTER(p2_query), C.c_int32, f64p, C.c_int32, C.c_void_p, f64p, C.c_int64,
                                          i64p, C.POINTER(p2_stats)]
        L.p2_describe_pattern.restype = C.c_int32
        L.p2_describe_pattern.argtypes = [C.POINTER(p2_hierarchy), i32p, C.c_int32, i32p, i32p, C.c_int32,
                                          C.POINTER(p2_options), C.c_int32, i32p, i32p, i32p, i32p, i32p, i32p]
        L.p2_search_placements.restype = C.c_int32
        L.p2_search_placements.argtypes = [C.POINTER(p2_hierarchy), i32p, C.c_int32, i32p, i32p, C.c_int32, f64p, C.c_int32,
                                           C.c_double, C.POINTER(p2_options), i32p, C.POINTER(p2_search_row), f64p, i32p,
                                           C.c_int64, i64p]
        L.p2_measure_alu_peak.restype = C.c_int32
        L.p2_measure_alu_peak.argtypes = [C.c_int32, C.POINTER(C.c_double), C.c_void_p]
        L.p2_measure_lds_peak.restype = C.c_int32
        L.p2_measure_lds_peak.argtypes = [C.c_int32, C.POINTER(C.c_double), C.c_void_p]
        L.p2_topk.restype = C.c_int32
        L.p2_topk.argtypes = [f64p, u64p, C.c_int64, C.c_int32, i64p]
        L.p2_topk_device.restype = C.c_int32
        L.p2_topk_device.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p]
        L.p2_topk_device_noalloc.restype = C.c_int32
        L.p2_topk_device_noalloc.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p,
                                             C.c_void_p]
        L.p2_release_thread.restype = C.c_int32
        L.p2_release_thread.argtypes = []
        L.p2_set_profiling.restype = C.c_int32
        L.p2_set_profiling.argtypes = [C.c_int32]
        L.p2_get_profile.restype = C.c_int32
        L.p2_get_profile.argtypes = [C.POINTER(p2_profile)]
        _lib = L
    return _lib


def _check(rc, allow=()):
    if rc != P2_OK and rc not in allow:
        raise P2Error(rc, lib().p2_last_error().decode())
    return rc


def _i32(x):
    return np.ascontiguousarray(np.asarray(x, dtype=np.int32))


def _f64(x):
    return np.ascontiguousarray(np.asarray(x, dtype=np.float64))


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t))


class _Hier:
    """Keeps the arrays of a p2_hierarchy alive."""

    def __init__(self, card, bw=None, alpha=None):
        self.card = _i32(card)
        self.bw = _f64(bw) if bw is not None else None
        self.alpha = _f64(alpha) if alpha is not None else None
        self.c = p2_hierarchy(len(self.card), _p(self.card, C.c_int32),
                              _p(self.bw, C.c_double) if self.bw is not None else None,
                              _p(self.alpha, C.c_double) if self.alpha is not None else None)


HIERARCHY = {"collapsed": 0, "system": 1, "column": 2, "row": 3, "reduction": 4}


FLAG_EVALUATE_EVERY_QUERY = 1
FLAG_ONE_ENUMERATION_AT_A_TIME = 2


def _options(n_chunks=0, form_mask=7, op_mask=31, algo=0, topk=0, engine=ENGINE_AUTO, stream=None, hierarchy=0, flags=0,
             max_row_classes=0, frontier_pairs=0):
    return p2_options(n_chunks, form_mask, op_mask, algo, topk, engine, HIERARCHY.get(hierarchy, hierarchy), flags,
                      max_row_classes, frontier_pairs, stream)


def p2_enumerate_placements(card, axes):
    """All parallelism matrices [count][n_axes][n_levels] (Sec. 3.1), lexicographic."""
    h, axes = _Hier(card), _i32(axes)
    n = C.c_int64()
    _check(lib().p2_enumerate_placements(C.byref(h.c), _p(axes, C.c_int32), len(axes), None, 0, C.byref(n)))
    out = np.zeros((max(n.value, 1), len(axes), len(h.card)), dtype=np.int32)
    _check(lib().p2_enumerate_placements(C.byref(h.c), _p(axes, C.c_int32), len(axes), _p(out, C.c_int32), n.value, C.byref(n)))
    return out[:n.value]


def p2_describe_pattern(card, axes, placement, reduce_axes, pattern_id, form_mask=7, op_mask=31, hierarchy=0):
    h, axes, placement, red = _Hier(card), _i32(axes), _i32(placement), _i32(reduce_axes)
    opt = _options(form_mask=form_mask, op_mask=op_mask, hierarchy=hierarchy)
    D = int(np.prod(h.card))
    s, f, fl, npat = C.c_int32(), C.c_int32(), C.c_int32(), C.c_int32()
    g = np.zeros(D, dtype=np.int32)
    r = np.zeros(D, dtype=np.int32)
    _check(lib().p2_describe_pattern(C.byref(h.c), _p(axes, C.c_int32), len(axes), _p(placement, C.c_int32),
                                     _p(red, C.c_int32), len(red), C.byref(opt), pattern_id, C.byref(s), C.byref(f),
                                     C.byref(fl), _p(g, C.c_int32), _p(r, C.c_int32), C.byref(npat)))
    return {"slice": s.value, "form": f.value, "form_level": fl.value, "group_of": g, "rank": r, "n_patterns": npat.value}


def p2_num_patterns(card, axes, placement, reduce_axes, form_mask=7, hierarchy=0):
    h, axes, placement, red = _Hier(card), _i32(axes), _i32(placement), _i32(reduce_axes)
    opt = _options(form_mask=form_mask, hierarchy=hierarchy)
    npat = C.c_int32()
    _check(lib().p2_describe_pattern(C.byref(h.c), _p(axes, C.c_int32), len(axes), _p(placement, C.c_int32),
                                     _p(red, C.c_int32), len(red), C.byref(opt), -1, None, None, None, None, None,
                                     C.byref(npat)), allow=(P2_EINVAL,))
    return npat.value


def _stats_dict(s):
    return {k: getattr(s, k) for k, _ in p2_stats._fields_}


class Batch:
    """A marshalled list of queries: the ctypes structures are built once, `run` calls
    p2_synthesize_batch into output buffers that are reused (grown on P2_ENOSPC)."""

    def __init__(self, queries, msg_bytes=(), stream=None):
        self.nq = len(queries)
        self._keep = []
        self._arr = (p2_query * self.nq)()
        for i, q in enumerate(queries):
            h = _Hier(q["card"], q.get("bw"), q.get("alpha"))
            axes, pl, red = _i32(q["axes"]), _i32(q["placement"]), _i32(q["reduce_axes"])
            opt = _options(q.get("n_chunks", 0), q.get("form_mask", 7), q.get("op_mask", 31), q.get("algo", 0), q.get("topk", 0),
                           q.get("engine", ENGINE_AUTO), stream, q.get("hierarchy", 0), q.get("flags", 0),
                           q.get("max_row_classes", 0), q.get("frontier_pairs", 0))
            self._keep.append((h, axes, pl, red, opt))
            self._arr[i] = p2_query(C.pointer(h.c), _p(axes, C.c_int32), len(axes), _p(pl, C.c_int32), _p(red, C.c_int32),
                                    len(red), int(q["max_len"]), C.pointer(opt))
        self._msg = _f64(list(msg_bytes))
        self.n_msg = len(self._msg)
        self._offs = np.zeros(self.nq + 1, dtype=np.int64)
        self._stats = (p2_stats * self.nq)()
        # with a shortlist asked for in every query the number of rows is bounded beforehand, and the
        # first call has room for them; otherwise a first call without room returns the counts
        topks = [int(q.get("topk", 0)) for q in queries]
        self._alloc(sum(topks) * self.n_msg if all(t > 0 for t in topks) and self.n_msg > 0 else 0)

    def _alloc(self, cap):
        self.cap = cap
        self._progs = np.zeros(max(cap, 1), dtype=PROGRAM_DTYPE)
        self._cost = np.zeros((max(cap, 1), max(self.n_msg, 1)), dtype=np.float64)

    def run_raw(self):
        """One p2_synthesize_batch call (two if the output buffers had to grow)."""
        while True:
            rc = lib().p2_synthesize_batch(self._arr, self.nq, _p(self._msg, C.c_double), self.n_msg,
                                           self._progs.ctypes.data_as(C.c_void_p) if self.cap else None,
                                           _p(self._cost, C.c_double) if self.cap else None, self.cap,
                                           _p(self._offs, C.c_int64), self._stats)
            if rc == P2_ENOSPC or (rc == P2_OK and self.cap == 0 and self._offs[self.nq] > 0):
                self._alloc(int(self._offs[self.nq]))
                continue
            _check(rc)
            return

    def results(self):
        out = []
        for i in range(self.nq):
            a, b = int(self._offs[i]), int(self._offs[i + 1])
            out.append({"programs": self._progs[a:b].copy(), "cost": self._cost[a:b, :self.n_msg].copy(),
                        "stats": _stats_dict(self._stats[i])})
        return out

    def run(self):
        self.run_raw()
        return self.results()


def p2_synthesize_batch(queries, msg_bytes=(), cap=None, stream=None):
    """queries: list of dicts with card, bw, alpha, axes, placement, reduce_axes, max_len and optional
    n_chunks, form_mask, op_mask, algo, topk, engine, hierarchy, flags, max_row_classes, frontier_pairs.  Returns a list of results, one per query:
    {"programs": structured array, "cost": [n][n_msg], "stats": dict}."""
    b = Batch(queries, msg_bytes, stream)
    if cap is not None:
        b._alloc(cap)
        _check(lib().p2_synthesize_batch(b._arr, b.nq, _p(b._msg, C.c_double), b.n_msg,
                                         b._progs.ctypes.data_as(C.c_void_p), _p(b._cost, C.c_double), cap,
                                         _p(b._offs, C.c_int64), b._stats))
        return b.results()
    return b.run()


def p2_synthesize(card, axes, placement, reduce_axes, max_len, msg_bytes=(), bw=None, alpha=None, n_chunks=0,
                  form_mask=7, op_mask=31, topk=0, engine=ENGINE_AUTO, cap=None, stream=None, algo=0, hierarchy=0,
                  flags=0, max_row_classes=0):
    """Valid programs of one placement with their simulated costs (through the single-query entry point).
    hierarchy: a P2_HIERARCHY_* number or one of "collapsed", "system", "column", "row", "reduction"."""
    h, axes_a, pl, red = _Hier(card, bw, alpha), _i32(axes), _i32(placement), _i32(reduce_axes)
    opt = _options(n_chunks, form_mask, op_mask, algo, topk, engine, stream, hierarchy, flags, max_row_classes)
    msg = _f64(list(msg_bytes))
    n_msg = len(msg)
    count, cands, st = C.c_int64(), C.c_uint64(), p2_stats()

    def call(progs_p, cost_p, cap_):
        return lib().p2_synthesize(C.byref(h.c), _p(axes_a, C.c_int32), len(axes_a), _p(pl, C.c_int32), _p(red, C.c_int32),
                                   len(red), max_len, _p(msg, C.c_double), n_msg, C.byref(opt), progs_p, cost_p, cap_,
                                   C.byref(count), C.byref(cands), C.byref(st))
    if cap is None:
        _check(call(None, None, 0), allow=(P2_ENOSPC,))
        cap = count.value
    progs = np.zeros(max(cap, 1), dtype=PROGRAM_DTYPE)
    cost = np.zeros((max(cap, 1), max(n_msg, 1)), dtype=np.float64)
    _check(call(progs.ctypes.data_as(C.c_void_p), _p(cost, C.c_double), cap))
    n = count.value
    return {"programs": progs[:n].copy(), "cost": cost[:n, :n_msg].copy(), "candidates": cands.value,
            "stats": _stats_dict(st)}


def p2_search_placements(card, axes, reduce_sets, max_len, msg_bytes, bw=None, alpha=None, weights=None, n_chunks=0,
                         form_mask=7, op_mask=31, algo=0, engine=ENGINE_AUTO, stream=None):
    """Every placement x every requested reduction in one batch: best program, AllReduce baseline, ranking."""
    h, axes_a = _Hier(card, bw, alpha), _i32(axes)
    flat = _i32([a for red in reduce_sets for a in red])
    lens = _i32([len(red) for red in reduce_sets])
    w = _f64(list(weights)) if weights is not None else None
    opt = _options(n_chunks, form_mask, op_mask, algo, 0, engine, stream)
    count = C.c_int64()

    def call(pl_p, rows_p, tot_p, ord_p, cap):
        return lib().p2_search_placements(C.byref(h.c), _p(axes_a, C.c_int32), len(axes_a), _p(flat, C.c_int32),
                                          _p(lens, C.c_int32), len(lens), _p(w, C.c_double) if w is not None else None,
                                          max_len, float(msg_bytes), C.byref(opt), pl_p, rows_p, tot_p, ord_p, cap,
                                          C.byref(count))
    _check(call(None, None, None, None, 0))
    n, ns = count.value, len(lens)
    pls = np.zeros((max(n, 1), len(axes_a), len(card)), dtype=np.int32)
    rows = (p2_search_row * max(n * ns, 1))()
    total = np.zeros(max(n, 1), dtype=np.float64)
    order = np.zeros(max(n, 1), dtype=np.int32)
    _check(call(_p(pls, C.c_int32), rows, _p(total, C.c_double), _p(order, C.c_int32), n))
    out_rows = {}
    for p in range(n):
        for s_ in range(ns):
            r = rows[p * ns + s_]
            out_rows[(p, s_)] = {"valid": int(r.valid), "candidates": int(r.candidates),
                                 "best_index": int(r.best.index) if r.best.len else None,
                                 "best_instr": [int(r.best.instr[t]) for t in range(r.best.len)],
                                 "best_cost": float(r.best_cost), "allreduce_cost": float(r.allreduce_cost)}
    return {"placements": pls[:n].tolist(), "rows": out_rows, "total": total[:n].tolist(), "order": order[:n].tolist()}


def p2_measure_alu_peak(reps=5, stream=None):
    """Measured rate of independent 32-bit integer vector instructions, lane-operations per second."""
    out = C.c_double()
    _check(lib().p2_measure_alu_peak(reps, C.byref(out), stream))
    return out.value


def p2_measure_lds_peak(reps=5, stream=None):
    """Measured rate of 128-bit reads from the local data share, bytes per second."""
    out = C.c_double()
    _check(lib().p2_measure_lds_peak(reps, C.byref(out), stream))
    return out.value


def p2_release_thread():
    _check(lib().p2_release_thread())


def p2_set_profiling(on):
    """False / True, or 2: of the frontier engine's launches time only classification and children."""
    _check(lib().p2_set_profiling(2 if on == 2 and on is not True else 1 if on else 0))


def p2_get_profile():
    p = p2_profile()
    _check(lib().p2_get_profile(C.byref(p)))
    return {k: getattr(p, k) for k, _ in p2_profile._fields_}


def p2_topk(cost, index, k):
    cost = _f64(cost)
    index = np.ascontiguousarray(np.asarray(index, dtype=np.uint64))
    out = np.zeros(max(min(k, len(cost)), 1), dtype=np.int64)
    _check(lib().p2_topk(_p(cost, C.c_double), _p(index, C.c_uint64), len(cost), k, _p(out, C.c_int64)))
    return out[:min(k, len(cost))].copy()


def p2_topk_device(cost_ptr, cost_stride, index_ptr, n, k, out_pos_ptr, stream=None):
    """Device pointers (e.g. torch tensor .data_ptr()); out_pos: int64[min(k, n)] on the device."""
    _check(lib().p2_topk_device(cost_ptr, cost_stride, index_ptr, n, k, out_pos_ptr, stream))


def p2_topk_device_noalloc(cost_ptr, cost_stride, index_ptr, n, k, out_pos_ptr, out_nan_ptr=None, stream=None):
    """Same on the library's fixed scratch (k <= 64): only queues kernels; synchronise the stream before reading."""
    _check(lib().p2_topk_device_noalloc(cost_ptr, cost_stride, index_ptr, n, k, out_pos_ptr, out_nan_ptr, stream))

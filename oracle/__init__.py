"""CPU oracle for batched pipeline-schedule evaluation -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper over ``fporacle.c`` (plain C, int64 times, single-threaded
event loop).  Only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this package; the product
package never does, and this package never imports the product package.

A *problem* is any object with the attributes ``n_devices, n_stages,
n_microbatches, has_w`` (ints) and ``stage_device[S], edge_src[E], edge_dst[E],
edge_comm[E], dur[8][S], mem_units[S], mem_cap[D]`` (array-likes of ints).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fporacle.c")
_LIB = os.path.join(_HERE, "libfporacle.so")
_GEN_SRC = os.path.join(_HERE, "fpgenoracle.c")
_GEN_LIB = os.path.join(_HERE, "libfpgenoracle.so")
_SLIDE_SRC = os.path.join(_HERE, "fpslideoracle.c")
_SLIDE_LIB = os.path.join(_HERE, "libfpslideoracle.so")
_SYNC_SRC = os.path.join(_HERE, "fpsyncoracle.c")
_SYNC_LIB = os.path.join(_HERE, "libfpsyncoracle.so")
_COPY_SRC = os.path.join(_HERE, "fpcopyoracle.c")
_COPY_LIB = os.path.join(_HERE, "libfpcopyoracle.so")

FLAG_DEADLOCK = 1
FLAG_INCOMPLETE = 2
FLAG_OVER_CAP = 4
INT64_MAX = np.iinfo(np.int64).max
NKINDS = 8


def _compile(src: str, lib: str, force: bool) -> str:
    if force or not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(src):
        tmp = lib + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-o", tmp, src])
        os.replace(tmp, lib)
    return lib


def build(force: bool = False) -> str:
    """Compile the oracle's C files with gcc (plain C, no GPU toolchain)."""
    _compile(_GEN_SRC, _GEN_LIB, force)
    _compile(_SLIDE_SRC, _SLIDE_LIB, force)
    _compile(_SYNC_SRC, _SYNC_LIB, force)
    _compile(_COPY_SRC, _COPY_LIB, force)
    return _compile(_SRC, _LIB, force)


class _CProblem(ctypes.Structure):
    _fields_ = [
        ("n_devices", ctypes.c_int32),
        ("n_stages", ctypes.c_int32),
        ("n_microbatches", ctypes.c_int32),
        ("has_w", ctypes.c_int32),
        ("stage_device", ctypes.c_void_p),
        ("n_edges", ctypes.c_int32),
        ("edge_src", ctypes.c_void_p),
        ("edge_dst", ctypes.c_void_p),
        ("edge_comm", ctypes.c_void_p),
        ("dur", ctypes.c_void_p),
        ("mem_units", ctypes.c_void_p),
        ("mem_cap", ctypes.c_void_p),
    ]


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.fporacle_eval_one.restype = ctypes.c_int
        _lib.fporacle_evaluate.restype = ctypes.c_int
        _lib.fporacle_eval_one_mb.restype = ctypes.c_int
        _lib.fporacle_evaluate_mb.restype = ctypes.c_int
        _lib.fporacle_eval_one_links.restype = ctypes.c_int
        _lib.fporacle_evaluate_links.restype = ctypes.c_int
        _lib.fporacle_topk.restype = ctypes.c_int
        _lib.fporacle_rank.restype = ctypes.c_int
    return _lib


def _i32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


class _Marshalled:
    """Keeps the int32 arrays alive next to the C struct that points at them."""

    def __init__(self, problem):
        self.D = int(problem.n_devices)
        self.S = int(problem.n_stages)
        self.m = int(problem.n_microbatches)
        self.arrays = dict(
            stage_device=_i32(problem.stage_device), edge_src=_i32(problem.edge_src),
            edge_dst=_i32(problem.edge_dst), edge_comm=_i32(problem.edge_comm),
            dur=_i32(problem.dur).reshape(NKINDS, self.S), mem_units=_i32(problem.mem_units),
            mem_cap=_i32(problem.mem_cap))
        a = self.arrays
        assert a["stage_device"].shape == (self.S,) and a["mem_cap"].shape == (self.D,)
        self.c = _CProblem(self.D, self.S, self.m, int(problem.has_w),
                           a["stage_device"].ctypes.data, len(a["edge_src"]),
                           a["edge_src"].ctypes.data, a["edge_dst"].ctypes.data,
                           a["edge_comm"].ctypes.data, a["dur"].ctypes.data,
                           a["mem_units"].ctypes.data, a["mem_cap"].ctypes.data)


def decode(words):
    """(kind, chunk, micro-batch) of each op word."""
    w = np.ascontiguousarray(np.asarray(words, dtype=np.uint16))
    k = np.empty(w.shape, np.int32)
    c = np.empty(w.shape, np.int32)
    j = np.empty(w.shape, np.int32)
    _load().fporacle_decode(ctypes.c_void_p(w.ctypes.data), ctypes.c_int64(w.size),
                            ctypes.c_void_p(k.ctypes.data), ctypes.c_void_p(c.ctypes.data),
                            ctypes.c_void_p(j.ctypes.data))
    return k, c, j


def _mb_table(mp, dur_mb):
    """``dur_mb[8][S][m]`` as a contiguous int32 array (None stays None)."""
    if dur_mb is None:
        return None
    t = np.ascontiguousarray(np.asarray(dur_mb, dtype=np.int32))
    assert t.shape == (NKINDS, mp.S, mp.m), t.shape
    return t


def evaluate(problem, words, threads: int = 1, dur_mb=None, links: bool = False, variant_loop: bool = False):
    """Evaluate a batch ``words[C][D][stride]`` (uint16).

    Returns dict(makespan int64[C], idle int64[C][D], peak int32[C][D],
    flags uint8[C]).  ``threads`` > 1 only splits the batch over host threads;
    every candidate is still evaluated by the same single-threaded C routine.
    ``dur_mb[8][S][m]``: per-micro-batch costs in place of ``problem.dur``.  ``links``: every ordered
    pair of devices is a link that carries one value at a time (see fporacle_evaluate_links).  Without either
    the plain definition runs (eval_one in fporacle.c); ``variant_loop`` sends such a call through the
    variants' loop with both switches off instead (for the tests that compare the two loops).
    """
    lib = _load()
    mp = _Marshalled(problem)
    table = _mb_table(mp, dur_mb)
    plain = table is None and not links and not variant_loop
    table_ptr = ctypes.c_void_p(table.ctypes.data if table is not None else None)
    w = np.ascontiguousarray(np.asarray(words, dtype=np.uint16))
    assert w.ndim == 3 and w.shape[1] == mp.D, w.shape
    C, _, stride = w.shape
    out = dict(makespan=np.empty(C, np.int64), idle=np.empty((C, mp.D), np.int64),
               peak=np.empty((C, mp.D), np.int32), flags=np.empty(C, np.uint8))

    def run(lo, hi):
        if hi <= lo:
            return 0
        if plain:
            return lib.fporacle_evaluate(
                ctypes.byref(mp.c), ctypes.c_void_p(w[lo:hi].ctypes.data), ctypes.c_int64(hi - lo),
                ctypes.c_int32(stride), ctypes.c_void_p(out["makespan"][lo:hi].ctypes.data),
                ctypes.c_void_p(out["idle"][lo:hi].ctypes.data),
                ctypes.c_void_p(out["peak"][lo:hi].ctypes.data),
                ctypes.c_void_p(out["flags"][lo:hi].ctypes.data))
        if links:
            return lib.fporacle_evaluate_links(
                ctypes.byref(mp.c), table_ptr, ctypes.c_void_p(w[lo:hi].ctypes.data), ctypes.c_int64(hi - lo),
                ctypes.c_int32(stride), ctypes.c_void_p(out["makespan"][lo:hi].ctypes.data),
                ctypes.c_void_p(out["idle"][lo:hi].ctypes.data),
                ctypes.c_void_p(out["peak"][lo:hi].ctypes.data),
                ctypes.c_void_p(out["flags"][lo:hi].ctypes.data))
        return lib.fporacle_evaluate_mb(
            ctypes.byref(mp.c), table_ptr, ctypes.c_void_p(w[lo:hi].ctypes.data), ctypes.c_int64(hi - lo),
            ctypes.c_int32(stride), ctypes.c_void_p(out["makespan"][lo:hi].ctypes.data),
            ctypes.c_void_p(out["idle"][lo:hi].ctypes.data),
            ctypes.c_void_p(out["peak"][lo:hi].ctypes.data),
            ctypes.c_void_p(out["flags"][lo:hi].ctypes.data))

    threads = max(1, min(int(threads), C if C else 1))
    if threads == 1:
        rcs = [run(0, C)]
    else:
        # many small slices so that uneven candidates balance over the threads
        n_slices = min(C, threads * 8)
        bounds = np.linspace(0, C, n_slices + 1).astype(np.int64)
        with ThreadPoolExecutor(threads) as ex:
            rcs = list(ex.map(lambda i: run(int(bounds[i]), int(bounds[i + 1])), range(n_slices)))
    if any(rcs):
        raise ValueError("fporacle: invalid problem description")
    return out


def evaluate_trace(problem, words_one, dur_mb=None, links: bool = False, variant_loop: bool = False):
    """One candidate ``words[D][stride]``; also returns every op's start/finish."""
    lib = _load()
    mp = _Marshalled(problem)
    table = _mb_table(mp, dur_mb)
    w = np.ascontiguousarray(np.asarray(words_one, dtype=np.uint16))
    assert w.ndim == 2 and w.shape[0] == mp.D
    stride = w.shape[1]
    ms = np.empty(1, np.int64)
    idle = np.empty(mp.D, np.int64)
    peak = np.empty(mp.D, np.int32)
    fl = np.empty(1, np.uint8)
    st = np.empty((mp.D, stride), np.int64)
    fi = np.empty((mp.D, stride), np.int64)
    tail = (ctypes.c_void_p(w.ctypes.data), ctypes.c_int32(stride), ctypes.c_void_p(ms.ctypes.data),
            ctypes.c_void_p(idle.ctypes.data), ctypes.c_void_p(peak.ctypes.data), ctypes.c_void_p(fl.ctypes.data),
            ctypes.c_void_p(st.ctypes.data), ctypes.c_void_p(fi.ctypes.data))
    table_ptr = ctypes.c_void_p(table.ctypes.data if table is not None else None)
    if table is None and not links and not variant_loop:
        rc = lib.fporacle_eval_one(ctypes.byref(mp.c), *tail)
    else:
        rc = (lib.fporacle_eval_one_links if links else lib.fporacle_eval_one_mb)(ctypes.byref(mp.c), table_ptr, *tail)
    if rc:
        raise ValueError("fporacle: invalid problem description")
    return dict(makespan=int(ms[0]), idle=idle, peak=peak, flags=int(fl[0]), start=st, finish=fi)


def topk(makespan, flags, k: int):
    """k best feasible candidates by (makespan, index).  Returns (idx[k], makespan[k], count)."""
    lib = _load()
    ms = np.ascontiguousarray(np.asarray(makespan, dtype=np.int64))
    fl = np.ascontiguousarray(np.asarray(flags, dtype=np.uint8))
    idx = np.empty(k, np.int64)
    oms = np.empty(k, np.int64)
    cnt = np.zeros(1, np.int32)
    lib.fporacle_topk(ctypes.c_void_p(ms.ctypes.data), ctypes.c_void_p(fl.ctypes.data),
                      ctypes.c_int64(ms.size), ctypes.c_int32(k), ctypes.c_void_p(idx.ctypes.data),
                      ctypes.c_void_p(oms.ctypes.data), ctypes.c_void_p(cnt.ctypes.data))
    return idx, oms, int(cnt[0])


RANK_MODES = {"makespan": 0, "makespan_peak": 1, "peak_makespan": 2, "idle": 3}


def rank(results, k: int, mode: str = "makespan_peak", include_over_cap: bool = False):
    """k best candidates of evaluated ``results`` (dict as returned by ``evaluate``) by a two-part
    key.  Returns (idx[k], k1[k], k2[k], count)."""
    lib = _load()
    ms = np.ascontiguousarray(results["makespan"], dtype=np.int64)
    idle = np.ascontiguousarray(results["idle"], dtype=np.int64)
    peak = np.ascontiguousarray(results["peak"], dtype=np.int32)
    fl = np.ascontiguousarray(results["flags"], dtype=np.uint8)
    n, D = idle.shape if idle.ndim == 2 else (0, 1)
    idx, k1, k2 = np.empty(k, np.int64), np.empty(k, np.int64), np.empty(k, np.int64)
    cnt = np.zeros(1, np.int32)
    rc = lib.fporacle_rank(ctypes.c_void_p(ms.ctypes.data), ctypes.c_void_p(idle.ctypes.data),
                           ctypes.c_void_p(peak.ctypes.data), ctypes.c_void_p(fl.ctypes.data),
                           ctypes.c_int64(n), ctypes.c_int32(D), ctypes.c_int32(k),
                           ctypes.c_int32(RANK_MODES[mode]), ctypes.c_int32(int(include_over_cap)),
                           ctypes.c_void_p(idx.ctypes.data), ctypes.c_void_p(k1.ctypes.data),
                           ctypes.c_void_p(k2.ctypes.data), ctypes.c_void_p(cnt.ctypes.data))
    if rc:
        raise ValueError("fporacle_rank: bad mode")
    return idx, k1, k2, int(cnt[0])


def pareto(results, kmax: int):
    """Pareto front of (makespan, largest peak) over the completed candidates of ``results``.
    Returns (idx[kmax], makespan[kmax], peak[kmax], count), ascending makespan."""
    lib = _load()
    ms = np.ascontiguousarray(results["makespan"], dtype=np.int64)
    peak = np.ascontiguousarray(results["peak"], dtype=np.int32)
    fl = np.ascontiguousarray(results["flags"], dtype=np.uint8)
    n, D = peak.shape if peak.ndim == 2 else (0, 1)
    idx, oms, opk = np.empty(kmax, np.int64), np.empty(kmax, np.int64), np.empty(kmax, np.int32)
    cnt = np.zeros(1, np.int32)
    lib.fporacle_pareto(ctypes.c_void_p(ms.ctypes.data), ctypes.c_void_p(peak.ctypes.data),
                        ctypes.c_void_p(fl.ctypes.data), ctypes.c_int64(n), ctypes.c_int32(D),
                        ctypes.c_int32(kmax), ctypes.c_void_p(idx.ctypes.data), ctypes.c_void_p(oms.ctypes.data),
                        ctypes.c_void_p(opk.ctypes.data), ctypes.c_void_p(cnt.ctypes.data))
    return idx, oms, opk, int(cnt[0])


def apply_caps(results, caps):
    """Flags of ``results`` with OVER_CAP recomputed against ``caps`` ([D] or [n][D])."""
    lib = _load()
    peak = np.ascontiguousarray(results["peak"], dtype=np.int32)
    fl = np.array(results["flags"], dtype=np.uint8, copy=True)
    caps = np.ascontiguousarray(caps, dtype=np.int32)
    n, D = peak.shape if peak.ndim == 2 else (0, 1)
    per = 1 if caps.ndim == 2 else 0
    assert caps.shape == ((n, D) if per else (D,))
    lib.fporacle_apply_caps(ctypes.c_void_p(peak.ctypes.data), ctypes.c_void_p(caps.ctypes.data),
                            ctypes.c_int32(per), ctypes.c_int64(n), ctypes.c_int32(D),
                            ctypes.c_void_p(fl.ctypes.data))
    return fl


# ---------------------------------------------------------------------------------------------
# weight-gradient sliding oracle (fpslideoracle.c)

_slide_lib = None


def wslide(problem, words, stride_out: int, threads: int = 1, links: bool = False):
    """Slide the weight-gradient items of a batch ``words[C][D][stride]`` into idle time.
    Returns dict(ops uint16[C][D][stride_out], makespan, idle, peak, flags) of the new lists.
    links: under the link-occupancy variant of the cost model."""
    global _slide_lib
    if _slide_lib is None:
        _slide_lib = ctypes.CDLL(_compile(_SLIDE_SRC, _SLIDE_LIB, False))
        _slide_lib.fpslide_oracle_batch_links.restype = ctypes.c_int
    mp = _Marshalled(problem)   # the same field layout as fpslide_problem
    w = np.ascontiguousarray(np.asarray(words, dtype=np.uint16))
    assert w.ndim == 3 and w.shape[1] == mp.D, w.shape
    C, _, stride = w.shape
    out = dict(ops=np.zeros((C, mp.D, stride_out), np.uint16), makespan=np.empty(C, np.int64),
               idle=np.empty((C, mp.D), np.int64), peak=np.empty((C, mp.D), np.int32),
               flags=np.empty(C, np.uint8))

    def run(lo, hi):
        if hi <= lo:
            return 0
        return _slide_lib.fpslide_oracle_batch_links(
            ctypes.byref(mp.c), ctypes.c_int32(1 if links else 0), ctypes.c_void_p(w[lo:hi].ctypes.data),
            ctypes.c_int64(hi - lo),
            ctypes.c_int32(stride), ctypes.c_void_p(out["ops"][lo:hi].ctypes.data), ctypes.c_int32(stride_out),
            ctypes.c_void_p(out["makespan"][lo:hi].ctypes.data), ctypes.c_void_p(out["idle"][lo:hi].ctypes.data),
            ctypes.c_void_p(out["peak"][lo:hi].ctypes.data), ctypes.c_void_p(out["flags"][lo:hi].ctypes.data))

    threads = max(1, min(int(threads), C if C else 1))
    bounds = np.linspace(0, C, min(C, threads * 8) + 1).astype(np.int64) if C else np.zeros(1, np.int64)
    with ThreadPoolExecutor(threads) as ex:
        rcs = list(ex.map(lambda i: run(int(bounds[i]), int(bounds[i + 1])), range(len(bounds) - 1)))
    if any(rcs):
        raise ValueError("fpslideoracle: needs a problem with split backward and at most 4 stages per device")
    return out


# ---------------------------------------------------------------------------------------------
# schedule generator oracle (fpgenoracle.c)

POLICY_INTS = 8
CTTP_BWD_FIRST, CTTP_FWD_FIRST, CTTP_INTERLEAVED = 0, 1, 2
DIR_BREADTH, DIR_DEPTH = 0, 1
GEN_STUCK = 1
GEN_OVERFLOW = 2


class _CGenProblem(ctypes.Structure):
    _fields_ = [
        ("n_devices", ctypes.c_int32),
        ("n_stages", ctypes.c_int32),
        ("n_microbatches", ctypes.c_int32),
        ("has_w", ctypes.c_int32),
        ("stage_device", ctypes.c_void_p),
        ("n_edges", ctypes.c_int32),
        ("edge_src", ctypes.c_void_p),
        ("edge_dst", ctypes.c_void_p),
    ]


_gen_lib = None


def _load_gen():
    global _gen_lib
    if _gen_lib is None:
        build()
        _gen_lib = ctypes.CDLL(_GEN_LIB)
        _gen_lib.fpgen_oracle_one.restype = ctypes.c_int
        _gen_lib.fpgen_oracle_generate.restype = ctypes.c_int
    return _gen_lib


def generate(problem, policy, inflight, stride: int, threads: int = 1, diagnostics: bool = False):
    """Run the scheduler on n parameter sets.

    policy int32 [n][D][8] = (cttp, unit1, unit2, forward direction, forward interval or 0,
    backward direction, backward interval or 0, 0) per actor; inflight int32 [n][S].
    Returns dict(words uint16 [n][D][stride], steps int32 [n], status uint8 [n]) and, with
    ``diagnostics``, prefix_violations int32 [n] (see fpgenoracle.c).
    """
    lib = _load_gen()
    D, S = int(problem.n_devices), int(problem.n_stages)
    arrays = (_i32(problem.stage_device), _i32(problem.edge_src), _i32(problem.edge_dst))
    cp = _CGenProblem(D, S, int(problem.n_microbatches), int(problem.has_w), arrays[0].ctypes.data,
                      len(arrays[1]), arrays[1].ctypes.data, arrays[2].ctypes.data)
    pol = _i32(policy)
    inf = _i32(inflight)
    assert pol.ndim == 3 and pol.shape[1:] == (D, POLICY_INTS), pol.shape
    n = pol.shape[0]
    assert inf.shape == (n, S), inf.shape
    out = dict(words=np.zeros((n, D, stride), np.uint16), steps=np.zeros(n, np.int32),
               status=np.zeros(n, np.uint8))
    viol = np.zeros(n, np.int32)

    def run(lo, hi):
        rc = 0
        for i in range(lo, hi):
            rc |= lib.fpgen_oracle_one(
                ctypes.byref(cp), ctypes.c_void_p(pol[i].ctypes.data), ctypes.c_void_p(inf[i].ctypes.data),
                ctypes.c_int32(stride), ctypes.c_void_p(out["words"][i].ctypes.data),
                ctypes.c_void_p(out["steps"][i:].ctypes.data), ctypes.c_void_p(out["status"][i:].ctypes.data),
                ctypes.c_void_p(viol[i:].ctypes.data))
        return rc

    threads = max(1, min(int(threads), n if n else 1))
    if threads == 1:
        rcs = [run(0, n)]
    else:
        bounds = np.linspace(0, n, min(n, threads * 8) + 1).astype(np.int64)
        with ThreadPoolExecutor(threads) as ex:
            rcs = list(ex.map(lambda i: run(int(bounds[i]), int(bounds[i + 1])), range(len(bounds) - 1)))
    if any(rcs):
        raise ValueError("fpgenoracle: invalid problem or policy")
    if diagnostics:
        out["prefix_violations"] = viol
    return out


# ---- synchronisation stages and dependency pairs (fpsyncoracle.c) ---------------------------------

class _CSyncProblem(ctypes.Structure):
    _fields_ = _CProblem._fields_ + [("group", ctypes.c_void_p), ("n_pairs", ctypes.c_int32),
                                      ("pairs", ctypes.c_void_p)]


_sync_lib = None


def _load_sync():
    global _sync_lib
    if _sync_lib is None:
        build()
        _sync_lib = ctypes.CDLL(_SYNC_LIB)
        _sync_lib.fpsync_eval_one.restype = ctypes.c_int
        _sync_lib.fpsync_evaluate.restype = ctypes.c_int
    return _sync_lib


def _sync_problem(problem, group, pairs):
    mp = _Marshalled(problem)
    grp = _i32(np.ones(mp.S, np.int32) if group is None else group)
    prs = _i32(np.zeros((0, 5), np.int32) if pairs is None else pairs).reshape(-1, 5)
    assert grp.shape == (mp.S,)
    a = mp.arrays
    c = _CSyncProblem(mp.D, mp.S, mp.m, int(problem.has_w), a["stage_device"].ctypes.data, len(a["edge_src"]),
                      a["edge_src"].ctypes.data, a["edge_dst"].ctypes.data, a["edge_comm"].ctypes.data,
                      a["dur"].ctypes.data, a["mem_units"].ctypes.data, a["mem_cap"].ctypes.data,
                      grp.ctypes.data, len(prs), prs.ctypes.data)
    return mp, c, (grp, prs)


def evaluate_sync(problem, words, group=None, pairs=None, threads: int = 1):
    """Evaluate ``words[C][D][stride]`` under the model with synchronisation stages and dependency pairs
    (fpsyncoracle.c): ``group[S]`` micro-batches per item of each stage (None = 1 everywhere), ``pairs``
    rows (kind_from, stage_from, kind_to, stage_to, latency).  Returns the dict of ``evaluate``."""
    lib = _load_sync()
    mp, c, keep = _sync_problem(problem, group, pairs)
    w = np.ascontiguousarray(np.asarray(words, dtype=np.uint16))
    assert w.ndim == 3 and w.shape[1] == mp.D, w.shape
    C, _, stride = w.shape
    out = dict(makespan=np.empty(C, np.int64), idle=np.empty((C, mp.D), np.int64),
               peak=np.empty((C, mp.D), np.int32), flags=np.empty(C, np.uint8))

    def run(lo, hi):
        if hi <= lo:
            return 0
        return lib.fpsync_evaluate(ctypes.byref(c), ctypes.c_void_p(w[lo:hi].ctypes.data), ctypes.c_int64(hi - lo),
                                   ctypes.c_int32(stride), ctypes.c_void_p(out["makespan"][lo:hi].ctypes.data),
                                   ctypes.c_void_p(out["idle"][lo:hi].ctypes.data),
                                   ctypes.c_void_p(out["peak"][lo:hi].ctypes.data),
                                   ctypes.c_void_p(out["flags"][lo:hi].ctypes.data))

    threads = max(1, min(int(threads), C if C else 1))
    if threads == 1:
        rcs = [run(0, C)]
    else:
        n_slices = min(C, threads * 8)
        bounds = np.linspace(0, C, n_slices + 1).astype(np.int64)
        with ThreadPoolExecutor(threads) as ex:
            rcs = list(ex.map(lambda i: run(int(bounds[i]), int(bounds[i + 1])), range(n_slices)))
    if any(rcs):
        raise ValueError("fpsyncoracle: invalid problem description")
    return out


def evaluate_sync_trace(problem, words_one, group=None, pairs=None):
    """One candidate ``words[D][stride]`` under the same model; also every op's start and finish."""
    lib = _load_sync()
    mp, c, keep = _sync_problem(problem, group, pairs)
    w = np.ascontiguousarray(np.asarray(words_one, dtype=np.uint16))
    assert w.ndim == 2 and w.shape[0] == mp.D
    stride = w.shape[1]
    ms, fl = np.empty(1, np.int64), np.empty(1, np.uint8)
    idle, peak = np.empty(mp.D, np.int64), np.empty(mp.D, np.int32)
    st, fi = np.empty((mp.D, stride), np.int64), np.empty((mp.D, stride), np.int64)
    rc = lib.fpsync_eval_one(ctypes.byref(c), ctypes.c_void_p(w.ctypes.data), ctypes.c_int32(stride),
                             ctypes.c_void_p(ms.ctypes.data), ctypes.c_void_p(idle.ctypes.data),
                             ctypes.c_void_p(peak.ctypes.data), ctypes.c_void_p(fl.ctypes.data),
                             ctypes.c_void_p(st.ctypes.data), ctypes.c_void_p(fi.ctypes.data))
    if rc:
        raise ValueError("fpsyncoracle: invalid problem description")
    return dict(makespan=int(ms[0]), idle=idle, peak=peak, flags=int(fl[0]), start=st, finish=fi)


# ---- a copy engine for offload and reload items (fpcopyoracle.c) ----------------------------------

_copy_lib = None


def _load_copy():
    global _copy_lib
    if _copy_lib is None:
        build()
        _copy_lib = ctypes.CDLL(_COPY_LIB)
        _copy_lib.fpcopy_eval_one.restype = ctypes.c_int
        _copy_lib.fpcopy_evaluate.restype = ctypes.c_int
    return _copy_lib


def evaluate_copy(problem, words, depth: int = 4, threads: int = 1):
    """Evaluate ``words[C][D][stride]`` under the model in which offload and reload items run on a copy
    engine that holds at most ``depth`` transfers (fpcopyoracle.c).  Returns the dict of ``evaluate``."""
    lib = _load_copy()
    mp = _Marshalled(problem)
    w = np.ascontiguousarray(np.asarray(words, dtype=np.uint16))
    assert w.ndim == 3 and w.shape[1] == mp.D, w.shape
    C, _, stride = w.shape
    out = dict(makespan=np.empty(C, np.int64), idle=np.empty((C, mp.D), np.int64),
               peak=np.empty((C, mp.D), np.int32), flags=np.empty(C, np.uint8))

    def run(lo, hi):
        if hi <= lo:
            return 0
        return lib.fpcopy_evaluate(ctypes.byref(mp.c), ctypes.c_int32(depth), ctypes.c_void_p(w[lo:hi].ctypes.data),
                                   ctypes.c_int64(hi - lo), ctypes.c_int32(stride),
                                   ctypes.c_void_p(out["makespan"][lo:hi].ctypes.data),
                                   ctypes.c_void_p(out["idle"][lo:hi].ctypes.data),
                                   ctypes.c_void_p(out["peak"][lo:hi].ctypes.data),
                                   ctypes.c_void_p(out["flags"][lo:hi].ctypes.data))

    threads = max(1, min(int(threads), C if C else 1))
    if threads == 1:
        rcs = [run(0, C)]
    else:
        n_slices = min(C, threads * 8)
        bounds = np.linspace(0, C, n_slices + 1).astype(np.int64)
        with ThreadPoolExecutor(threads) as ex:
            rcs = list(ex.map(lambda i: run(int(bounds[i]), int(bounds[i + 1])), range(n_slices)))
    if any(rcs):
        raise ValueError("fpcopyoracle: invalid problem description or depth")
    return out


def evaluate_copy_trace(problem, words_one, depth: int = 4):
    """One candidate ``words[D][stride]`` under the same model; also every op's start and finish."""
    lib = _load_copy()
    mp = _Marshalled(problem)
    w = np.ascontiguousarray(np.asarray(words_one, dtype=np.uint16))
    assert w.ndim == 2 and w.shape[0] == mp.D
    stride = w.shape[1]
    ms, fl = np.empty(1, np.int64), np.empty(1, np.uint8)
    idle, peak = np.empty(mp.D, np.int64), np.empty(mp.D, np.int32)
    st, fi = np.empty((mp.D, stride), np.int64), np.empty((mp.D, stride), np.int64)
    rc = lib.fpcopy_eval_one(ctypes.byref(mp.c), ctypes.c_int32(depth), ctypes.c_void_p(w.ctypes.data),
                             ctypes.c_int32(stride), ctypes.c_void_p(ms.ctypes.data), ctypes.c_void_p(idle.ctypes.data),
                             ctypes.c_void_p(peak.ctypes.data), ctypes.c_void_p(fl.ctypes.data),
                             ctypes.c_void_p(st.ctypes.data), ctypes.c_void_p(fi.ctypes.data))
    if rc:
        raise ValueError("fpcopyoracle: invalid problem description or depth")
    return dict(makespan=int(ms[0]), idle=idle, peak=peak, flags=int(fl[0]), start=st, finish=fi)

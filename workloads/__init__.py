"""Seeded synthetic inputs: the five benchmark problems and their candidate batches.

Input generation only -- no evaluation.  ``config(i)`` builds problem ``i``
(1..5) with its seeded duration tables; ``generate(spec, ...)`` list-schedules
candidates with the C generator ``fpgen.c`` (built with gcc on first use).
Neither the CPU oracle nor the GPU package is imported here.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

from .problem import (B, F, FD, L, MAX_CHUNKS, NKINDS, NO_CAP, O, R, W, Problem, chain_problem,
                      gpipe_lists, make_problem, one_f_one_b_lists, pack_lists, pack_word)

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fpgen.c")
_LIB = os.path.join(_HERE, "libfpgen.so")
_SYNC_SRC = os.path.join(_HERE, "fpsyncgen.c")
_SYNC_LIB = os.path.join(_HERE, "libfpsyncgen.so")
BASE_SEED = 0xF1E0


def build(force: bool = False) -> str:
    for src, lib in ((_SYNC_SRC, _SYNC_LIB), (_SRC, _LIB)):
        if force or not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(src):
            tmp = lib + ".tmp.%d" % os.getpid()
            subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-pthread", "-o", tmp, src])
            os.replace(tmp, lib)
    return _LIB


class _CParams(ctypes.Structure):
    _fields_ = [
        ("n_devices", ctypes.c_int32), ("n_stages", ctypes.c_int32),
        ("n_microbatches", ctypes.c_int32), ("has_w", ctypes.c_int32),
        ("stage_device", ctypes.c_void_p), ("n_edges", ctypes.c_int32),
        ("edge_src", ctypes.c_void_p), ("edge_dst", ctypes.c_void_p), ("edge_comm", ctypes.c_void_p),
        ("dur", ctypes.c_void_p),
        ("recompute", ctypes.c_int32), ("offload", ctypes.c_int32),
        ("max_marks_per_device", ctypes.c_int32), ("cap_units", ctypes.c_int32),
        ("seed", ctypes.c_uint64),
        ("deadlock_per_mille", ctypes.c_int32), ("benign_per_mille", ctypes.c_int32),
    ]


@dataclass
class Spec:
    """A benchmark configuration: the problem plus the generator's knobs."""

    index: int
    problem: Problem
    n_candidates: int
    stride: int               # words per device row (multiple of 64)
    top_k: int
    recompute: int = 0
    offload: int = 0
    max_marks_per_device: int = 0
    cap_units: int = 0
    deadlock_per_mille: int = 0
    benign_per_mille: int = 10
    seed: int = BASE_SEED
    fixed_cases: tuple = ()   # names of textbook orders appended after the generated ones


def _mix64(x):
    x = (x + 0x9E3779B97F4A7C15) & 0xFFFFFFFFFFFFFFFF
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & 0xFFFFFFFFFFFFFFFF
    return x ^ (x >> 31)


class _TableRng:
    """Counter-based integers for the seeded duration tables."""

    def __init__(self, seed):
        self.key, self.ctr = _mix64(seed), 0

    def uniform_int(self, lo, hi):
        self.ctr += 1
        return lo + _mix64(self.key ^ (self.ctr * 0x2545F4914F6CDD1D & 0xFFFFFFFFFFFFFFFF)) % (hi - lo + 1)


def config(index: int, n_candidates: int | None = None) -> Spec:
    """The five benchmark configurations (stage counts, durations, caps, batch sizes)."""
    rng = _TableRng(BASE_SEED + index)
    if index == 1:
        prob = chain_problem(4, 8, v=1, f=2, b=4, comm=1, name="cfg1_p4_m8_FB")
        return Spec(1, prob, n_candidates or 1024, 64, 16, cap_units=4, seed=BASE_SEED + 1,
                    fixed_cases=("gpipe", "1f1b"))
    if index in (2, 3, 4):
        p, m, v = {2: (8, 32, 2), 3: (16, 64, 2), 4: (32, 128, 2)}[index]
        S = p * v
        if index == 2:
            dur = {F: [rng.uniform_int(8, 12) for _ in range(S)], B: [rng.uniform_int(14, 20) for _ in range(S)],
                   W: [rng.uniform_int(6, 10) for _ in range(S)]}
            comm = [rng.uniform_int(1, 3) for _ in range(S - 1)]
            cap = 3 * p // 2
        elif index == 3:
            def jit(base):
                return [base + rng.uniform_int(-(base // 10), base // 10) for _ in range(S)]
            dur = {F: jit(10), B: jit(20), W: jit(10)}
            for k in (F, B, W):
                dur[k][0] = (13 * dur[k][0] + 5) // 10          # embedding stage: 1.3x
                dur[k][S - 1] = (16 * dur[k][S - 1] + 5) // 10  # LM head + loss: 1.6x
            comm = [1] * (S - 1)
            cap = p
        else:
            dur = {F: [rng.uniform_int(20, 30) for _ in range(S)], B: [rng.uniform_int(40, 60) for _ in range(S)],
                   W: [rng.uniform_int(15, 25) for _ in range(S)]}
            comm = [rng.uniform_int(2, 6) for _ in range(S - 1)]
            cap = 3 * p // 4
        dur[FD] = list(dur[F])
        dur[R] = list(dur[F])
        edges = [(s, s + 1, comm[s]) for s in range(S - 1)]
        prob = make_problem(p, S, m, 1, [s % p for s in range(S)], edges, dur, mem_cap=cap,
                            name=f"cfg{index}_p{p}_m{m}_v{v}")
        base_len = 3 * m * v
        if index == 4:
            return Spec(4, prob, n_candidates or 65536, 896, 128, recompute=1, max_marks_per_device=128,
                        cap_units=cap, seed=BASE_SEED + 4)
        return Spec(index, prob, n_candidates or {2: 65536, 3: 262144}[index], -(-base_len // 64) * 64,
                    {2: 16, 3: 64}[index], cap_units=cap, seed=BASE_SEED + index,
                    deadlock_per_mille=20 if index == 2 else 0)
    if index == 5:
        # two towers of 6 stages (vision 0..5, text 6..11) merging into 4 fusion stages 12..15
        m = 64
        f = [12] * 6 + [8] * 6 + [16] * 4
        dur = {F: f, B: [2 * x for x in f], W: list(f), FD: list(f), R: list(f), O: 5, L: 5}
        edges = [(s, s + 1, 1) for s in range(5)] + [(5, 12, 1)]
        edges += [(s, s + 1, 1) for s in range(6, 11)] + [(11, 12, 1)]
        edges += [(s, s + 1, 1) for s in range(12, 15)]
        prob = make_problem(16, 16, m, 1, list(range(16)), edges, dur, mem_cap=12, name="cfg5_two_towers")
        return Spec(5, prob, n_candidates or 131072, 256, 64, offload=1, max_marks_per_device=32,
                    cap_units=12, seed=BASE_SEED + 5, deadlock_per_mille=10)
    raise ValueError("config index must be 1..5")


def _i32(a):
    return np.ascontiguousarray(np.asarray(a, np.int32))


def generate(spec: Spec, n: int | None = None, first: int = 0, threads: int | None = None,
             with_generator_clock: bool = False, out: np.ndarray | None = None):
    """Candidates [first, first+n) of ``spec`` as uint16[n][D][stride] (+ fixed cases when the
    range reaches the end of the batch).  ``out`` may be a preallocated (e.g. pinned) buffer."""
    lib = ctypes.CDLL(build())
    lib.fpgen_generate.restype = ctypes.c_int
    p = spec.problem
    total = spec.n_candidates
    n = total - first if n is None else n
    arrs = [_i32(p.stage_device), _i32(p.edge_src), _i32(p.edge_dst), _i32(p.edge_comm), _i32(p.dur)]
    cp = _CParams(p.n_devices, p.n_stages, p.n_microbatches, p.has_w, arrs[0].ctypes.data,
                  len(arrs[1]), arrs[1].ctypes.data, arrs[2].ctypes.data, arrs[3].ctypes.data,
                  arrs[4].ctypes.data, spec.recompute, spec.offload, spec.max_marks_per_device,
                  spec.cap_units, spec.seed, spec.deadlock_per_mille, spec.benign_per_mille)
    n_fixed = len(spec.fixed_cases) if first + n >= total else 0
    shape = (n + n_fixed, p.n_devices, spec.stride)
    if out is None:
        out = np.zeros(shape, np.uint16)
    assert out.shape == shape and out.dtype == np.uint16 and out.flags.c_contiguous
    clock = np.full(n + n_fixed, -1, np.int64)
    threads = threads or min(16, os.cpu_count() or 1)
    rc = lib.fpgen_generate(ctypes.byref(cp), ctypes.c_int64(first), ctypes.c_int64(n),
                            ctypes.c_int32(spec.stride), ctypes.c_void_p(out.ctypes.data),
                            ctypes.c_void_p(clock.ctypes.data), ctypes.c_int32(threads))
    if rc:
        raise RuntimeError(f"fpgen_generate failed ({rc})")
    for i, name in enumerate(spec.fixed_cases[:n_fixed]):
        lists = {"gpipe": gpipe_lists, "1f1b": one_f_one_b_lists}[name](p.n_devices, p.n_microbatches)
        out[n + i] = pack_lists(lists, spec.stride)
    return (out, clock) if with_generator_clock else out


def count_ops(words: np.ndarray) -> int:
    """Number of real (non-END) op words that an evaluator reads: per row, up to the first END."""
    w = words.reshape(-1, words.shape[-1])
    is_end = (w >> 13) == 0
    first_end = np.where(is_end.any(1), is_end.argmax(1), w.shape[1])
    return int(first_end.sum())


# ---------------------------------------------------------------------------------------------
# parameter sets for the schedule generator (inputs only: the scheduler itself is not here)

POLICY_INTS = 8
NO_LIMIT = 2**31 - 1


def policy_sets(problem: Problem, n: int, seed: int = BASE_SEED + 100):
    """n seeded parameter sets for the scheduler: (policy int32 [n][D][8], inflight int32 [n][S]).

    The mix follows the tuner's grid (schedule types = computation type traversal priority x stage
    traversal priorities, per placement) widened by per-actor settings and in-flight limits:
    * half of the sets use one policy for all actors, the others one per actor;
    * computation type priority: backward-first 50 %, interleaved 40 % (units 1, sometimes 2-3),
      forward-first 10 %;
    * stage traversal: direction uniform; interval not set 40 %, else one of p/2, p, 2p or 1..4
      (p = number of devices);
    * in-flight limit per stage (v = stages per device): none 5 %; 1F1B-like
      ceil((p - d) / v) + slack for a per-set slack in [0, p/4] 50 %; one uniform limit in [2, p/2]
      for all stages 45 %.
    """
    rng = np.random.default_rng(seed)
    D, S = problem.n_devices, problem.n_stages
    per_actor = rng.random(n) < 0.5
    pol = np.zeros((n, D, POLICY_INTS), np.int32)
    shape = (n, D)
    cttp = rng.choice(3, size=shape, p=[0.5, 0.1, 0.4]).astype(np.int32)
    big_unit = rng.random(shape) < 0.25
    unit_f = np.where((cttp == 2) & big_unit, rng.integers(2, 4, shape), 1)
    unit_b = np.where((cttp == 2) & big_unit, rng.integers(1, 4, shape), 1)
    choices = np.array([max(1, D // 2), D, 2 * D, 1, 2, 3, 4], np.int32)

    def interval():
        v = choices[rng.integers(0, len(choices), shape)]
        return np.where(rng.random(shape) < 0.4, 0, v)

    fields = [cttp, unit_f, unit_b, rng.integers(0, 2, shape), interval(), rng.integers(0, 2, shape), interval()]
    for i, f in enumerate(fields):
        f = np.asarray(f, np.int32)
        pol[:, :, i] = np.where(per_actor[:, None], f, f[:, :1])
    kind = rng.random(n)
    dev = np.asarray(problem.stage_device, np.int64)
    v = max(1, int(np.bincount(dev, minlength=D).max()))
    slack = rng.integers(0, D // 4 + 1, n)
    flat = rng.integers(2, max(3, D // 2 + 1), n)
    like_1f1b = -(-(D - dev) // v)[None, :] + slack[:, None]
    inflight = np.where(kind[:, None] < 0.05, NO_LIMIT,
                        np.where(kind[:, None] < 0.55, like_1f1b, flat[:, None])).astype(np.int32)
    return pol, np.broadcast_to(inflight, (n, S)).copy()


def microbatch_costs(problem: Problem, seed: int = BASE_SEED + 200) -> np.ndarray:
    """Seeded costs per micro-batch, int32 [NKINDS][S][m]: the problem's cost of every (type, stage)
    scaled by a per-micro-batch factor drawn uniformly from [1/2, 3/2) in steps of 1/256 and rounded to
    the nearest integer -- micro-batches that pack sequences of unequal total length."""
    rng = np.random.default_rng(seed)
    base = np.asarray(problem.dur, np.int64).reshape(NKINDS, problem.n_stages)[:, :, None]
    factor = rng.integers(128, 384, problem.n_microbatches)[None, None, :]
    return ((base * factor + 128) >> 8).astype(np.int32)


def generator_stride(problem: Problem) -> int:
    """Row stride (words, multiple of 8) that holds the longest list the scheduler can emit."""
    per_dev = int(np.bincount(problem.stage_device, minlength=problem.n_devices).max())
    longest = per_dev * problem.n_microbatches * (3 if problem.has_w else 2)
    return max(8, -(-longest // 8) * 8)


# ---------------------------------------------------------------------------------------------
# problems with synchronisation stages and dependency pairs (inputs only)

class _CSyncParams(ctypes.Structure):
    _fields_ = [
        ("n_devices", ctypes.c_int32), ("n_stages", ctypes.c_int32),
        ("n_microbatches", ctypes.c_int32), ("has_w", ctypes.c_int32),
        ("stage_device", ctypes.c_void_p), ("n_edges", ctypes.c_int32),
        ("edge_src", ctypes.c_void_p), ("edge_dst", ctypes.c_void_p),
        ("group", ctypes.c_void_p), ("n_pairs", ctypes.c_int32), ("pairs", ctypes.c_void_p),
        ("seed", ctypes.c_uint64), ("swap_per_mille", ctypes.c_int32),
    ]


@dataclass
class SyncSpec:
    """A problem with synchronisation stages: the plain description plus the group size of every stage
    and the dependency pairs (rows kind_from, stage_from, kind_to, stage_to, latency)."""

    problem: Problem
    group: np.ndarray
    pairs: np.ndarray
    n_candidates: int
    stride: int
    top_k: int
    seed: int = BASE_SEED + 300
    swap_per_mille: int = 20


def sync_config(n_candidates: int | None = None, sync_every: int = 4) -> SyncSpec:
    """The multimodal workload with a registered synchronisation (paper Sections 2.2, 4.2 and 7.2: two
    submodules whose last stages exchange their output states through a synchronisation instruction, once
    every few micro-batches): a vision tower of 6 stages (F 12, B 24, W 12) on devices 0..5 and a text
    tower of 6 stages (F 8, B 16, W 8) on devices 6..11, as in configuration 5, both feeding a
    synchronisation stage on device 11 that gathers every `sync_every` micro-batches (cost 6, its backward
    item 2, no activation of its own); 64 micro-batches, latency 1, split backward, cap 12 units per
    device; one user pair: the vision tower's first stage starts a micro-batch after the text tower's
    first stage has finished it.  65,536 candidates, top-64.  Stands in for the paper's CLIP runs."""
    m = 64
    f = [12] * 6 + [8] * 6 + [6]
    dur = {F: f, B: [24] * 6 + [16] * 6 + [2], W: [12] * 6 + [8] * 6 + [0], FD: list(f), R: list(f), O: 5, L: 5}
    edges = [(s, s + 1, 1) for s in range(5)] + [(s, s + 1, 1) for s in range(6, 11)] + [(5, 12, 1), (11, 12, 1)]
    prob = make_problem(12, 13, m, 1, list(range(12)) + [11], edges, dur, mem_units=[1] * 12 + [0], mem_cap=12,
                        name=f"multimodal_sync_every_{sync_every}")
    group = np.asarray([1] * 12 + [sync_every], np.int32)
    pairs = np.asarray([[F, 6, F, 0, 1]], np.int32)
    # longest row: device 11 holds a tower stage and the synchronisation stage
    longest = 3 * m + 3 * (-(-m // sync_every))
    return SyncSpec(prob, group, pairs, n_candidates or 65536, -(-(longest + 1) // 8) * 8, 64)


def generate_sync(spec: SyncSpec, n: int | None = None, first: int = 0, threads: int | None = None) -> np.ndarray:
    """Candidates [first, first + n) of ``spec`` as uint16 [n][D][stride] (fpsyncgen.c: randomised
    step-wise list scheduling over groups and pairs; orders only)."""
    from concurrent.futures import ThreadPoolExecutor
    build()
    lib = ctypes.CDLL(_SYNC_LIB)
    lib.fpsyncgen_generate.restype = ctypes.c_int
    p = spec.problem
    n = spec.n_candidates - first if n is None else n
    arrs = [_i32(p.stage_device), _i32(p.edge_src), _i32(p.edge_dst), _i32(spec.group),
            _i32(spec.pairs).reshape(-1, 5)]
    cp = _CSyncParams(p.n_devices, p.n_stages, p.n_microbatches, p.has_w, arrs[0].ctypes.data, len(arrs[1]),
                      arrs[1].ctypes.data, arrs[2].ctypes.data, arrs[3].ctypes.data, len(arrs[4]),
                      arrs[4].ctypes.data, spec.seed, spec.swap_per_mille)
    out = np.zeros((n, p.n_devices, spec.stride), np.uint16)
    threads = max(1, min(threads or min(16, os.cpu_count() or 1), n or 1))
    bounds = np.linspace(0, n, threads * 4 + 1).astype(np.int64)

    def run(i):
        lo, hi = int(bounds[i]), int(bounds[i + 1])
        if hi <= lo:
            return 0
        return lib.fpsyncgen_generate(ctypes.byref(cp), ctypes.c_int64(first + lo), ctypes.c_int64(hi - lo),
                                      ctypes.c_int32(spec.stride), ctypes.c_void_p(out[lo:hi].ctypes.data))

    with ThreadPoolExecutor(threads) as ex:
        if any(ex.map(run, range(len(bounds) - 1))):
            raise RuntimeError("fpsyncgen_generate failed")
    return out

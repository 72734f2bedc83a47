"""Plain containers and fixed textbook orders for pipeline-schedule inputs.

This module holds input *descriptions* only (tables of integers and per-device
op orders); it computes no start/finish time, memory figure or flag.  It is
shared by the tests, the benchmark, the CPU oracle's callers and the GPU
binding's callers, and imports neither of the two implementations.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

# op kinds of the 16-bit op word (kind<<13 | chunk<<11 | micro-batch)
END, F, B, W, R, O, L, FD = range(8)
NKINDS = 8
KIND_NAMES = ("END", "F", "B", "W", "R", "O", "L", "FD")
MAX_CHUNKS = 4
MAX_MB = 2048
NO_CAP = np.iinfo(np.int32).max


@dataclass
class Problem:
    """One pipeline-parallel training problem (paper Section 4.1 data model:
    stages in a DAG, a stage->actor placement; Section 3: profiled costs)."""

    n_devices: int
    n_stages: int
    n_microbatches: int
    has_w: int
    stage_device: np.ndarray   # [S]
    edge_src: np.ndarray       # [E]
    edge_dst: np.ndarray       # [E]
    edge_comm: np.ndarray      # [E]
    dur: np.ndarray            # [NKINDS][S]
    mem_units: np.ndarray      # [S]
    mem_cap: np.ndarray        # [D]
    name: str = ""
    notes: dict = field(default_factory=dict)

    def local_stage(self):
        """[D][MAX_CHUNKS] stage id of each device-local chunk (-1 = none)."""
        ls = -np.ones((self.n_devices, MAX_CHUNKS), np.int32)
        cnt = [0] * self.n_devices
        for s in range(self.n_stages):
            d = int(self.stage_device[s])
            ls[d, cnt[d]] = s
            cnt[d] += 1
        return ls

    def stage_chunk(self):
        """[S] device-local chunk index of each stage."""
        ch = np.zeros(self.n_stages, np.int32)
        cnt = [0] * self.n_devices
        for s in range(self.n_stages):
            d = int(self.stage_device[s])
            ch[s] = cnt[d]
            cnt[d] += 1
        return ch


def make_problem(n_devices, n_stages, n_microbatches, has_w, stage_device, edges, dur,
                 mem_units=None, mem_cap=None, name="", notes=None):
    """edges: iterable of (src, dst, comm); dur: dict kind->[S] or array [NKINDS][S]."""
    S = n_stages
    edges = list(edges)
    if isinstance(dur, dict):
        table = np.zeros((NKINDS, S), np.int32)
        for k, row in dur.items():
            table[k] = np.broadcast_to(np.asarray(row, np.int32), (S,))
    else:
        table = np.asarray(dur, np.int32).reshape(NKINDS, S).copy()
    return Problem(
        n_devices=int(n_devices), n_stages=int(S), n_microbatches=int(n_microbatches),
        has_w=int(has_w), stage_device=np.asarray(stage_device, np.int32).copy(),
        edge_src=np.asarray([e[0] for e in edges], np.int32),
        edge_dst=np.asarray([e[1] for e in edges], np.int32),
        edge_comm=np.asarray([e[2] for e in edges], np.int32),
        dur=table,
        mem_units=(np.ones(S, np.int32) if mem_units is None
                   else np.broadcast_to(np.asarray(mem_units, np.int32), (S,)).copy()),
        mem_cap=(np.full(n_devices, NO_CAP, np.int32) if mem_cap is None
                 else np.broadcast_to(np.asarray(mem_cap, np.int32), (n_devices,)).copy()),
        name=name, notes=dict(notes or {}))


def chain_problem(p, m, v=1, f=1, b=1, w=None, comm=0, mem_cap=None, r=None, name=""):
    """Chain of S = p*v stages with circular placement dev(s) = s mod p
    (paper Section 2.1: one-to-one for v=1, circular for v>1)."""
    S = p * v
    dur = {F: f, B: b, FD: f, R: (f if r is None else r)}
    if w is not None:
        dur[W] = w
    edges = [(s, s + 1, comm) for s in range(S - 1)]
    return make_problem(p, S, m, int(w is not None), [s % p for s in range(S)], edges, dur,
                        mem_cap=mem_cap, name=name or f"chain_p{p}_m{m}_v{v}")


def pack_word(kind, chunk, mb):
    return (int(kind) << 13) | (int(chunk) << 11) | int(mb)


def pack_lists(lists, stride=None, align=8):
    """lists[d] = [(kind, chunk, mb), ...]  ->  uint16[D][stride], END-padded."""
    longest = max((len(x) for x in lists), default=0)
    if stride is None:
        stride = max(align, -(-longest // align) * align)
    assert stride >= longest
    out = np.zeros((len(lists), stride), np.uint16)
    for d, ops in enumerate(lists):
        for i, (k, c, j) in enumerate(ops):
            out[d, i] = pack_word(k, c, j)
    return out


def gpipe_lists(p, m):
    """GPipe: every device runs all forwards, then all backwards (v=1, no W)."""
    return [[(F, 0, j) for j in range(m)] + [(B, 0, j) for j in range(m)] for _ in range(p)]


def one_f_one_b_lists(p, m):
    """1F1B (paper Section 2.1, one-to-one placement): device d runs
    min(m, p-d-1) warm-up forwards, then forward/backward pairs, then drains."""
    out = []
    for d in range(p):
        warm = min(m, p - d - 1)
        ops = [(F, 0, j) for j in range(warm)]
        nf, nb = warm, 0
        while nb < m:
            if nf < m:
                ops.append((F, 0, nf))
                nf += 1
            ops.append((B, 0, nb))
            nb += 1
        out.append(ops)
    return out


def interleaved_1f1b_lists(p, v, m):
    """Interleaved 1F1B (paper Section 2.1: the circular placement, stage s on device s mod p), as the
    schedule is defined where it was published (Narayanan et al., SC'21): the m * v forward items of a
    device are numbered k = 0, 1, ... in groups of p micro-batches per chunk, chunks ascending (item k =
    chunk (k div p) mod v, micro-batch (k div pv) p + k mod p); the backward items likewise with the
    chunks descending; device d runs 2 (p - d - 1) + (v - 1) p forward items to warm up, then
    alternates one forward and one backward item, then drains the backward items.  m must be a
    multiple of p.  Items are (kind, chunk, micro-batch)."""
    assert m % p == 0 and v >= 1
    total = m * v

    def item(k, forward):
        c = (k // p) % v
        return (F if forward else B, c if forward else v - 1 - c, (k // (p * v)) * p + k % p)

    out = []
    for d in range(p):
        warm = min(2 * (p - d - 1) + (v - 1) * p, total)
        ops = [item(k, True) for k in range(warm)]
        for i in range(total - warm):
            ops += [item(warm + i, True), item(i, False)]
        ops += [item(i, False) for i in range(total - warm, total)]
        out.append(ops)
    return out

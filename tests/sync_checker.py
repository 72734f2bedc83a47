"""Independent checker for the model with synchronisation stages and dependency pairs (pins
``oracle/fpsyncoracle.c``; never the GPU path).

Critical-path method, not an event loop: one node per listed op, an edge from each op to the next op of
its device, an edge for every dependency (stage DAG and pairs, expanded over the micro-batch groups), a
cycle test by Kahn's algorithm, finish time = longest path (node weight = cost, edge weight = latency);
memory and legality from an order-only scan of each list.  Pure Python, small cases only.
"""
from __future__ import annotations

from collections import deque

END, F, B, W, R, O, L, FD = range(8)
_TRANS = {F: ("absent", "res"), FD: ("absent", "disc"), R: ("disc", "res"), O: ("res", "off"),
          L: ("off", "res"), B: ("res", "bdone"), W: ("bdone", "done")}
_FAILED = dict(deadlock=True, incomplete=None, makespan=None, idle=None, peak=None)


def check(problem, words, group=None, pairs=()):
    """One candidate words[D][stride] -> dict(deadlock, incomplete, makespan, idle, peak)."""
    D, S, m = problem.n_devices, problem.n_stages, problem.n_microbatches
    group = [1] * S if group is None else [int(x) for x in group]
    n_items = [-(-m // n) for n in group]
    dev = [int(x) for x in problem.stage_device]
    stages_of = [[s for s in range(S) if dev[s] == d] for d in range(D)]
    lists = []
    for d in range(D):
        ops = []
        for w in words[d]:
            w = int(w)
            if w >> 13 == END:
                break
            c = (w >> 11) & 3
            ops.append((w >> 13, stages_of[d][c] if c < len(stages_of[d]) else None, w & 0x7FF))
        lists.append(ops)

    # order-only scan: legality at each position, memory, busy time
    state, peak, busy = {}, [0] * D, [0] * D
    for d, ops in enumerate(lists):
        mem = 0
        for kind, s, g in ops:
            if s is None or g >= n_items[s] or (kind == W and not problem.has_w):
                return _FAILED
            need, nxt = _TRANS[kind]
            if state.get((s, g), "absent") != need:
                return _FAILED
            state[(s, g)] = nxt
            u = int(problem.mem_units[s])
            if kind in (F, FD, R, L):
                mem += u
                peak[d] = max(peak[d], mem)
            if kind in (FD, O, W) or (kind == B and not problem.has_w):
                mem -= u
            busy[d] += int(problem.dur[kind][s])

    # who produces what: (class, stage, item) -> node
    cls = {F: "f", FD: "f", B: "b", W: "w"}
    where = {}
    for d, ops in enumerate(lists):
        for i, (kind, s, g) in enumerate(ops):
            if kind in cls:
                where[(cls[kind], s, g)] = (d, i)
    # what an item waits for: [(class, producer stage, latency)] per (consumer kind, stage)
    waits = {}
    for a, b, c in zip(problem.edge_src, problem.edge_dst, problem.edge_comm):
        a, b, c = int(a), int(b), int(c)
        lat = c if dev[a] != dev[b] else 0
        for kind in (F, FD):
            waits.setdefault((kind, b), []).append(("f", a, lat))
        waits.setdefault((B, a), []).append(("b", b, lat))
    for k1, s1, k2, s2, lat in pairs:
        k1, s1, k2, s2, lat = int(k1), int(s1), int(k2), int(s2), int(lat)
        for kind in ((F, FD) if k2 == F else (k2,)):
            waits.setdefault((kind, s2), []).append((cls[k1], s1, lat if dev[s1] != dev[s2] else 0))

    edges_in = {}
    for d, ops in enumerate(lists):
        for i, (kind, s, g) in enumerate(ops):
            ins = [((d, i - 1), 0)] if i else []
            lo, hi = g * group[s], min(m, (g + 1) * group[s]) - 1
            for c, a, lat in waits.get((kind, s), []):
                for ga in range(lo // group[a], hi // group[a] + 1):
                    if (c, a, ga) not in where:
                        return _FAILED          # waits for an item that is in no list
                    ins.append((where[(c, a, ga)], lat))
            edges_in[(d, i)] = ins

    indeg = {n: len(e) for n, e in edges_in.items()}
    out_edges = {n: [] for n in edges_in}
    for n, ins in edges_in.items():
        for src, wgt in ins:
            out_edges[src].append((n, wgt))
    ready = {n: 0 for n in edges_in}
    finish = {}
    q = deque(n for n in edges_in if indeg[n] == 0)
    while q:
        n = q.popleft()
        kind, s, g = lists[n[0]][n[1]]
        finish[n] = ready[n] + int(problem.dur[kind][s])
        for nxt, wgt in out_edges[n]:
            ready[nxt] = max(ready[nxt], finish[n] + wgt)
            indeg[nxt] -= 1
            if indeg[nxt] == 0:
                q.append(nxt)
    if len(finish) != len(edges_in):
        return _FAILED
    terminal = "done" if problem.has_w else "bdone"
    incomplete = any(state.get((s, g), "absent") != terminal for s in range(S) for g in range(n_items[s]))
    makespan = max(finish.values(), default=0)
    return dict(deadlock=False, incomplete=incomplete, makespan=makespan, idle=[makespan - b for b in busy],
                peak=peak, finish=finish)

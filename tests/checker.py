"""Independent checker used only to pin the CPU oracle (never the GPU path).

Textbook critical-path method instead of an event loop: build the union graph
of one candidate (device-order edges + dependency edges), test it for cycles
with Kahn's algorithm, take every op's finish time as the longest path into it
(node weight = duration, edge weight = communication latency), and get the
memory peak from an order-only prefix scan of each device's list.  Pure Python
dictionaries; meant for small cases.
"""
from __future__ import annotations

from collections import deque

END, F, B, W, R, O, L, FD = range(8)

# activation state machine, written as {kind: (required state, next state)}
_ABSENT, _RES, _DISC, _OFF, _BDONE, _DONE = "absent", "res", "disc", "off", "bdone", "done"
_TRANS = {F: (_ABSENT, _RES), FD: (_ABSENT, _DISC), R: (_DISC, _RES), O: (_RES, _OFF),
          L: (_OFF, _RES), B: (_RES, _BDONE), W: (_BDONE, _DONE)}


def decode_lists(problem, words):
    """uint16[D][stride] -> per-device [(kind, stage or None, mb, chunk)] up to the first END."""
    ls = problem.local_stage()
    out = []
    for d in range(problem.n_devices):
        ops = []
        for w in words[d]:
            w = int(w)
            kind, chunk, mb = w >> 13, (w >> 11) & 3, w & 0x7FF
            if kind == END:
                break
            stage = int(ls[d][chunk]) if ls[d][chunk] >= 0 else None
            ops.append((kind, stage, mb, chunk))
        out.append(ops)
    return out


def check(problem, words, dur_mb=None, links=False):
    """Returns dict(deadlock, incomplete, makespan, idle, peak, finish) for one candidate.

    dur_mb[kind][stage][micro-batch], if given, is the weight of every node instead of
    problem.dur[kind][stage].  links: every value sent to another device becomes a node of its own
    (weight = the edge's latency) between its producer and its consumer, and the transfer nodes of one
    ordered pair of devices form a chain in the order their producers stand in the sending device's list
    (several values of one producer: in the order of the edge list) -- a link carries one value at a time."""
    D, S, m = problem.n_devices, problem.n_stages, problem.n_microbatches

    def weight(kind, s, j):
        return int(dur_mb[kind][s][j]) if dur_mb is not None else int(problem.dur[kind][s])
    lists = decode_lists(problem, words)
    dev = [int(x) for x in problem.stage_device]
    preds = {s: [] for s in range(S)}
    succs = {s: [] for s in range(S)}
    for a, b, c in zip(problem.edge_src, problem.edge_dst, problem.edge_comm):
        preds[int(b)].append((int(a), int(c)))
        succs[int(a)].append((int(b), int(c)))

    # 1. order-only pass per device: legality of each op at its position,
    #    memory prefix scan, final states.
    state = {}
    stuck = False
    peak = [0] * D
    busy = [0] * D
    valid_len = []
    for d, ops in enumerate(lists):
        mem = 0
        n_ok = 0
        for kind, s, j, _chunk in ops:
            if s is None or j >= m or (kind == W and not problem.has_w):
                stuck = True
                break
            need, nxt = _TRANS[kind]
            if state.get((s, j), _ABSENT) != need:
                stuck = True
                break
            state[(s, j)] = nxt
            u = int(problem.mem_units[s])
            if kind in (F, FD, R, L):
                mem += u
                peak[d] = max(peak[d], mem)
            if kind in (FD, O):
                mem -= u
            if kind == W or (kind == B and not problem.has_w):
                mem -= u
            busy[d] += weight(kind, s, j)
            n_ok += 1
        valid_len.append(n_ok)
    if stuck:
        return dict(deadlock=True, incomplete=None, makespan=None, idle=None, peak=None, finish=None)

    # 2. union graph over all ops
    where_fwd, where_bwd = {}, {}
    for d, ops in enumerate(lists):
        for i, (kind, s, j, _c) in enumerate(ops):
            if kind in (F, FD):
                where_fwd[(s, j)] = (d, i)
            elif kind == B:
                where_bwd[(s, j)] = (d, i)
    edges_in = {}
    nodes = [(d, i) for d, ops in enumerate(lists) for i in range(len(ops))]
    for n in nodes:
        edges_in[n] = []
    missing_producer = False
    transfer_weight = {}
    for d, ops in enumerate(lists):
        for i, (kind, s, j, _c) in enumerate(ops):
            if i > 0:
                edges_in[(d, i)].append(((d, i - 1), 0))
            if kind in (F, FD):
                for sp, c in preds[s]:
                    if (sp, j) not in where_fwd:
                        missing_producer = True
                    elif links and dev[sp] != d:
                        edges_in[(d, i)].append((("send", "f", sp, s, j), 0))
                    else:
                        edges_in[(d, i)].append((where_fwd[(sp, j)], c if dev[sp] != d else 0))
            elif kind == B:
                for sn, c in succs[s]:
                    if (sn, j) not in where_bwd:
                        missing_producer = True
                    elif links and dev[sn] != d:
                        edges_in[(d, i)].append((("send", "b", sn, s, j), 0))
                    else:
                        edges_in[(d, i)].append((where_bwd[(sn, j)], c if dev[sn] != d else 0))
    if missing_producer:
        return dict(deadlock=True, incomplete=None, makespan=None, idle=None, peak=None, finish=None)
    if links:
        # one node per value sent to another device; per ordered device pair a chain in sending order
        last_on_link = {}
        edge_list = list(zip(problem.edge_src, problem.edge_dst, problem.edge_comm))
        for d, ops in enumerate(lists):
            for i, (kind, s, j, _c) in enumerate(ops):
                if kind not in (F, FD, B):
                    continue
                for a, b, c in edge_list:   # in the order of the edge list
                    a, b, c = int(a), int(b), int(c)
                    if kind == B:
                        if b != s or dev[a] == d:
                            continue
                        node, to = ("send", "b", s, a, j), dev[a]
                    else:
                        if a != s or dev[b] == d:
                            continue
                        node, to = ("send", "f", s, b, j), dev[b]
                    nodes.append(node)
                    transfer_weight[node] = c
                    edges_in[node] = [((d, i), 0)]
                    if (d, to) in last_on_link:
                        edges_in[node].append((last_on_link[(d, to)], 0))
                    last_on_link[(d, to)] = node
        # a consumer may name a transfer whose producer never runs: then it is stuck
        for n in list(nodes):
            for src, _w in edges_in[n]:
                if src not in edges_in:
                    return dict(deadlock=True, incomplete=None, makespan=None, idle=None, peak=None, finish=None)

    # 3. Kahn + longest path
    indeg = {n: len(edges_in[n]) for n in nodes}
    out_edges = {n: [] for n in nodes}
    for n in nodes:
        for src, wgt in edges_in[n]:
            out_edges[src].append((n, wgt))
    ready = {n: 0 for n in nodes}
    finish = {}
    q = deque(n for n in nodes if indeg[n] == 0)
    done = 0
    while q:
        n = q.popleft()
        if n in transfer_weight:
            finish[n] = ready[n] + transfer_weight[n]
        else:
            d, i = n
            kind, s, j, _c = lists[d][i]
            finish[n] = ready[n] + weight(kind, s, j)
        done += 1
        for nxt, wgt in out_edges[n]:
            ready[nxt] = max(ready[nxt], finish[n] + wgt)
            indeg[nxt] -= 1
            if indeg[nxt] == 0:
                q.append(nxt)
    if done != len(nodes):
        return dict(deadlock=True, incomplete=None, makespan=None, idle=None, peak=None, finish=None)

    terminal = _DONE if problem.has_w else _BDONE
    incomplete = any(state.get((s, j), _ABSENT) != terminal for s in range(S) for j in range(m))
    finish = {n: t for n, t in finish.items() if n not in transfer_weight}   # the ops' own finish times
    makespan = max(finish.values(), default=0)
    return dict(deadlock=False, incomplete=incomplete, makespan=makespan,
                idle=[makespan - b for b in busy], peak=peak, finish=finish)

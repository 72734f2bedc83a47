"""Independent checker for the copy-engine model (pins ``oracle/fpcopyoracle.c``; never the GPU path).

No event loop: the ops of one candidate are put into a dependency graph (the op in front of it in its list;
for a copy item the copy item before it and the one `depth` places before it; for a backward item the
reload of its activation; the stage DAG), visited in topological order (Kahn), and every op's times follow
from the recurrences of the model.  Memory: all events of a device sorted by (time, timeline, position).
Pure Python, small cases only."""
from __future__ import annotations

from collections import deque

END, F, B, W, R, O, L, FD = range(8)
_TRANS = {F: ("absent", "res"), FD: ("absent", "disc"), R: ("disc", "res"), O: ("res", "off"),
          L: ("off", "res"), B: ("res", "bdone"), W: ("bdone", "done")}
_FAILED = dict(deadlock=True, incomplete=None, makespan=None, idle=None, peak=None)


def check(problem, words, depth=4):
    D, S, m = problem.n_devices, problem.n_stages, problem.n_microbatches
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
    # legality in list order
    state = {}
    for d, ops in enumerate(lists):
        for kind, s, j in ops:
            if s is None or j >= m or (kind == W and not problem.has_w):
                return _FAILED
            need, nxt = _TRANS[kind]
            if state.get((s, j), "absent") != need:
                return _FAILED
            state[(s, j)] = nxt
    preds = {s: [] for s in range(S)}
    succs = {s: [] for s in range(S)}
    for a, b, c in zip(problem.edge_src, problem.edge_dst, problem.edge_comm):
        preds[int(b)].append((int(a), int(c)))
        succs[int(a)].append((int(b), int(c)))
    where_f, where_b = {}, {}
    for d, ops in enumerate(lists):
        for i, (kind, s, j) in enumerate(ops):
            if kind in (F, FD):
                where_f[(s, j)] = (d, i)
            if kind == B:
                where_b[(s, j)] = (d, i)
    # dependency graph
    needs = {}
    for d, ops in enumerate(lists):
        copies, last_reload = [], {}
        for i, (kind, s, j) in enumerate(ops):
            n = [("walk", (d, i - 1))] if i else []
            if kind in (O, L):
                if copies:
                    n.append(("engine", copies[-1]))
                if len(copies) >= depth:
                    n.append(("room", copies[-depth]))
                copies.append((d, i))
                if kind == L:
                    last_reload[(s, j)] = (d, i)
            elif kind in (F, FD):
                for sp, c in preds[s]:
                    if (sp, j) not in where_f:
                        return _FAILED
                    n.append(("input", where_f[(sp, j)], c if dev[sp] != d else 0))
            elif kind == B:
                for sn, c in succs[s]:
                    if (sn, j) not in where_b:
                        return _FAILED
                    n.append(("input", where_b[(sn, j)], c if dev[sn] != d else 0))
                if (s, j) in last_reload:
                    n.append(("input", last_reload[(s, j)], 0))
            needs[(d, i)] = n
    indeg = {n: len(v) for n, v in needs.items()}
    users = {n: [] for n in needs}
    for n, v in needs.items():
        for dep in v:
            users[dep[1]].append(n)
    start, finish, leave = {}, {}, {}      # leave: when the walk moves on behind the op
    q = deque(n for n in needs if indeg[n] == 0)
    while q:
        n = q.popleft()
        kind, s, j = lists[n[0]][n[1]]
        reach = room = engine = ready = 0
        for dep in needs[n]:
            if dep[0] == "walk":
                reach = leave[dep[1]]
            elif dep[0] == "room":
                room = finish[dep[1]]
            elif dep[0] == "engine":
                engine = finish[dep[1]]
            else:
                ready = max(ready, finish[dep[1]] + dep[2])
        if kind in (O, L):
            leave[n] = max(reach, room)
            start[n] = max(leave[n], engine)
            finish[n] = start[n] + int(problem.dur[kind][s])
        else:
            start[n] = max(reach, ready)
            finish[n] = leave[n] = start[n] + int(problem.dur[kind][s])
        for u in users[n]:
            indeg[u] -= 1
            if indeg[u] == 0:
                q.append(u)
    if len(finish) != len(needs):
        return _FAILED
    terminal = "done" if problem.has_w else "bdone"
    incomplete = any(state.get((s, j), "absent") != terminal for s in range(S) for j in range(m))
    makespan = max(finish.values(), default=0)
    peak, idle = [], []
    for d, ops in enumerate(lists):
        events, busy = [], 0
        for i, (kind, s, j) in enumerate(ops):
            u = int(problem.mem_units[s])
            line = 1 if kind in (O, L) else 0
            if kind in (F, FD, R, L):
                events.append((start[(d, i)], line, i, 0, u))
            if kind in (FD, O, W) or (kind == B and not problem.has_w):
                events.append((finish[(d, i)], line, i, 1, -u))
            if not line:
                busy += int(problem.dur[kind][s])
        mem = top = 0
        for _t, _line, _i, _o, delta in sorted(events):
            mem += delta
            top = max(top, mem)
        peak.append(top)
        idle.append(makespan - busy)
    return dict(deadlock=False, incomplete=incomplete, makespan=makespan, idle=idle, peak=peak,
                start=start, finish=finish)

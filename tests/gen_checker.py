"""Independent model of the schedule generator for the CPU tests.

Written differently from ``oracle/fpgenoracle.c`` on purpose: no instruction items, no queues --
only how many micro-batches of each (type, stage) have been scheduled.  That is enough because
the items of one type and stage are scheduled in ascending micro-batch order and become
dependency-free in that order too (the oracle's own diagnostic counts violations of this), so
"the smallest micro-batch in the reorder queue" is simply the next one, and it is in the queue iff
every count it depends on is ahead of it.  Pure Python, small cases only.
"""
from __future__ import annotations

F, B, W = 0, 1, 2
KIND = {F: 1, B: 2, W: 3}


def simulate(problem, policy, inflight, reading="no-idle"):
    """policy[D][8], inflight[S] -> (lists[d] = [(kind, chunk, mb)], steps, stuck).

    reading: how an interval position behaves when the stage it stands on has nothing eligible.
      "no-idle"  (the oracle's): the position moves on, in the traversal direction, to the next stage
                 with an eligible item; the type is skipped only if no stage has one.
      "strict":  the position moves only after `interval` items (or when every item of the type on that
                 stage is scheduled); while the stage has nothing eligible the type yields nothing and
                 the next type is tried.
      "literal": Algorithm 1 as printed: the position moves only after `interval` items, and whatever
                 the fetch at the position yields is returned -- a type whose reorder queue is not empty
                 ends the step function, with an item or without, and later types are not tried.
    The last two exist to show what they lead to (tests/test_genoracle.py); nothing else uses them."""
    D, S, m = problem.n_devices, problem.n_stages, problem.n_microbatches
    dev = [int(x) for x in problem.stage_device]
    preds = {s: [] for s in range(S)}
    succs = {s: [] for s in range(S)}
    for a, b in zip(problem.edge_src, problem.edge_dst):
        preds[int(b)].append(int(a))
        succs[int(a)].append(int(b))
    stages = [[s for s in range(S) if dev[s] == d] for d in range(D)]
    chunk = {s: stages[dev[s]].index(s) for s in range(S)}
    types = [F, B, W] if problem.has_w else [F, B]
    done = {t: [0] * S for t in (F, B, W)}
    turn = [[F, 0] for _ in range(D)]
    pos = [{t: (0 if (policy[d][3] if t == F else policy[d][5] if t == B else 0) == 0 else len(stages[d]) - 1)
            for t in (F, B, W)} for d in range(D)]
    stepped = [{t: 0 for t in (F, B, W)} for _ in range(D)]
    lists = [[] for _ in range(D)]
    total = len(types) * S * m
    n_done, steps = 0, 0

    def ahead(t, s, snap):
        """micro-batches of (t, s) whose dependencies are resolved"""
        if t == F:
            return min([snap[F][p] for p in preds[s]] + [m])
        if t == B:
            return min([snap[F][s]] + [snap[B][q] for q in succs[s]])
        return snap[B][s]

    while n_done < total:
        snap = {t: list(done[t]) for t in (F, B, W)}
        picks = []
        for d in range(D):
            cttp = policy[d][0]
            order = [B, F] if cttp == 0 else [F, B] if cttp == 1 else [turn[d][0], B if turn[d][0] == F else F]
            if problem.has_w:
                order = order + [W]
            pick = None
            for t in order:
                ready = {s: ahead(t, s, snap) > snap[t][s] for s in stages[d]}
                if not any(ready.values()):
                    continue
                ok = {s: ready[s] and (t != F or snap[F][s] - snap[B][s] < inflight[s]) for s in stages[d]}
                direction = policy[d][3] if t == F else policy[d][5] if t == B else 0
                interval = policy[d][4] if t == F else policy[d][6] if t == B else 0
                n = len(stages[d])
                if interval > 0 and reading != "no-idle":
                    p = pos[d][t]
                    step = 1 if direction == 0 else -1
                    if stepped[d][t] == interval or (reading == "strict" and snap[t][stages[d][p]] == m):
                        for _ in range(n):   # on to the next stage that still has items of the type
                            p = (p + step) % n
                            if snap[t][stages[d][p]] < m:
                                break
                        pos[d][t], stepped[d][t] = p, 0
                    if ok[stages[d][p]]:
                        stepped[d][t] += 1
                        pick = (t, stages[d][p])
                    elif reading == "literal":
                        break                 # return whatever the fetch gave: a nop
                elif interval > 0:
                    p = pos[d][t]
                    if not any(ok.values()):
                        continue
                    if stepped[d][t] == interval or not ok[stages[d][p]]:
                        for _ in range(n):
                            p = (p + 1) % n if direction == 0 else (p - 1) % n
                            if ok[stages[d][p]]:
                                break
                        pos[d][t], stepped[d][t] = p, 0
                    stepped[d][t] += 1
                    pick = (t, stages[d][p])
                else:
                    seq = stages[d] if direction == 0 else stages[d][::-1]
                    for s in seq:
                        if ok[s]:
                            pick = (t, s)
                            break
                if pick:
                    break
            picks.append(pick)
        if not any(picks):
            return lists, steps, True
        steps += 1
        for d, pick in enumerate(picks):
            if not pick:
                continue
            t, s = pick
            lists[d].append((KIND[t], chunk[s], done[t][s]))
            done[t][s] += 1
            n_done += 1
            if policy[d][0] == 2 and t == turn[d][0]:
                turn[d][1] += 1
                if turn[d][1] >= (policy[d][1] if t == F else policy[d][2]):
                    turn[d] = [B if t == F else F, 0]
    return lists, steps, False

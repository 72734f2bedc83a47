"""Small pure-Python input builders for the CPU tests (no timing arithmetic)."""
from __future__ import annotations

import numpy as np

from workloads.problem import B, F, FD, L, O, R, W, make_problem, pack_lists


def two_tower_problem(m=4, has_w=1, comm=1, mem_cap=None):
    """Tiny non-chain DAG: stages 0->1 and 2->3 merge into 4->5; one stage per device."""
    edges = [(0, 1, comm), (1, 4, comm), (2, 3, comm), (3, 4, comm), (4, 5, comm)]
    dur = {F: [3, 3, 2, 2, 4, 4], B: [6, 6, 4, 4, 8, 8], W: [3, 3, 2, 2, 4, 4],
           FD: [3, 3, 2, 2, 4, 4], R: [3, 3, 2, 2, 4, 4], O: 5, L: 5}
    if not has_w:
        dur.pop(W)
    return make_problem(6, 6, m, has_w, list(range(6)), edges, dur, mem_cap=mem_cap,
                        name="two_tower_tiny")


def dag_problem(edges, n_stages, stage_device, n_devices, m=4, has_w=1, mem_cap=None, seed=0):
    """Any stage DAG with seeded heterogeneous durations / latencies."""
    rng = np.random.default_rng(seed)
    S = n_stages
    f = rng.integers(1, 9, S)
    dur = {F: f, FD: f, R: rng.integers(1, 9, S), B: rng.integers(1, 15, S), O: rng.integers(1, 6, S),
           L: rng.integers(1, 6, S)}
    if has_w:
        dur[W] = rng.integers(0, 7, S)
    e = [(a, b, int(rng.integers(0, 5))) for a, b in edges]
    return make_problem(n_devices, S, m, has_w, stage_device, e, dur, mem_units=rng.integers(1, 4, S),
                        mem_cap=mem_cap, name="dag")


def random_valid_lists(problem, rng, p_recompute=0.0, p_offload=0.0):
    """A random deadlock-free candidate: repeatedly append, to its device's list,
    one op drawn uniformly from the ops whose prerequisites are already listed."""
    S, m = problem.n_stages, problem.n_microbatches
    dev = [int(x) for x in problem.stage_device]
    chunk = [int(x) for x in problem.stage_chunk()]
    preds = {s: [] for s in range(S)}
    succs = {s: [] for s in range(S)}
    for a, b in zip(problem.edge_src, problem.edge_dst):
        preds[int(b)].append(int(a))
        succs[int(a)].append(int(b))
    recompute = rng.random((S, m)) < p_recompute
    offload = rng.random((S, m)) < p_offload
    # per (s, j): the remaining chain of kinds it still has to go through
    chains = {}
    for s in range(S):
        for j in range(m):
            ch = [FD, R] if recompute[s, j] else [F]
            if offload[s, j]:
                ch += [O, L]
            ch.append(B)
            if problem.has_w:
                ch.append(W)
            chains[(s, j)] = ch
    fwd_done = np.zeros((S, m), bool)
    bwd_done = np.zeros((S, m), bool)
    lists = [[] for _ in range(problem.n_devices)]
    remaining = sum(len(c) for c in chains.values())
    while remaining:
        ready = []
        for (s, j), ch in chains.items():
            if not ch:
                continue
            k = ch[0]
            if k in (F, FD) and not all(fwd_done[sp, j] for sp in preds[s]):
                continue
            if k == B and not all(bwd_done[sn, j] for sn in succs[s]):
                continue
            ready.append((s, j))
        s, j = ready[rng.integers(len(ready))]
        k = chains[(s, j)].pop(0)
        if k in (F, FD):
            fwd_done[s, j] = True
        if k == B:
            bwd_done[s, j] = True
        lists[dev[s]].append((k, chunk[s], j))
        remaining -= 1
    return lists


def perturb(lists, rng, n_swaps=1):
    """Swap random positions inside random device lists (may or may not deadlock)."""
    out = [list(x) for x in lists]
    for _ in range(n_swaps):
        d = int(rng.integers(len(out)))
        if len(out[d]) < 2:
            continue
        a, b = rng.integers(len(out[d]), size=2)
        out[d][a], out[d][b] = out[d][b], out[d][a]
    return out


def batch_from_lists(list_of_lists, stride=None):
    longest = max(len(x) for lists in list_of_lists for x in lists)
    if stride is None:
        stride = max(8, -(-(longest + 1) // 8) * 8)
    return np.stack([pack_lists(lists, stride) for lists in list_of_lists])


def random_sync_lists(problem, group, pairs, rng, p_recompute=0.0, p_offload=0.0):
    """A random deadlock-free candidate of a problem with synchronisation stages (``group[S]``
    micro-batches per item) and dependency pairs: one op at a time, drawn from the ops all of whose
    prerequisites (stage DAG and pairs, over the overlapping items) are already listed.  Returns None
    if the pairs leave nothing to draw before everything is listed (a cyclic set of pairs)."""
    S, m = problem.n_stages, problem.n_microbatches
    group = [int(x) for x in group]
    n_items = [-(-m // n) for n in group]
    dev = [int(x) for x in problem.stage_device]
    chunk = [int(x) for x in problem.stage_chunk()]
    cls = {F: "f", FD: "f", B: "b", W: "w"}
    waits = {}
    for a, b in zip(problem.edge_src, problem.edge_dst):
        for kind in (F, FD):
            waits.setdefault((kind, int(b)), []).append(("f", int(a)))
        waits.setdefault((B, int(a)), []).append(("b", int(b)))
    for k1, s1, k2, s2, _lat in pairs:
        for kind in ((F, FD) if int(k2) == F else (int(k2),)):
            waits.setdefault((kind, int(s2)), []).append((cls[int(k1)], int(s1)))
    chains = {}
    for s in range(S):
        for g in range(n_items[s]):
            ch = [FD, R] if rng.random() < p_recompute else [F]
            if rng.random() < p_offload:
                ch += [O, L]
            ch.append(B)
            if problem.has_w:
                ch.append(W)
            chains[(s, g)] = ch
    listed = set()
    lists = [[] for _ in range(problem.n_devices)]
    remaining = sum(len(c) for c in chains.values())
    while remaining:
        ready = []
        for (s, g), ch in chains.items():
            if not ch:
                continue
            lo, hi = g * group[s], min(m, (g + 1) * group[s]) - 1
            if all((c, a, ga) in listed for c, a in waits.get((ch[0], s), [])
                   for ga in range(lo // group[a], hi // group[a] + 1)):
                ready.append((s, g))
        if not ready:
            return None
        s, g = ready[rng.integers(len(ready))]
        k = chains[(s, g)].pop(0)
        if k in cls:
            listed.add((cls[k], s, g))
        lists[dev[s]].append((k, chunk[s], g))
        remaining -= 1
    return lists


def random_sync_problem(rng, trial):
    """Random chain or DAG, one to three stages per device, random group sizes and pairs."""
    D = int(rng.integers(2, 6))
    S = int(rng.integers(D, min(3 * D, 10) + 1))
    m = int(rng.integers(2, 9))
    has_w = int(rng.integers(2))
    stage_device = list(rng.permutation(D)) + [int(rng.integers(D)) for _ in range(S - D)]
    while max(np.bincount(stage_device)) > 4:
        stage_device = list(rng.permutation(D)) + [int(rng.integers(D)) for _ in range(S - D)]
    order = rng.permutation(S)                     # a random topological order of the stages
    edges = []
    for i in range(1, S):
        for a in rng.choice(order[:i], size=min(i, int(rng.integers(1, 3))), replace=False):
            edges.append((int(a), int(order[i]), int(rng.integers(0, 4))))
    dur = {k: rng.integers(0 if k != B else 1, 9, S) for k in (F, B, R, O, L)}
    dur[FD] = dur[F]
    if has_w:
        dur[W] = rng.integers(0, 6, S)
    prob = make_problem(D, S, m, has_w, stage_device, edges, dur, mem_units=rng.integers(0, 3, S),
                        mem_cap=rng.integers(m, 4 * m, D))
    group = [int(rng.choice([1, 1, 2, 3, m])) for _ in range(S)]
    pos = {int(s): i for i, s in enumerate(order)}
    pairs = []
    for _ in range(int(rng.integers(0, 4))):
        a, b = (int(x) for x in rng.choice(S, 2, replace=False))
        if pos[a] > pos[b]:
            a, b = b, a
        kinds = [(F, F), (F, B), (B, W) if has_w else (F, B), (W, W) if has_w else (B, B), (F, R), (B, L)]
        k1, k2 = kinds[int(rng.integers(len(kinds)))]
        if k1 == B and k2 in (B, W):               # backward-to-backward pairs run down the order
            a, b = b, a
        pairs.append((k1, a, k2, b, int(rng.integers(0, 4))))
    return prob, group, pairs


def random_slot_sync_problem(rng):
    """A problem with synchronisation stages and pairs of the kind the slot kernel has a form for: a stage DAG
    with at most two inputs and outputs per stage, pairs that run forward-to-forward or backward-to-backward
    (and keep those bounds), groups of micro-batches only on stages all of whose neighbours have one item per
    micro-batch."""
    D = int(rng.integers(2, 7))
    S = int(rng.integers(D, min(3 * D, 11) + 1))
    m = int(rng.integers(2, 10))
    has_w = int(rng.integers(2))
    stage_device = [int(x) for x in rng.permutation(D)] + [int(rng.integers(D)) for _ in range(S - D)]
    while max(np.bincount(stage_device)) > 4:
        stage_device = [int(x) for x in rng.permutation(D)] + [int(rng.integers(D)) for _ in range(S - D)]
    # edges a -> b with a < b, in- and out-degree at most two
    fin, fout, bin_, bout = [0] * S, [0] * S, [0] * S, [0] * S   # degrees per direction
    edges, nbr = [], [set() for _ in range(S)]
    for b in range(int(rng.integers(1, min(3, S) + 1)), S):
        cands = [a for a in range(b) if fout[a] < 2]
        for a in rng.choice(cands, size=min(len(cands), int(rng.integers(1, 3))), replace=False) if cands else []:
            a = int(a)
            edges.append((a, b, int(rng.integers(0, 4))))
            fout[a] += 1; fin[b] += 1; bin_[a] += 1; bout[b] += 1
            nbr[a].add(b); nbr[b].add(a)
    pairs = []
    for _ in range(int(rng.integers(0, 4))):
        a, b = sorted(int(x) for x in rng.choice(S, 2, replace=False))
        if rng.random() < 0.5:
            if fout[a] < 2 and fin[b] < 2:                 # forward of a before forward of b
                pairs.append((F, a, F, b, int(rng.integers(0, 4))))
                fout[a] += 1; fin[b] += 1
                nbr[a].add(b); nbr[b].add(a)
        elif bout[b] < 2 and bin_[a] < 2:                  # backward of b before backward of a
            pairs.append((B, b, B, a, int(rng.integers(0, 4))))
            bout[b] += 1; bin_[a] += 1
            nbr[a].add(b); nbr[b].add(a)
    group = [1] * S
    for s in rng.permutation(S):
        s = int(s)
        if rng.random() < 0.4 and all(group[t] == 1 for t in nbr[s]):
            group[s] = int(rng.choice([2, 3, m]))
    dur = {k: rng.integers(0 if k != B else 1, 9, S) for k in (F, B, R, O, L)}
    dur[FD] = dur[F]
    if has_w:
        dur[W] = rng.integers(0, 6, S)
    prob = make_problem(D, S, m, has_w, stage_device, edges, dur, mem_units=rng.integers(0, 3, S),
                        mem_cap=rng.integers(m, 4 * m, D))
    return prob, group, pairs

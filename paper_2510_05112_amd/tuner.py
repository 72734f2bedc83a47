"""The tuner's grid of schedule types (paper Section 6) as parameter sets for ``Problem.generate``.

Host-side glue only: it enumerates schedule types -- (stage placement strategy, forward and
backward stage traversal priority, computation type traversal priority) -- under the rules the
paper states for its grid search, and hands them to the library, whose kernels generate, time
and rank the schedules.  No scheduling or timing arithmetic happens here.

Rules taken from Section 6: the parameter values come from the table of built-in values; an
interval is tried only together with the circular placement; forward-first type priority is
left out unless the user asks for it; unit1 = unit2 = 1.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


CTTP_BWD_FIRST, CTTP_FWD_FIRST, CTTP_INTERLEAVED = 0, 1, 2
BREADTH_FIRST, DEPTH_FIRST = 0, 1
NO_LIMIT = 2**31 - 1
_CTTP_NAMES = {CTTP_BWD_FIRST: "bwdpass-first", CTTP_FWD_FIRST: "fwdpass-first", CTTP_INTERLEAVED: "interleaved"}
_DIR_NAMES = {BREADTH_FIRST: "breadth-first", DEPTH_FIRST: "depth-first"}


def placement(strategy: str, n_devices: int, n_stages: int) -> list[int]:
    """Stage -> device for the built-in placement strategies of a chain of stages (Section 4.1,
    Section 2.1): one-to-one, circular (stage s on device s mod p), V-shape (the second half of
    the stages walks the devices back).  The bidirectional strategy shares stages between actors
    and is not expressible as one stage -> device map."""
    p, S = n_devices, n_stages
    if strategy == "one-to-one":
        if S != p:
            raise ValueError("one-to-one needs as many stages as devices")
        return list(range(p))
    if strategy == "circular":
        return [s % p for s in range(S)]
    if strategy == "v-shape":
        return [(s % p) if (s // p) % 2 == 0 else (p - 1 - s % p) for s in range(S)]
    raise ValueError(f"unknown placement strategy {strategy!r}")


def bidirectional(n_devices: int, v_shape: bool = False):
    """The bidirectional placement strategy (Section 4.1's built-in strategies; Section 2.1): two
    replicas of a chain of stages, one laid down the devices and one up, each taking half of the
    micro-batches, so that every device holds early and late stages.  In the scheduler's terms
    that is a stage DAG of two separate chains; micro-batch j of the problem stands for the j-th
    micro-batch of either replica.  v_shape: every replica is itself a V-shape chain of 2p stages
    (the combination Section 7.1 also searches), four stages per device.  Returns
    (stage_device, edges [(src, dst)], replica_stage: the model stage each scheduler stage is a
    copy of, for the caller's cost tables)."""
    p = n_devices
    down = list(range(p)) + (list(range(p - 1, -1, -1)) if v_shape else [])
    n = len(down)                                  # stages per replica
    stage_device = down + [p - 1 - d for d in down]
    edges = [(s, s + 1) for s in range(n - 1)] + [(n + s, n + s + 1) for s in range(n - 1)]
    return stage_device, edges, list(range(n)) * 2


@dataclass
class ScheduleType:
    cttp: int
    f_dir: int
    f_interval: int
    b_dir: int
    b_interval: int

    def label(self) -> str:
        def stp(d, n):
            return _DIR_NAMES[d] if not n else f"({_DIR_NAMES[d]}, {n})"
        return f"cttp={_CTTP_NAMES[self.cttp]} fstp={stp(self.f_dir, self.f_interval)} bstp={stp(self.b_dir, self.b_interval)}"

    def policy_row(self) -> list[int]:
        return [self.cttp, 1, 1, self.f_dir, self.f_interval, self.b_dir, self.b_interval, 0]


def schedule_types(n_devices: int, circular: bool, forward_first: bool = False) -> list[ScheduleType]:
    """The schedule types of the grid for one placement.  `circular`: the placement puts several
    stages on an actor in circular order, the only case in which an interval (= the number of
    devices, the group size of the interleaved schedules) is tried."""
    cttps = [CTTP_BWD_FIRST, CTTP_INTERLEAVED] + ([CTTP_FWD_FIRST] if forward_first else [])
    intervals = [0, n_devices] if circular else [0]
    return [ScheduleType(c, fd, fi, bd, bi)
            for c in cttps for fd in (BREADTH_FIRST, DEPTH_FIRST) for fi in intervals
            for bd in (BREADTH_FIRST, DEPTH_FIRST) for bi in intervals]


def grid(problem, circular: bool, inflight_options=None, forward_first: bool = False):
    """Parameter sets of the grid for one problem (= one placement): every schedule type, the same
    for all actors, times every in-flight option.  inflight_options: list of int32 [S] arrays
    (default: no limit, and the 1F1B-like limit ceil((p - d) / v) per stage).
    Returns (labels, policy int32 [n][D][8], inflight int32 [n][S])."""
    D, S = int(problem.n_devices), int(problem.n_stages)
    dev = np.asarray(problem.stage_device, np.int64)
    if inflight_options is None:
        v = max(1, int(np.bincount(dev, minlength=D).max()))
        inflight_options = [np.full(S, NO_LIMIT, np.int32), (-(-(D - dev) // v)).astype(np.int32)]
    types = schedule_types(D, circular, forward_first)
    labels, pol, inf = [], [], []
    for t in types:
        for i, limit in enumerate(inflight_options):
            labels.append(f"{t.label()} inflight#{i}")
            pol.append([t.policy_row()] * D)
            inf.append(np.asarray(limit, np.int32))
    return labels, np.asarray(pol, np.int32), np.stack(inf).astype(np.int32)


def tune(handle, problem, circular: bool, k: int = 8, inflight_options=None, forward_first: bool = False,
         slide: bool = False, fused: bool = False):
    """Generate, time and rank the grid of one problem on the GPU.  handle: a ``Problem`` created
    with a stride of at least ``stride_for(problem)``.  slide: for problems with split backward,
    also rank every generated schedule after the weight-gradient sliding pass (Section 5.2, bubble
    optimizations); such entries have ``slid`` set.  Returns the k best feasible schedules as a list
    of dicts (label, makespan, index into the grid, slid).  The schedules are timed with whatever cost
    model the handle is set to (``set_microbatch_costs``, ``set_link_occupancy``); the sliding pass
    follows the link switch and refuses costs per micro-batch.  fused: one kernel generates and times the
    schedules (plain cost model; ``Problem.generate_evaluate``, with ``slide`` a second launch that has the
    sliding pass in it) and only the winners' rows are written: the entries then carry them as ``ops``
    (uint16 [D][stride]; the slid list for entries with ``slid`` set)."""
    import torch

    labels, pol, inf = grid(problem, circular, inflight_options, forward_first)
    n = len(labels)
    stride = stride_for(problem)
    if fused:
        d_pol, d_inf = torch.from_numpy(pol).cuda(), torch.from_numpy(inf).cuda()
        res, _ = handle.generate_evaluate(d_pol, d_inf)
        if slide and problem.has_w:
            slid, _ = handle.generate_evaluate(d_pol, d_inf, slide=True)
            res = {name: torch.cat([res[name], slid[name]]) for name in ("makespan", "idle", "peak", "flags")}
        top = handle.topk(res, min(k, 1024))
        torch.cuda.synchronize()
        cnt = int(top["count"].item())
        idx, ms = top["idx"].cpu().numpy()[:cnt], top["makespan"].cpu().numpy()[:cnt]
        # the winners' rows as generated, and for entries ranked after the sliding pass their slid lists
        rows = handle.generate_selected(d_pol, d_inf, torch.from_numpy(idx % n).cuda(), stride)["ops"]
        ops = rows.cpu().numpy().view(np.uint16)
        if (idx >= n).any():
            ops = np.where((idx >= n)[:, None, None], handle.wslide(rows, stride)["ops"].cpu().numpy().view(np.uint16), ops)
        return [dict(label=labels[int(i) % n] + (" +slide" if i >= n else ""), makespan=int(t), index=int(i) % n,
                     slid=bool(i >= n), ops=ops[r]) for r, (i, t) in enumerate(zip(idx, ms))]
    out = handle.generate(torch.from_numpy(pol).cuda(), torch.from_numpy(inf).cuda(), stride)
    res = handle.evaluate(out["ops"])
    if slide and problem.has_w:
        # only the results of the slid lists are ranked: the one-kernel form, which writes no list
        slid = handle.wslide_evaluate(out["ops"])
        res = {name: torch.cat([res[name], slid[name]]) for name in ("makespan", "idle", "peak", "flags")}
    top = handle.topk(res, min(k, 1024))
    torch.cuda.synchronize()
    cnt = int(top["count"].item())
    idx, ms = top["idx"].cpu().numpy()[:cnt], top["makespan"].cpu().numpy()[:cnt]
    return [dict(label=labels[int(i) % n] + (" +slide" if i >= n else ""), makespan=int(t), index=int(i) % n,
                 slid=bool(i >= n)) for i, t in zip(idx, ms)]


# ---- shared stages: the weight-gradient synchronisation of the bidirectional placement ----------------

def shared_stage_sync(problem, replica_stage, sync_cost):
    """A placement that holds every model stage on two actors (the bidirectional strategy, Section 4.1: a
    stage shared among actors) trains ONE model only if the holders of a stage add up their weight
    gradients before the optimizer step: where the scheduler meets a shared stage it inserts a
    synchronisation instruction.  In the library's terms (``Problem.set_sync``) that is, per holder of a
    shared model stage, a synchronisation stage on the holder's device with ONE item for all micro-batches
    (group m) whose forward item is the exchange (cost ``sync_cost[model stage]``; its backward and
    weight-gradient items cost nothing), and dependency pairs that let it start only when the last
    gradient-producing items (W, or B without split backward) of EVERY holder of that model stage have
    finished.  replica_stage[s]: the model stage that scheduler stage s is a copy of (``bidirectional``'s
    third result).  Returns (problem with the synchronisation stages appended, group, pairs); the first
    stages, their chunk numbers and so every op word of the original problem stay valid."""
    from types import SimpleNamespace
    S, D, m = int(problem.n_stages), int(problem.n_devices), int(problem.n_microbatches)
    dev = [int(x) for x in problem.stage_device]
    holders = {}
    for s, model_stage in enumerate(replica_stage):
        holders.setdefault(int(model_stage), []).append(s)
    shared = {ms: hs for ms, hs in holders.items() if len(hs) > 1}
    last = 3 if problem.has_w else 2          # the kind whose items produce the weight gradients
    new_dev, pairs = [], []
    dur = np.asarray(problem.dur, np.int32).reshape(8, S)
    extra = np.zeros((8, sum(len(hs) for hs in shared.values())), np.int32)
    for ms in sorted(shared):
        for s in shared[ms]:
            q = S + len(new_dev)
            extra[1, len(new_dev)] = extra[7, len(new_dev)] = extra[4, len(new_dev)] = int(sync_cost[ms])
            new_dev.append(dev[s])
            pairs += [(last, other, 1, q, 0) for other in shared[ms]]
    if max(np.bincount(dev + new_dev, minlength=D)) > 4:
        raise ValueError("more than four stages on a device")
    out = SimpleNamespace(
        n_devices=D, n_stages=S + len(new_dev), n_microbatches=m, has_w=int(problem.has_w),
        stage_device=np.asarray(dev + new_dev, np.int32), edge_src=np.asarray(problem.edge_src, np.int32),
        edge_dst=np.asarray(problem.edge_dst, np.int32), edge_comm=np.asarray(problem.edge_comm, np.int32),
        dur=np.concatenate([dur, extra], axis=1),
        mem_units=np.concatenate([np.asarray(problem.mem_units, np.int32), np.zeros(len(new_dev), np.int32)]),
        mem_cap=np.asarray(problem.mem_cap, np.int32), name=getattr(problem, "name", "") + "+grad-sync")
    group = np.asarray([1] * S + [m] * len(new_dev), np.int32)
    return out, group, np.asarray(pairs, np.int32).reshape(-1, 5)


def append_sync_items(ops, problem, shared_problem):
    """ops: CUDA int16 tensor [n][D][stride] of schedules for `problem`, END-padded in full (what
    ``Problem.generate`` writes).  Appends, at the end of every device's list, the items of the
    synchronisation stages that ``shared_stage_sync`` put on that device (forward, backward and, with split
    backward, weight gradient of item 0, stage by stage).  Returns a new tensor whose stride has room."""
    import torch
    S = int(problem.n_stages)
    dev = np.asarray(shared_problem.stage_device)
    D = int(problem.n_devices)
    kinds = (1, 2, 3) if problem.has_w else (1, 2)
    tails = []
    for d in range(D):
        on_d = [s for s in range(int(shared_problem.n_stages)) if dev[s] == d]
        tails.append([(k << 13) | (on_d.index(q) << 11) for q in on_d if q >= S for k in kinds])
    width = max(len(t) for t in tails)
    n, _, stride = ops.shape
    new_stride = -(-(stride + width) // 8) * 8
    out = torch.zeros((n, D, new_stride), dtype=ops.dtype, device=ops.device)
    out[:, :, :stride] = ops
    length = (ops != 0).sum(dim=2)                                   # [n][D]: items listed per device
    for d in range(D):
        for i, word in enumerate(tails[d]):
            signed = word - 65536 if word >= 32768 and ops.dtype == torch.int16 else word
            out[:, d, :].scatter_(1, (length[:, d] + i).unsqueeze(1), torch.full((n, 1), signed, dtype=ops.dtype, device=ops.device))
    return out


def tune_shared(gen_handle, sync_handle, problem, shared_problem, k: int = 8, inflight_options=None,
                forward_first: bool = False):
    """``tune`` for a placement with shared stages: the schedules are generated for `problem` (two separate
    chains, ``gen_handle``), the inserted synchronisation items are appended, and the lists are timed and
    ranked under the synchronisation model (``sync_handle``: a handle of ``shared_problem`` on which
    ``set_sync`` was called with ``shared_stage_sync``'s group and pairs).  Returns the k best as ``tune``
    does."""
    import torch
    labels, pol, inf = grid(problem, False, inflight_options, forward_first)
    out = gen_handle.generate(torch.from_numpy(pol).cuda(), torch.from_numpy(inf).cuda(), stride_for(problem))
    ops = append_sync_items(out["ops"], problem, shared_problem)
    res = sync_handle.evaluate(ops)
    top = sync_handle.topk(res, min(k, 1024))
    torch.cuda.synchronize()
    cnt = int(top["count"].item())
    idx, ms = top["idx"].cpu().numpy()[:cnt], top["makespan"].cpu().numpy()[:cnt]
    return [dict(label=labels[int(i)], makespan=int(t), index=int(i), slid=False) for i, t in zip(idx, ms)]


def stride_for(problem) -> int:
    """Row stride (words, multiple of 8) that holds the longest list the generator can emit."""
    per_dev = int(np.bincount(np.asarray(problem.stage_device), minlength=int(problem.n_devices)).max())
    longest = per_dev * int(problem.n_microbatches) * (3 if problem.has_w else 2)
    return max(8, -(-longest // 8) * 8)

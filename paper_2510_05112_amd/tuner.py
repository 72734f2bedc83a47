"""The tuner's grid (paper Section 6) as parameter sets for ``Problem.generate``, and the outer loop
over pipeline depth, data-parallel width and micro-batch size around it (``tune_parallel``).

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
         slide: bool = False):
    """Generate, time and rank the grid of one problem on the GPU.  handle: a ``Problem`` created
    with a stride of at least ``stride_for(problem)``.  slide: for problems with split backward,
    also rank every generated schedule after the weight-gradient sliding pass (Section 5.2, bubble
    optimizations); such entries have ``slid`` set.  Returns the k best feasible schedules as a list
    of dicts (label, makespan, index into the grid, slid).  The schedules are timed with whatever cost
    model the handle is set to (``set_microbatch_costs``, ``set_link_occupancy``); the sliding pass
    follows the link switch and refuses costs per micro-batch."""
    import torch

    labels, pol, inf = grid(problem, circular, inflight_options, forward_first)
    n = len(labels)
    stride = stride_for(problem)
    out = handle.generate(torch.from_numpy(pol).cuda(), torch.from_numpy(inf).cuda(), stride)
    res = handle.evaluate(out["ops"])
    if slide and problem.has_w:
        slid = handle.wslide(out["ops"], stride)
        res = {name: torch.cat([res[name], slid[name]]) for name in ("makespan", "idle", "peak", "flags")}
    top = handle.topk(res, min(k, 1024))
    torch.cuda.synchronize()
    cnt = int(top["count"].item())
    idx, ms = top["idx"].cpu().numpy()[:cnt], top["makespan"].cpu().numpy()[:cnt]
    return [dict(label=labels[int(i) % n] + (" +slide" if i >= n else ""), makespan=int(t), index=int(i) % n,
                 slid=bool(i >= n)) for i, t in zip(idx, ms)]


# ---- the outer dimensions of the grid: pipeline depth, data-parallel width, micro-batch size ----------

@dataclass
class ProblemDesc:
    """The fields of ``fpsched_problem_desc`` (what ``Problem`` takes)."""
    n_devices: int
    n_stages: int
    n_microbatches: int
    has_w: int
    stage_device: np.ndarray
    edge_src: np.ndarray
    edge_dst: np.ndarray
    edge_comm: np.ndarray
    dur: np.ndarray          # int32 [8][S]
    mem_units: np.ndarray
    mem_cap: np.ndarray
    name: str = ""


def parallel_grid(n_gpus: int, n_layers: int, global_batch: int, pp_options=None, mbs_options=None,
                  max_microbatches: int = 2048):
    """The (pp, dp, mbs) part of the tuner's parameter space (Section 6): every pipeline depth pp that
    divides the number of GPUs and does not exceed the number of layers, dp = n_gpus / pp, and every
    micro-batch size mbs that divides the per-replica batch global_batch / dp; the number of
    micro-batches of an iteration is then m = global_batch / (dp mbs).  Returns [(pp, dp, mbs, m)]."""
    out = []
    for pp in (pp_options or range(1, n_gpus + 1)):
        if n_gpus % pp or pp > n_layers:
            continue
        dp = n_gpus // pp
        if global_batch % dp:
            continue
        per_replica = global_batch // dp
        for mbs in (mbs_options or range(1, per_replica + 1)):
            if per_replica % mbs == 0 and per_replica // mbs <= max_microbatches:
                out.append((pp, dp, mbs, per_replica // mbs))
    return out


def split_layers(n_layers: int, n_stages: int) -> list[int]:
    """Layers per stage of an even split; the first n_layers mod n_stages stages take one more."""
    base, extra = divmod(n_layers, n_stages)
    return [base + (1 if s < extra else 0) for s in range(n_stages)]


def chain_problem_from_layers(pp: int, stages_per_device: int, m: int, strategy: str, layer_cost, mbs: int,
                              comm: int, layer_mem_units: int, mem_cap: int, n_layers: int, has_w: bool = True):
    """One problem of the outer grid: a chain of pp * stages_per_device stages placed by `strategy`.
    The cost of a stage is the sum of the costs of its layers (the estimator sketched after Section 6);
    layer_cost(mbs) -> (forward, backward, weight-gradient) integer cost of ONE layer for a micro-batch of
    mbs samples (with has_w false the backward cost stands for both parts).  A stage holds
    layer_mem_units * mbs activation units per layer and micro-batch."""
    S = pp * stages_per_device
    layers = np.asarray(split_layers(n_layers, S), np.int64)
    f, b, w = (int(x) for x in layer_cost(mbs))
    dur = np.zeros((8, S), np.int32)
    dur[1] = dur[7] = dur[4] = layers * f      # forward, discarding forward, recomputation
    dur[2] = layers * b
    if has_w:
        dur[3] = layers * w
    src = np.arange(S - 1, dtype=np.int32)
    return ProblemDesc(pp, S, m, int(has_w), np.asarray(placement(strategy, pp, S), np.int32), src, src + 1,
                       np.full(S - 1, comm, np.int32), dur, (layers * layer_mem_units * mbs).astype(np.int32),
                       np.full(pp, mem_cap, np.int32), name=f"{strategy} pp={pp} mbs={mbs}")


def tune_parallel(n_gpus: int, n_layers: int, global_batch: int, layer_cost, comm: int = 1, layer_mem_units: int = 1,
                  mem_cap: int = NO_LIMIT, strategies=("one-to-one", "circular"), stages_per_device: int = 2,
                  has_w: bool = True, k: int = 1, device: int = 0, pp_options=None, mbs_options=None,
                  slide: bool = False):
    """The whole grid search of Section 6 on the GPU: for every (pp, dp, mbs) of `parallel_grid` and every
    placement strategy, build the problem (`chain_problem_from_layers`; one-to-one has one stage per
    device, the others `stages_per_device`), generate and time its schedule types (`tune`) and keep the k
    best of each; the result is sorted by makespan, which is the time of one iteration of a replica in
    the units of layer_cost.  Configurations whose every schedule exceeds the memory cap give no entry.
    Returns a list of dicts (pp, dp, mbs, microbatches, placement, label, makespan, slid)."""
    from .binding import Problem
    found = []
    for pp, dp, mbs, m in parallel_grid(n_gpus, n_layers, global_batch, pp_options, mbs_options):
        for strategy in strategies:
            v = 1 if strategy == "one-to-one" else stages_per_device
            if pp * v > n_layers or (strategy != "one-to-one" and (v < 2 or pp < 2)):
                continue
            prob = chain_problem_from_layers(pp, v, m, strategy, layer_cost, mbs, comm, layer_mem_units, mem_cap,
                                             n_layers, has_w)
            handle = Problem(prob, stride_for(prob), device=device)
            try:
                for best in tune(handle, prob, strategy == "circular", k=k, slide=slide):
                    found.append(dict(pp=pp, dp=dp, mbs=mbs, microbatches=m, placement=strategy, label=best["label"],
                                      makespan=best["makespan"], slid=best["slid"]))
            finally:
                handle.close()
    found.sort(key=lambda e: e["makespan"])   # stable: ties keep the order of the enumeration
    return found


def stride_for(problem) -> int:
    """Row stride (words, multiple of 8) that holds the longest list the generator can emit."""
    per_dev = int(np.bincount(np.asarray(problem.stage_device), minlength=int(problem.n_devices)).max())
    longest = per_dev * int(problem.n_microbatches) * (3 if problem.has_w else 2)
    return max(8, -(-longest // 8) * 8)

/*
 * fpsched.h -- C ABI of the MI355X (gfx950) batched pipeline-schedule evaluator.
 *
 * The library scores candidate pipeline-parallel schedules the way the paper's
 * auto-tuner needs them scored (Section 3: the offline tuner picks the most
 * suitable of the enumerated schedules; Section 7.1: the winners are those whose
 * bubble ratio is lowest): for every candidate it propagates dependencies
 * to get each op's start and finish time, then reports makespan, per-device
 * idle (bubble) time, per-device peak activation memory and a deadlock flag,
 * and reduces a batch to its k best candidates under the memory cap.  It also
 * runs the paper's scheduler itself (Section 5: step function, reorder queues,
 * in-flight limits) as a generator of candidates (fpsched_generate, or fused with the
 * evaluation: fpsched_generate_evaluate), moves the
 * weight-gradient items of candidate lists into idle time (fpsched_wslide;
 * Section 5.2, bubble optimizations), and ranks evaluated candidates by other
 * keys than the makespan (fpsched_rank, fpsched_pareto, fpsched_apply_caps).
 *
 * All entry points are plain C, take plain pointers (marked HOST or DEVICE) and
 * sizes, return 0 on success or a negative FPSCHED_E* code, and never throw or
 * abort.  A problem with an individual candidate (deadlock, malformed words) is
 * never a call error: it is reported in that candidate's flags.
 *
 * Ownership and threads.  The caller owns every buffer it passes, the workspaces
 * included; the library owns only the opaque handle and the few KB of tables it
 * uploads when the handle is created (it allocates nothing afterwards, except for the tables
 * of fpsched_problem_set_microbatch_costs and fpsched_problem_set_link_occupancy).  A handle is
 * immutable after creation except for fpsched_problem_select_kernel and those two calls: calls on
 * distinct handles, and calls on one handle that use distinct workspaces and
 * output buffers, may run from different host threads and on different streams.
 * Device calls only enqueue kernels on the given stream and return.
 *
 * Environment variables, read when the call they belong to runs; none changes a result:
 *   FPSCHED_SLOT_WAVES=n  (fpsched_problem_create, the two cost-model setters) at most n wavefronts
 *                         per workgroup of the main evaluation kernel, one workgroup per compute unit;
 *   FPSCHED_GEN_WAVES=n   (fpsched_generate) n resident wavefronts per compute unit, default 24;
 *   FPSCHED_MB_GLOBAL=1   (fpsched_problem_set_microbatch_costs) keep the cost table in device
 *                         memory even where it would fit LDS;
 *   FPSCHED_VERBOSE=1     the two cost-model setters print the kernel form and shape they chose.
 */
#ifndef FPSCHED_H
#define FPSCHED_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FPSCHED_VERSION 100

/* ---- op words ------------------------------------------------------------
 * A schedule is, per device, a sequence of instructions (Section 4, "FlexPipe's
 * Instructions"); an instruction item is (type, micro-batch, stage) (Section
 * 5.1, "Instruction Item").  One item = one unsigned 16-bit word:
 *     bits 15..13  kind        bits 12..11  device-local chunk      bits 10..0  micro-batch
 * The stage is the chunk-th stage (ascending stage id) placed on the device
 * whose row the word sits in.  Kinds F/B/W are the paper's FwdPass, BwdPass (or
 * CompInputGrad when the backward is split) and CompWeightGrad (Table 1); R, O,
 * L and FD model recomputation and offloading, which the paper only names.
 * Kind 0 ends a device's list: the row is read up to its first END word (or
 * the row stride); anything after it is ignored. */
enum {
  FPSCHED_END = 0, /* end of list / padding                                       */
  FPSCHED_F = 1,   /* forward; activation stays resident                          */
  FPSCHED_B = 2,   /* backward (input gradient when has_w); frees iff !has_w      */
  FPSCHED_W = 3,   /* weight gradient; frees the activation (has_w only)          */
  FPSCHED_R = 4,   /* recompute a discarded activation                            */
  FPSCHED_O = 5,   /* offload a resident activation (freed at the op's end)       */
  FPSCHED_L = 6,   /* reload an offloaded activation                              */
  FPSCHED_FD = 7,  /* forward whose activation is discarded at the op's end       */
  FPSCHED_NKINDS = 8
};
#define FPSCHED_WORD(kind, chunk, mb) ((uint16_t)(((kind) << 13) | ((chunk) << 11) | (mb)))
#define FPSCHED_MAX_DEVICES 64
#define FPSCHED_MAX_CHUNKS 4
#define FPSCHED_MAX_MICROBATCHES 2048

/* ---- per-candidate flags --------------------------------------------------- */
#define FPSCHED_FLAG_DEADLOCK 1u   /* some listed op can never issue                          */
#define FPSCHED_FLAG_INCOMPLETE 2u /* all ops issued but some (stage, micro-batch) did not
                                      finish its backward; or, together with DEADLOCK, a
                                      device is stuck at a malformed word                     */
#define FPSCHED_FLAG_OVER_CAP 4u   /* evaluated fine, but peak[d] > mem_cap[d] for some d     */
/* Candidates with DEADLOCK or INCOMPLETE get makespan = INT64_MAX, idle = -1, peak = -1. */

/* ---- error codes ----------------------------------------------------------- */
#define FPSCHED_OK 0
#define FPSCHED_EINVAL (-1)    /* bad argument (null pointer, size out of range, bad table) */
#define FPSCHED_ENOMEM (-2)    /* host or device allocation failed / workspace too small    */
#define FPSCHED_EHIP (-3)      /* a HIP runtime call failed                                 */
#define FPSCHED_EOVERFLOW (-4) /* the problem's time bound does not fit the kernel's int32  */
#define FPSCHED_ENODEV (-5)    /* host-only handle used for a device call                   */
#define FPSCHED_EUNSUPPORTED (-6) /* problem too large for the on-chip tables               */
#define FPSCHED_ESCRATCH (-7)  /* batch too large for the static scratch of
                                  fpsched_evaluate_topk_static                              */

/* ---- problem description (Section 4.1 data model: Stage / StageSet = the DAG
 * of stages, Actor = device; placement per Section 2.1; costs per (kind, stage)
 * as the profiler of Section 3 delivers them; in-flight memory limit per
 * Section 4.2).  All pointers are HOST memory, read during the call only. */
typedef struct {
  int32_t n_devices;       /* D, 1..64                                                   */
  int32_t n_stages;        /* S, 1..4*D                                                  */
  int32_t n_microbatches;  /* m, 1..2048                                                 */
  int32_t has_w;           /* 0: B is the whole backward and frees; 1: B then W, W frees */
  const int32_t *stage_device; /* [S] device of each stage; at most 4 stages per device  */
  int32_t n_edges;             /* edges of the stage DAG (a chain has S-1)               */
  const int32_t *edge_src;     /* [E]                                                    */
  const int32_t *edge_dst;     /* [E]                                                    */
  const int32_t *edge_comm;    /* [E] >= 0; latency added iff the two stages sit on
                                  different devices; same for activations and gradients  */
  const int32_t *dur;          /* [FPSCHED_NKINDS][S] >= 0; row 0 unused                 */
  const int32_t *mem_units;    /* [S] >= 0, activation size of one (stage, micro-batch)  */
  const int32_t *mem_cap;      /* [D] >= 0, per-device cap (INT32_MAX = none)            */
} fpsched_problem_desc;

typedef struct fpsched_problem fpsched_problem; /* opaque, library-owned */

/* Validates the description (the edge list must be a DAG), precomputes the
 * lookup tables and, unless device_id < 0, uploads them to that GPU.
 * device_id < 0 gives a host-only handle: fpsched_encode / fpsched_validate
 * work, device calls return FPSCHED_ENODEV.  max_stride_words bounds the row
 * stride later passed to fpsched_evaluate (it enters the int32 time bound:
 * FPSCHED_EOVERFLOW if D * max_stride * (max dur + max comm) >= 2^31). */
int fpsched_problem_create(const fpsched_problem_desc *desc, int device_id, int32_t max_stride_words,
                           fpsched_problem **out);
void fpsched_problem_destroy(fpsched_problem *p);

/* Variant of the cost model: micro-batches of unequal size.  The paper profiles one cost per
 * (type, stage) (estimator sketch after Section 6); its related-work section (Section 8,
 * "Frameworks") names dynamic micro-batching, where the micro-batches of an iteration differ in
 * length and so in cost.  dur_mb: HOST, int32 [FPSCHED_NKINDS][S][m], >= 0 (row 0 unused), copied;
 * from then on fpsched_evaluate uses  finish = start + dur_mb[kind][stage][micro-batch]  and counts
 * those costs as the devices' busy time; nothing else changes.  NULL switches back to desc.dur.
 * Synchronous: waits for the device's queued work (the previous table may be in use) and must
 * not run concurrently with other calls on the handle.  The first call on a device handle
 * allocates two tables of device memory (FPSCHED_ENOMEM), freed by fpsched_problem_destroy.
 * FPSCHED_EINVAL for a negative value, FPSCHED_EOVERFLOW if D * max_stride * (max value + max
 * comm) >= 2^31, FPSCHED_EUNSUPPORTED if no kernel fits these values: the handle then keeps
 * what it had.  After FPSCHED_EHIP / FPSCHED_ENOMEM, and when the table cannot be combined with
 * link occupancy that is switched on, it is back on desc.dur.  While a table is set,
 * fpsched_wslide returns FPSCHED_EUNSUPPORTED (the sliding pass knows one cost per (type, stage));
 * fpsched_generate ignores costs anyway.  Works on a host-only handle (validation only). */
int fpsched_problem_set_microbatch_costs(fpsched_problem *p, const int32_t *dur_mb);

/* Variant of the cost model: links that carry one value at a time.  The paper lists P2P send and
 * receive among its instructions (Section 4, "FlexPipe's Instructions") and leaves out how they
 * overlap (end of Section 5.2); fpsched_evaluate reads a transfer as a pure latency.  With on != 0
 * every ordered pair of devices (from, to) is a link: a value (the activation of a forward item
 * for a successor stage on another device, the gradient of a backward item for a predecessor
 * stage on another device) leaves when its item has finished and the link is free, occupies the
 * link for edge_comm and arrives at its end; the values of a device leave in the order its items
 * run (two values of one item: in the order of the edge list).  A consumer is ready when all its
 * inputs have arrived; everything else is unchanged, and with latencies of zero the two models
 * coincide.  on == 0 switches back.  Only the slot kernel has this form: FPSCHED_EUNSUPPORTED if
 * the problem does not fit it (more than two inputs or outputs per stage, or
 * D * max_stride * (max dur + 2 * max comm) >= 2^24), and from fpsched_evaluate while the general
 * kernel is selected.  Together with costs per micro-batch (either call may come first; the two are
 * independent: one says what an item costs, the other when its result arrives) it needs the cost
 * table in LDS: the call that would complete the pair answers FPSCHED_EUNSUPPORTED otherwise and
 * the handle stays on the variant it had.  fpsched_wslide follows the switch (the
 * weight-gradient items send nothing, so its rule is unchanged; the times it works with are this
 * model's).
 * The first call on a device handle allocates one more table image (FPSCHED_ENOMEM); not to be
 * called concurrently with other calls on the handle.  Works on a host-only handle (flag only). */
int fpsched_problem_set_link_occupancy(fpsched_problem *p, int32_t on);

/* Synchronisation stages and dependency pairs.  The paper lets a user register a new instruction --
 * its example is the synchronisation that exchanges the output states of the submodules of a
 * multimodal model (SyncWithGather, Section 7.2) -- attached to a stage registered for it, state how
 * many of the instructions it depends on must have been scheduled before it (the comparison system
 * synchronises once every few micro-batches, Section 2.2), and add data dependencies as pairs
 * ((type1, stage_i), (type2, stage_j)): type1 of stage_i before type2 of stage_j (Section 4.2,
 * "Registration of new instructions"; Section 5.1, "Data dependency").  In this library:
 *   - group: HOST int32 [S], >= 1, or NULL (all 1).  A stage with group n has ceil(m / n) items per
 *     kind; item g stands for the micro-batches g n .. min(m, (g + 1) n) - 1, and the micro-batch
 *     field of its op words holds g (a larger value is a malformed word).  A synchronisation every n
 *     micro-batches is a stage of the DAG with group n: its forward item is the synchronisation, its
 *     backward (and weight-gradient) item what the backward pass has to do there, possibly at cost 0.
 *   - along a DAG edge or a pair, an item waits for EVERY item of the other stage whose micro-batches
 *     overlap its own.
 *   - pairs: HOST [n_pairs].  An item of kind_to on stage_to starts no earlier than the finish of the
 *     items of kind_from on stage_from, plus `latency` if the two stages sit on different devices.
 *     kind_from: FPSCHED_F (stands for F and FD, whichever ran), FPSCHED_B or FPSCHED_W; kind_to: any
 *     kind (FPSCHED_F also constrains FD).  Pairs that close a cycle make candidates deadlock, which
 *     their flags report.
 * From then on fpsched_evaluate (and fpsched_evaluate_topk_static) time the candidates under this
 * model -- with the slot kernel when every pair runs forward-to-forward or backward-to-backward, no
 * stage has more than two inputs or outputs in a direction (pairs included) and the neighbours of a
 * stage with group > 1 all have group 1, else with a kernel that keeps whole finish-time tables in LDS
 * (fpsched_problem_active_kernel says which; the slot kernel needs the workspace as in the plain
 * model); fpsched_encode and fpsched_validate check micro-batch fields against the item counts.
 * (NULL, 0, NULL) switches back.
 * Copied; synchronous (waits for the device's queued work); allocates one table of device memory
 * (FPSCHED_ENOMEM), freed by fpsched_problem_destroy.  FPSCHED_EINVAL for a group < 1, a stage or
 * kind out of range, a negative latency, W without split backward, or a pair from an item to
 * itself; FPSCHED_EOVERFLOW if D * max_stride * (max dur + max latency) >= 2^31; FPSCHED_EUNSUPPORTED
 * if the tables do not fit LDS, or while costs per micro-batch or link occupancy are set (and those
 * two setters, fpsched_wslide and fpsched_generate answer FPSCHED_EUNSUPPORTED while this is set): the
 * handle then keeps what it had.  Works on a host-only handle (validation, encode, validate). */
typedef struct {
  int32_t kind_from, stage_from; /* the item waited for  */
  int32_t kind_to, stage_to;     /* the item that waits  */
  int32_t latency;               /* >= 0, added iff the two stages sit on different devices */
} fpsched_dependency;
int fpsched_problem_set_sync(fpsched_problem *p, const int32_t *group, int32_t n_pairs,
                             const fpsched_dependency *pairs);

/* Variant of the cost model: a copy engine for offload and reload items.  The paper names CPU offloading
 * among the memory optimisations of pipeline schedules (Section 8) and does not say how an offload is
 * timed; fpsched_evaluate runs O and L items on the device's compute timeline like any other item.
 * With depth >= 1 they run on a copy timeline of the device, beside the computation:
 *   - each timeline is serial and keeps the order of the device's list; the walk through the list
 *     hands a transfer to the copy engine when it reaches it (every compute item in front of it has
 *     finished) and goes on at once; the engine holds at most `depth` unfinished transfers, and a
 *     walk that reaches a transfer while `depth` are unfinished waits for the oldest of them;
 *   - a transfer starts at max(hand-over, finish of the transfer before it) and takes
 *     dur[kind][stage]; a backward item starts no earlier than the finish of the reload of its
 *     activation; the activation state machine follows the list order as before;
 *   - memory is counted over time: +units at the start of F, FD, R, L, -units at the end of FD, O
 *     and W (B without split backward); peak[d] is the largest running sum over the device's events
 *     in time order, the compute timeline's events first at equal times;
 *   - makespan = the latest finish on either timeline; idle[d] = makespan - the costs of d's compute
 *     items.  Flags, sentinels and ranking are unchanged.  Lists without O and L items are timed
 *     exactly as before.
 * depth == 0 switches back; 1 <= depth <= FPSCHED_MAX_COPY_DEPTH.  FPSCHED_EINVAL if depth is out of
 * range or some stage has dur[O] < 1 or dur[L] < 1 (a transfer takes time); FPSCHED_EUNSUPPORTED if
 * the tables do not fit LDS or while costs per micro-batch, link occupancy or fpsched_problem_set_sync
 * are in force (and those setters, fpsched_wslide answer FPSCHED_EUNSUPPORTED while this is): the
 * handle keeps what it had.  Synchronous; allocates one table of device memory at most; works on a
 * host-only handle (validation only).  Both evaluation kernels have a form of this model: the slot
 * kernel's runs when the problem fits it (fpsched_problem_select_kernel chooses as for the plain
 * model), and then fpsched_evaluate needs its workspace as in the plain model. */
#define FPSCHED_MAX_COPY_DEPTH 7
int fpsched_problem_set_copy_engine(fpsched_problem *p, int32_t depth);

/* DEVICE buffers the caller owns (e.g. torch tensors); all must hold n_cand entries. */
typedef struct {
  int64_t *makespan; /* [C]     max finish time over all devices                          */
  int64_t *idle;     /* [C][D]  makespan - busy time of the device (head/tail included)   */
  int32_t *peak;     /* [C][D]  peak resident activation units                            */
  uint8_t *flags;    /* [C]     FPSCHED_FLAG_* bits                                       */
} fpsched_results;

/* Bytes of DEVICE workspace fpsched_evaluate / fpsched_topk need for this batch (>= 256;
 * k may be 0 when only fpsched_evaluate is called).  The workspace must be 16-byte aligned;
 * the library keeps no other device scratch.  Two calls may share a workspace only if they
 * run one after the other on the same stream. */
size_t fpsched_workspace_bytes(const fpsched_problem *p, int64_t n_cand, int32_t k);

/* Evaluate n_cand candidates.  d_ops: DEVICE, uint16 [n_cand][D][stride_words],
 * 16-byte aligned, stride_words a multiple of 8 and <= the handle's max stride.
 * Start rule (Section 5.1 "Data dependency" + the estimator's task graph with
 * start/end/cost): forward items wait for the forward items of the predecessor
 * stages, backward items for the backward items of the successor stages, each
 * device runs its list in order;  start = max(device free, inputs' finish +
 * cross-device latency),  finish = start + dur[kind][stage].
 * Asynchronous: work is enqueued on hip_stream (a hipStream_t, NULL = default
 * stream) and the call returns.  n_cand == 0 is a no-op. */
int fpsched_evaluate(const fpsched_problem *p, const uint16_t *d_ops, int64_t n_cand,
                     int32_t stride_words, fpsched_results out, void *d_workspace,
                     size_t workspace_bytes, void *hip_stream);

/* k best candidates with flags == 0 by (makespan ascending, index ascending)
 * (Section 7.1: least bubble ratio; total work per problem is fixed, so this is
 * least makespan).  d_idx, d_makespan: DEVICE [k]; unused slots get -1 and
 * INT64_MAX.  d_count: DEVICE, min(k, #feasible).  1 <= k <= 1024.  Reads only
 * in.makespan and in.flags.  Asynchronous on hip_stream. */
int fpsched_topk(const fpsched_problem *p, fpsched_results in, int64_t n_cand, int32_t k,
                 int64_t *d_idx, int64_t *d_makespan, int32_t *d_count, void *d_workspace,
                 size_t workspace_bytes, void *hip_stream);

/* For callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  fpsched_evaluate followed by
 * fpsched_topk on the same results, with the work counter and the top-k key buffers in a
 * static array of FPSCHED_STATIC_SCRATCH_BYTES that every GPU the library runs on holds from
 * the first fpsched_problem_create on that GPU until the process ends; the call itself
 * allocates nothing, on the host or on the device.  Arguments, results and error codes are
 * those of the two calls; in addition FPSCHED_ESCRATCH if fpsched_workspace_bytes(p, n_cand, k)
 * exceeds the array (2 MiB: room for 172,032 candidates at k = 1024, 1.4 million at k = 128,
 * 16 million at k <= 16), in which case nothing is enqueued.  All calls on one GPU share that GPU's array:
 * two calls that overlap in time on one GPU (different streams, or different host threads
 * without ordering between their streams) race; calls on one stream, or ordered by events,
 * are safe, and so are calls on different GPUs.  Nothing of an earlier call's contents is read.
 * Asynchronous on hip_stream. */
#define FPSCHED_STATIC_SCRATCH_BYTES (2u << 20)
size_t fpsched_static_scratch_bytes(void);
int fpsched_evaluate_topk_static(const fpsched_problem *p, const uint16_t *d_ops, int64_t n_cand,
                                 int32_t stride_words, fpsched_results out, int32_t k,
                                 int64_t *d_idx, int64_t *d_makespan, int32_t *d_count,
                                 void *hip_stream);

/* Richer ranking of evaluated candidates: the k best by a two-part key, ties by index.
 * The paper ranks by bubble ratio (Section 7.1) and treats the memory footprint as the
 * second property of a schedule (Section 2); the modes make both usable as sort keys:
 *   FPSCHED_RANK_MAKESPAN        (makespan)                 -- the same order as fpsched_topk
 *   FPSCHED_RANK_MAKESPAN_PEAK   (makespan, largest peak[d])
 *   FPSCHED_RANK_PEAK_MAKESPAN   (largest peak[d], makespan)
 *   FPSCHED_RANK_IDLE            (sum of idle[d])
 * Candidates with DEADLOCK or INCOMPLETE never rank; OVER_CAP ones only if include_over_cap
 * is non-zero (ranking by memory instead of cutting at the cap).  d_key: DEVICE [k], the
 * key of each winner: primary << 32 | secondary for the two-part modes, the value itself
 * otherwise; unused slots idx -1, key INT64_MAX.  Workspace: fpsched_rank_workspace_bytes.
 * Reads every field of `in`.  1 <= k <= 1024.  Asynchronous on hip_stream. */
#define FPSCHED_RANK_MAKESPAN 0
#define FPSCHED_RANK_MAKESPAN_PEAK 1
#define FPSCHED_RANK_PEAK_MAKESPAN 2
#define FPSCHED_RANK_IDLE 3
size_t fpsched_rank_workspace_bytes(const fpsched_problem *p, int64_t n_cand, int32_t k);
int fpsched_rank(const fpsched_problem *p, fpsched_results in, int64_t n_cand, int32_t k,
                 int32_t mode, int32_t include_over_cap, int64_t *d_idx, int64_t *d_key,
                 int32_t *d_count, void *d_workspace, size_t workspace_bytes, void *hip_stream);

/* Weight-gradient sliding (Section 5.2, "Bubble optimizations": the weight-gradient part of a
 * backward pass is stashed and run in a later bubble of the same actor, so that the items
 * other actors wait for run first).  The paper shows the idea on a figure and states no rule
 * for which bubble takes which stashed item; this call applies the following one to every
 * candidate of a batch, for problems with split backward (has_w; else FPSCHED_EINVAL):
 *   - the W words of the input lists are dropped, the other items keep their order;
 *   - every device walks its list under the start rule of fpsched_evaluate; a B item that
 *     issues puts its W item at the back of the device's stash (first in, first out);
 *   - in front of the next item of the list, which starts at time t, the oldest stashed
 *     item runs at the time the device is free if it ends by t (free + dur[W][stage] <= t),
 *     then the next oldest, and so on; the item of the list is never delayed;
 *   - when the list ends, what is still stashed runs back to back.
 * d_ops_out: DEVICE uint16 [n_cand][D][stride_out_words], 16-byte aligned, stride_out_words
 * a multiple of 8 and <= the handle's max stride: the new lists (the order in which the
 * items issued), END-padded.  `out`: the evaluation of the new lists, as fpsched_evaluate
 * would report it for them.  A new row too short for all items of its device keeps the first
 * stride_out_words of them; the other devices are not affected (where the W items go never
 * moves an item of the list), and the candidate is reported as DEADLOCK | INCOMPLETE with
 * the sentinels.  Rows of candidates that fail otherwise hold the items that did issue.
 * The makespan may grow: an item that moves up can open idle time that the stashed items do
 * not fit into; evaluate both lists and rank.  Needs the slot tables (at most two inputs and
 * outputs per stage, see fpsched_problem_info), else FPSCHED_EUNSUPPORTED.  Cost model: the
 * handle's latencies as pure latencies or, after fpsched_problem_set_link_occupancy, as links
 * that carry one value at a time; FPSCHED_EUNSUPPORTED while costs per micro-batch are set.
 * Workspace: fpsched_wslide_workspace_bytes (DEVICE, 16-byte aligned; it holds sixteen bits
 * per op word and lane of a candidate plus a short list per row for the ops that wait 2^16 time
 * units or more, i.e. about the bytes of the input lists).  Asynchronous on hip_stream. */
size_t fpsched_wslide_workspace_bytes(const fpsched_problem *p, int64_t n_cand, int32_t stride_words);
int fpsched_wslide(const fpsched_problem *p, const uint16_t *d_ops, int64_t n_cand,
                   int32_t stride_words, uint16_t *d_ops_out, int32_t stride_out_words,
                   fpsched_results out, void *d_workspace, size_t workspace_bytes,
                   void *hip_stream);

/* The same pass when only the evaluation of the new lists is wanted (a search that ranks the
 * slid candidates and then asks fpsched_wslide for the lists of the few it keeps): `out` is
 * what fpsched_wslide reports with rows long enough for every item, without any list being
 * written (Section 5.2, bubble optimizations; the rules above).  One kernel: the walk of
 * fpsched_evaluate over the lists without their W words, in which a device runs its oldest
 * stashed W items in front of every item they end before.  Same arguments, alignment and
 * errors as fpsched_evaluate; workspace: fpsched_workspace_bytes(p, n_cand, 0) (DEVICE, 16-byte
 * aligned).  Cost model: as for fpsched_wslide (pure latencies, or links that carry one value
 * at a time).  FPSCHED_EINVAL without split backward; FPSCHED_EUNSUPPORTED without the slot
 * tables or while costs per micro-batch, synchronisation stages or the copy engine are set.
 * Asynchronous on hip_stream. */
int fpsched_wslide_evaluate(const fpsched_problem *p, const uint16_t *d_ops, int64_t n_cand,
                            int32_t stride_words, fpsched_results out, void *d_workspace,
                            size_t workspace_bytes, void *hip_stream);

/* Pareto front of (makespan, largest peak[d]) over the candidates that completed (neither
 * DEADLOCK nor INCOMPLETE; OVER_CAP is ignored: the front takes the place of a fixed cap).
 * The paper gives a schedule two properties, bubble ratio (Section 7.1) and memory footprint
 * (Section 2), and lets the tuner return several alternatives; the front is every candidate
 * that no other one matches or beats in both values (of candidates with the same pair the
 * one with the smallest index stands for all).  Output by ascending makespan, hence strictly
 * descending peak: d_idx, d_makespan (int64), d_peak (int32): DEVICE [kmax]; d_count: DEVICE,
 * min(kmax, size of the front) -- a count equal to kmax may mean that the tail was cut off;
 * unused slots idx -1, makespan INT64_MAX, peak -1.  1 <= kmax <= 1024; n_cand <= 2^24,
 * else FPSCHED_EINVAL.  Workspace: fpsched_pareto_workspace_bytes, 16-byte aligned.  Reads
 * in.makespan, in.peak, in.flags.  Asynchronous on hip_stream. */
size_t fpsched_pareto_workspace_bytes(const fpsched_problem *p, int64_t n_cand);
int fpsched_pareto(const fpsched_problem *p, fpsched_results in, int64_t n_cand, int32_t kmax,
                   int64_t *d_idx, int64_t *d_makespan, int32_t *d_peak, int32_t *d_count,
                   void *d_workspace, size_t workspace_bytes, void *hip_stream);

/* Judge evaluated candidates against other memory caps than the problem's, without timing
 * them again (Section 2: the footprint of a schedule against the memory of the devices it
 * is to run on): rewrites the OVER_CAP bit of d_flags (DEVICE uint8 [n_cand], in place) from
 * d_peak (DEVICE int32 [n_cand][D]); the other bits stay, failed candidates never get the
 * bit.  d_caps: DEVICE int32 [D] (per_candidate == 0) or [n_cand][D] (per_candidate != 0),
 * in the units of the problem's mem_units.  Asynchronous on hip_stream. */
int fpsched_apply_caps(const fpsched_problem *p, const int32_t *d_peak, const int32_t *d_caps,
                       int32_t per_candidate, int64_t n_cand, uint8_t *d_flags, void *hip_stream);

/* HOST helper: pack n items (kind, stage, micro-batch) of one device's list into
 * words (stage -> device-local chunk).  out_words: HOST [n].  EINVAL if an item
 * names a stage that is not on `device`, a bad kind or micro-batch. */
int fpsched_encode(const fpsched_problem *p, const int32_t *kind_stage_mb /* HOST [n][3] */,
                   int32_t device, int32_t n, uint16_t *out_words);

/* HOST helper: structural check of a HOST batch [n_cand][D][stride_words]: every word
 * before a row's first END has a valid chunk for its device, micro-batch < m,
 * and W only when has_w.  Returns the number of bad candidates (>= 0) or an error. */
int64_t fpsched_validate(const fpsched_problem *p, const uint16_t *h_ops, int64_t n_cand,
                         int32_t stride_words);

/* Introspection (HOST): which kernel variant the handle selected and how many
 * candidates one wavefront carries. */
int fpsched_problem_info(const fpsched_problem *p, int32_t *lanes_per_candidate,
                         int32_t *candidates_per_wave, int32_t *lds_bytes_per_wave);

/* Two evaluation kernels compute the same results.  SLOTS (default whenever its LDS
 * footprint fits): per-micro-batch mail slots, a few KB of LDS per candidate.  GENERAL:
 * whole finish-time tables in LDS, one wavefront per workgroup; kept for problems whose
 * state words do not fit the slot kernel and as a cross-check.  EUNSUPPORTED if the
 * requested kernel does not fit this problem. */
#define FPSCHED_KERNEL_AUTO 0
#define FPSCHED_KERNEL_GENERAL 1
#define FPSCHED_KERNEL_SLOTS 2
int fpsched_problem_select_kernel(fpsched_problem *p, int which);
/* Which of the two fpsched_evaluate would launch under the handle's present cost model and selection:
 * FPSCHED_KERNEL_SLOTS or FPSCHED_KERNEL_GENERAL (the table form: eval_general_kernel, or eval_sync_kernel
 * under the synchronisation or copy-engine model when the setting does not fit the slot kernel); a negative
 * code for a null or host-only handle. */
int fpsched_problem_active_kernel(const fpsched_problem *p);

/* ---- schedule generator: the actor-aware schedule of Section 5 -------------------------
 * One actor's scheduling priorities (Section 5.2; table of built-in values): the
 * computation type traversal priority with its scheduling units, and the stage traversal
 * priority (direction and optional interval) for forward and for backward items. */
#define FPSCHED_CTTP_BWD_FIRST 0
#define FPSCHED_CTTP_FWD_FIRST 1
#define FPSCHED_CTTP_INTERLEAVED 2
#define FPSCHED_STP_BREADTH_FIRST 0 /* ascending stage id  */
#define FPSCHED_STP_DEPTH_FIRST 1   /* descending stage id */
typedef struct {
  int32_t cttp;       /* FPSCHED_CTTP_*                                                    */
  int32_t unit_f;     /* unit1: forward items per turn (interleaved only, else 1)          */
  int32_t unit_b;     /* unit2: backward items per turn (interleaved only, else 1)         */
  int32_t f_dir;      /* FPSCHED_STP_* for forward items                                   */
  int32_t f_interval; /* 0 = not set                                                       */
  int32_t b_dir;      /* FPSCHED_STP_* for backward items                                  */
  int32_t b_interval; /* 0 = not set                                                       */
  int32_t reserved;   /* 0                                                                 */
} fpsched_actor_policy;

#define FPSCHED_GEN_STUCK 1      /* items remained and no actor could schedule any          */
#define FPSCHED_GEN_BAD_POLICY 4 /* a value outside its domain: nothing generated           */

/* Generate one schedule per parameter set (Section 5.2, Steps 1-5, with the step function
 * of Algorithm 1): in every scheduling step all actors look at the state the previous
 * step left and each schedules at most one instruction item -- forward (F), backward (B)
 * and, iff the problem splits the backward pass, weight-gradient (W) items; durations
 * play no part.  Dependencies: F(s,j) after F of every DAG predecessor of s, B(s,j) after
 * F(s,j) and B of every DAG successor, W(s,j) after B(s,j); within a type and stage,
 * micro-batches ascend.  Type order: bwdpass-first = B, F; fwdpass-first = F, B;
 * interleaved = the type whose turn it is, then the other (a turn ends after unit_f
 * forward / unit_b backward items of the turn's own type; the first turn is forward); W is
 * tried last, stages ascending.  Stage traversal without an interval: the actor's stages
 * in the traversal direction, first eligible wins; with an interval n: the actor stays on
 * one stage until it has scheduled n items of the type there (or the stage has no
 * eligible item), then moves on in the direction, cyclically, to the next stage that has
 * one; a type none of whose items is eligible is skipped, and the actor idles in a step
 * only when no type has an eligible item.  An F item of
 * stage s is eligible only while (#F - #B scheduled on s) < d_inflight[s] (Section 4.2,
 * the in-flight micro-batch limit; INT32_MAX = none, values < 1 are a bad policy).
 *
 * d_policy: DEVICE fpsched_actor_policy [n_sets][D]; d_inflight: DEVICE int32 [n_sets][S].
 * d_ops: DEVICE out, uint16 [n_sets][D][stride_words], 16-byte aligned, every row written
 * in full (END-padded); stride_words a multiple of 8 and >= (most stages on one device)
 * x m x (3 if has_w else 2).  d_steps: DEVICE out int32 [n_sets], scheduling steps taken
 * (the unit-time length of the schedule, bubbles included); d_status: DEVICE out uint8
 * [n_sets], 0 or FPSCHED_GEN_*.  d_workspace: DEVICE, 16-byte aligned, >= 256 bytes (a work
 * counter; the same rules as for fpsched_evaluate).  Asynchronous on hip_stream.
 * EUNSUPPORTED if the problem's tables do not fit LDS. */
int fpsched_generate(const fpsched_problem *p, const fpsched_actor_policy *d_policy,
                     const int32_t *d_inflight, int64_t n_sets, int32_t stride_words,
                     uint16_t *d_ops, int32_t *d_steps, uint8_t *d_status, void *d_workspace,
                     size_t workspace_bytes, void *hip_stream);

/* Generator and evaluator in one pass (the tuner's loop of Section 6: enumerate schedule types,
 * let the scheduler of Section 5 produce each schedule, let the estimator time it, rank): for every
 * parameter set the schedule fpsched_generate would write is timed while it is generated, and
 * only the results leave the chip -- out gets exactly what fpsched_evaluate gives for the rows
 * fpsched_generate writes for the same set (a set that ends stuck or has a bad policy leaves items
 * unscheduled: FPSCHED_FLAG_INCOMPLETE and the sentinels), d_steps and d_status what
 * fpsched_generate gives.  An item is scheduled only after all it depends on was scheduled in an
 * earlier step, so its start (Section 5.1, data dependency; start = max(device free, inputs'
 * finish + cross-device latency)) is known when it is placed.  The plain cost model only:
 * FPSCHED_EUNSUPPORTED while costs per micro-batch, link occupancy, synchronisation stages or the
 * copy engine are set, if a stage has more than two inputs or outputs, or if the tables do not
 * fit LDS; FPSCHED_EOVERFLOW if 3 S m (max dur + max comm) >= 2^30.  Buffers as for
 * fpsched_generate (no d_ops) and fpsched_evaluate; d_workspace >= 256 bytes.  The schedules of
 * the sets that fpsched_topk then names are obtained with fpsched_generate_selected. */
int fpsched_generate_evaluate(const fpsched_problem *p, const fpsched_actor_policy *d_policy,
                              const int32_t *d_inflight, int64_t n_sets, fpsched_results out,
                              int32_t *d_steps, uint8_t *d_status, void *d_workspace,
                              size_t workspace_bytes, void *hip_stream);

/* fpsched_generate_evaluate with the weight-gradient sliding pass in it (Section 5.2: the scheduler,
 * then the bubble optimization, then the estimator): `out` is what fpsched_wslide_evaluate reports
 * for the lists fpsched_generate writes for the same parameter sets, d_steps and d_status are those
 * of fpsched_generate.  Nothing but the results leaves the chip.  Same arguments, workspace and
 * errors as fpsched_generate_evaluate; FPSCHED_EINVAL for a problem without split backward. */
int fpsched_generate_slide_evaluate(const fpsched_problem *p, const fpsched_actor_policy *d_policy,
                                    const int32_t *d_inflight, int64_t n_sets, fpsched_results out,
                                    int32_t *d_steps, uint8_t *d_status, void *d_workspace,
                                    size_t workspace_bytes, void *hip_stream);

/* fpsched_generate for chosen parameter sets: row block i of d_ops (and d_steps[i], d_status[i])
 * is the schedule of parameter set d_select[i] (DEVICE int64 [n_selected], e.g. the indices
 * fpsched_topk wrote) of the n_sets sets that d_policy and d_inflight hold.  An entry outside
 * 0 .. n_sets - 1 (the -1 of an unused top-k slot) selects nothing: empty rows,
 * FPSCHED_GEN_BAD_POLICY; no set is ever read that the caller did not say is there. */
int fpsched_generate_selected(const fpsched_problem *p, const fpsched_actor_policy *d_policy,
                              const int32_t *d_inflight, int64_t n_sets, const int64_t *d_select,
                              int64_t n_selected, int32_t stride_words, uint16_t *d_ops,
                              int32_t *d_steps, uint8_t *d_status, void *d_workspace,
                              size_t workspace_bytes, void *hip_stream);

const char *fpsched_strerror(int code);
int fpsched_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FPSCHED_H */

/* CPU oracle of the schedule generator -- TEST INFRASTRUCTURE ONLY.
 *
 * What it computes (paper Section 5, "Scheduler"): the actor-aware schedule.
 * Every micro-batch computation is an instruction item (type, stage,
 * micro-batch) held in an instruction pool (Section 5.1 "Instruction pool");
 * items whose data dependencies are resolved sit in per-actor, per-type
 * reorder queues (Section 5.1 "Actor-aware reorder queues"); in every
 * scheduling step all actors run the step function (Algorithm 1) on the state
 * left by the previous step, each fetching at most one item (Section 5.2,
 * Steps 1-5; the local buffer keeps an actor's choice invisible to the other
 * actors until the step is over); the dependency resolver then moves the
 * successors whose dependencies are resolved into the reorder queues
 * (Section 5.1 "Dynamic data dependency resolver").  The result is one
 * instruction sequence per actor (= device), which the evaluator then times.
 *
 * This file does it item by item with explicit pool / queue flags and linear
 * scans, in the order of the paper's steps.  No counters, no shortcuts.
 *
 * Readings of the paper taken here:
 *  G1 instruction types: FwdPass (F), BwdPass (B), and the weight-gradient
 *     computation (W) iff the problem splits the backward pass.
 *  G3 dependencies: F(s,j) after F(p,j) for every DAG predecessor p of s;
 *     B(s,j) after F(s,j) and after B(q,j) for every DAG successor q;
 *     W(s,j) after B(s,j).  Step 1: the F items of the stages without a
 *     predecessor start in their reorder queue.
 *  G4 an item resolved in step t can be fetched from step t+1 on, also by
 *     the actor that resolved it.
 *  G5 type order (Algorithm 1, sort_inst_types): bwdpass-first = B, F, W;
 *     fwdpass-first = F, B, W; interleaved(unit1, unit2) = the type whose
 *     turn it is, then the other, then W; a turn ends after unit1 forward
 *     (unit2 backward) items of that type were scheduled in it; an item of
 *     another type scheduled meanwhile leaves the turn as it is.  The first
 *     turn is forward.  W is always tried last (it fills bubbles), scanning
 *     the actor's stages in ascending order.
 *  G6 stage traversal (Algorithm 1, parse_stp / fetch): a stage's candidate is
 *     the smallest micro-batch in the reorder queue for that stage.  Without
 *     an interval the actor's stages are scanned in the traversal direction
 *     (breadth-first = ascending stage id, depth-first = descending) and the
 *     first stage with an eligible candidate (in the queue and passing the
 *     check function) wins.  With an interval n the actor keeps (position,
 *     stepped) per type: when `stepped` has reached n, or the stage at the
 *     position has no eligible candidate, the position moves on in the
 *     traversal direction (cyclically) to the next stage that has one and
 *     `stepped` restarts; the candidate of the stage at the position is
 *     scheduled.  If no stage has an eligible candidate the next instruction
 *     type is tried: the actor idles in a step only if none of its items
 *     can be scheduled (Section 5.2, Step 2).
 *  G7 the check function is the in-flight rule: an F item of stage s is
 *     eligible only while (#F scheduled on s) - (#B scheduled on s) is below
 *     the stage's in-flight limit.
 *  G8 a step in which no actor schedules anything although items remain ends
 *     the process with status 1 (stuck); the sequences produced so far are
 *     kept.  (With limits >= 1 and an acyclic stage graph this cannot happen:
 *     the oldest unfinished micro-batch can always move.  The status is kept
 *     as a guard.)
 *
 * Pinned by tests (tests/test_genoracle.py): exact 1F1B and GPipe orders and
 * their 2(m+p-1) steps, the interleaved-1F1B length 2vm+2(p-1) for the paper's
 * interleaved setting, an independent counter-based simulator on random
 * policies, validity of every generated schedule under the evaluation oracle,
 * in-flight limits on every prefix, steps == unit-time makespan of the
 * generated order under the evaluation oracle, hand-worked small cases.
 * Parity unpinned: nothing printed in the paper gives a generated schedule
 * item by item (its figures are images), so no pin compares against a value
 * of the paper; the interleaved schedule is pinned by its length and by
 * properties, not item by item.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { T_F = 0, T_B = 1, T_W = 2, NTYPES = 3 };
enum { CTTP_BWD_FIRST = 0, CTTP_FWD_FIRST = 1, CTTP_INTERLEAVED = 2 };
enum { DIR_BREADTH = 0, DIR_DEPTH = 1 };
enum { POLICY_INTS = 8 };
enum { K_F = 1, K_B = 2, K_W = 3 };   /* op-word kinds of the three types */

typedef struct {
  int32_t n_devices;
  int32_t n_stages;
  int32_t n_microbatches;
  int32_t has_w;
  const int32_t *stage_device; /* [S] */
  int32_t n_edges;
  const int32_t *edge_src; /* [E] */
  const int32_t *edge_dst; /* [E] */
} fpgen_problem;

typedef struct {
  int D, S, m, ntypes;
  const fpgen_problem *P;
  uint8_t *scheduled; /* [NTYPES][S][m] the instruction pool's state */
  uint8_t *queued;    /* [NTYPES][S][m] item is in its actor's reorder queue */
  int stages_of[64][4], n_stages_of[64], chunk_of[256 * 16];
} gen_state;

static size_t item(const gen_state *g, int t, int s, int j) {
  return ((size_t)t * g->S + s) * g->m + j;
}

/* every dependency of the item scheduled? (G3) */
static int deps_resolved(const gen_state *g, int t, int s, int j) {
  const fpgen_problem *P = g->P;
  if (t == T_F) {
    for (int e = 0; e < P->n_edges; ++e)
      if (P->edge_dst[e] == s && !g->scheduled[item(g, T_F, P->edge_src[e], j)]) return 0;
    return 1;
  }
  if (t == T_B) {
    if (!g->scheduled[item(g, T_F, s, j)]) return 0;
    for (int e = 0; e < P->n_edges; ++e)
      if (P->edge_src[e] == s && !g->scheduled[item(g, T_B, P->edge_dst[e], j)]) return 0;
    return 1;
  }
  return g->scheduled[item(g, T_B, s, j)];
}

static void try_queue(gen_state *g, int t, int s, int j) {
  const size_t i = item(g, t, s, j);
  if (!g->scheduled[i] && !g->queued[i] && deps_resolved(g, t, s, j)) g->queued[i] = 1;
}

static int count_scheduled(const gen_state *g, int t, int s) {
  int n = 0;
  for (int j = 0; j < g->m; ++j) n += g->scheduled[item(g, t, s, j)];
  return n;
}

/* the stage's candidate: smallest micro-batch in the reorder queue, -1 if none (G6) */
static int candidate(const gen_state *g, int t, int s) {
  for (int j = 0; j < g->m; ++j)
    if (g->queued[item(g, t, s, j)]) return j;
  return -1;
}

/* the check function of the fetch (G7) */
static int passes_check(const gen_state *g, int t, int s, const int32_t *inflight) {
  if (t != T_F) return 1;
  return (int64_t)count_scheduled(g, T_F, s) - count_scheduled(g, T_B, s) < (int64_t)inflight[s];
}

static int eligible(const gen_state *g, int t, int s, const int32_t *inflight) {
  return candidate(g, t, s) >= 0 && passes_check(g, t, s, inflight);
}

typedef struct {
  int turn_type, turn_run;          /* interleaved: whose turn, items scheduled in it */
  int pos[NTYPES], stepped[NTYPES]; /* interval traversal state per type (index into the actor's stages) */
} actor_state;

/* One actor's step function (Algorithm 1).  Returns 1 and the item, or 0 (a bubble). */
static int step_function(const gen_state *g, int a, const int32_t *pol, const int32_t *inflight,
                         actor_state *st, int *out_t, int *out_s, int *out_j) {
  const int cttp = pol[0];
  int order[NTYPES], n_order = 0;
  if (cttp == CTTP_BWD_FIRST) { order[n_order++] = T_B; order[n_order++] = T_F; }
  else if (cttp == CTTP_FWD_FIRST) { order[n_order++] = T_F; order[n_order++] = T_B; }
  else { order[n_order++] = st->turn_type; order[n_order++] = st->turn_type == T_F ? T_B : T_F; }
  if (g->ntypes == 3) order[n_order++] = T_W;
  const int nst = g->n_stages_of[a];
  for (int oi = 0; oi < n_order; ++oi) {
    const int t = order[oi];
    /* is the reorder queue of (actor, type) empty? */
    int any = 0;
    for (int c = 0; c < nst && !any; ++c) any = candidate(g, t, g->stages_of[a][c]) >= 0;
    if (!any) continue;
    const int dir = t == T_F ? pol[3] : (t == T_B ? pol[5] : DIR_BREADTH);
    const int interval = t == T_F ? pol[4] : (t == T_B ? pol[6] : 0);
    if (interval > 0) {
      int p = st->pos[t];
      int any_eligible = 0;
      for (int c = 0; c < nst; ++c) any_eligible |= eligible(g, t, g->stages_of[a][c], inflight);
      if (!any_eligible) continue;
      if (st->stepped[t] == interval || !eligible(g, t, g->stages_of[a][p], inflight)) {
        /* move on, in the traversal direction, to the next stage with an eligible candidate */
        for (int k = 0; k < nst; ++k) {
          p = dir == DIR_BREADTH ? (p + 1) % nst : (p + nst - 1) % nst;
          if (eligible(g, t, g->stages_of[a][p], inflight)) break;
        }
        st->pos[t] = p;
        st->stepped[t] = 0;
      }
      const int s = g->stages_of[a][p];
      st->stepped[t] += 1;
      *out_t = t; *out_s = s; *out_j = candidate(g, t, s);
      return 1;
    } else {
      for (int k = 0; k < nst; ++k) {
        const int c = dir == DIR_BREADTH ? k : nst - 1 - k;
        const int s = g->stages_of[a][c];
        const int j = candidate(g, t, s);
        if (j >= 0 && passes_check(g, t, s, inflight)) {
          *out_t = t; *out_s = s; *out_j = j;
          return 1;
        }
      }
    }
  }
  return 0;
}

static uint16_t pack_word(int kind, int chunk, int mb) {
  return (uint16_t)((kind << 13) | (chunk << 11) | mb);
}

/* Generate one schedule.  policy: [D][POLICY_INTS] = {cttp, unit1, unit2, forward direction,
 * forward interval (0 = not set), backward direction, backward interval, 0}; inflight: [S].
 * out_words: [D][stride] (END-padded).  Returns 0, or -1 on an invalid description. */
int fpgen_oracle_one(const fpgen_problem *P, const int32_t *policy, const int32_t *inflight,
                     int32_t stride, uint16_t *out_words, int32_t *out_steps, uint8_t *out_status,
                     int32_t *out_prefix_violations) {
  gen_state g;
  g.D = P->n_devices; g.S = P->n_stages; g.m = P->n_microbatches; g.P = P;
  g.ntypes = P->has_w ? 3 : 2;
  if (g.D < 1 || g.D > 64 || g.S < 1 || g.S > 256 || g.m < 1 || g.m > 2048) return -1;
  memset(g.n_stages_of, 0, sizeof g.n_stages_of);
  for (int s = 0; s < g.S; ++s) {
    const int d = P->stage_device[s];
    if (d < 0 || d >= g.D || g.n_stages_of[d] >= 4) return -1;
    g.chunk_of[s] = g.n_stages_of[d];
    g.stages_of[d][g.n_stages_of[d]++] = s;
  }
  for (int a = 0; a < g.D; ++a) {
    const int32_t *pol = policy + (size_t)a * POLICY_INTS;
    if (pol[0] < 0 || pol[0] > 2 || pol[1] < 1 || pol[2] < 1 || pol[3] < 0 || pol[3] > 1 || pol[4] < 0 ||
        pol[5] < 0 || pol[5] > 1 || pol[6] < 0) return -1;
    if (pol[0] != CTTP_INTERLEAVED && (pol[1] != 1 || pol[2] != 1)) return -1;
  }
  for (int s = 0; s < g.S; ++s) if (inflight[s] < 1) return -1;
  const size_t n_items = (size_t)NTYPES * g.S * g.m;
  g.scheduled = calloc(n_items, 1);
  g.queued = calloc(n_items, 1);
  memset(out_words, 0, sizeof(uint16_t) * (size_t)g.D * stride);
  /* Step 1: the forward items of the stages without a predecessor are dependency-free */
  for (int s = 0; s < g.S; ++s)
    for (int j = 0; j < g.m; ++j)
      if (deps_resolved(&g, T_F, s, j)) g.queued[item(&g, T_F, s, j)] = 1;
  actor_state st[64];
  int len[64];
  for (int a = 0; a < g.D; ++a) {
    st[a].turn_type = T_F; st[a].turn_run = 0;
    for (int t = 0; t < NTYPES; ++t) {
      const int dir = t == T_F ? policy[a * POLICY_INTS + 3] : (t == T_B ? policy[a * POLICY_INTS + 5] : 0);
      st[a].pos[t] = dir == DIR_BREADTH ? 0 : (g.n_stages_of[a] > 0 ? g.n_stages_of[a] - 1 : 0);
      st[a].stepped[t] = 0;
    }
    len[a] = 0;
  }
  int64_t left = (int64_t)g.ntypes * g.S * g.m;
  int steps = 0, status = 0, violations = 0, overflow = 0;
  while (left > 0) {
    /* Step 2: every actor fetches from the state the previous step left */
    int pick_t[64], pick_s[64], pick_j[64], picked[64], n_picked = 0;
    for (int a = 0; a < g.D; ++a) {
      picked[a] = g.n_stages_of[a] > 0 &&
                  step_function(&g, a, policy + (size_t)a * POLICY_INTS, inflight, &st[a], &pick_t[a],
                                &pick_s[a], &pick_j[a]);
      n_picked += picked[a];
    }
    if (n_picked == 0) { status = 1; break; }
    ++steps;
    /* Steps 3 and 5: the choices become visible in the pool */
    for (int a = 0; a < g.D; ++a) {
      if (!picked[a]) continue;
      const int t = pick_t[a], s = pick_s[a], j = pick_j[a];
      g.scheduled[item(&g, t, s, j)] = 1;
      g.queued[item(&g, t, s, j)] = 0;
      --left;
      if (len[a] < stride) out_words[(size_t)a * stride + len[a]] = pack_word(t == T_F ? K_F : (t == T_B ? K_B : K_W), g.chunk_of[s], j);
      else overflow = 1;
      ++len[a];
      const int32_t *pol = policy + (size_t)a * POLICY_INTS;
      if (pol[0] == CTTP_INTERLEAVED && t == st[a].turn_type) {
        const int unit = t == T_F ? pol[1] : pol[2];
        if (++st[a].turn_run >= unit) { st[a].turn_type = t == T_F ? T_B : T_F; st[a].turn_run = 0; }
      }
    }
    /* Step 4: the resolver looks at the successors of every item scheduled in this step and
     * queues those whose dependencies are now all resolved */
    for (int a = 0; a < g.D; ++a) {
      if (!picked[a]) continue;
      const int t = pick_t[a], s = pick_s[a], j = pick_j[a];
      if (t == T_F) {
        for (int e = 0; e < P->n_edges; ++e)
          if (P->edge_src[e] == s) try_queue(&g, T_F, P->edge_dst[e], j);
        try_queue(&g, T_B, s, j);
      } else if (t == T_B) {
        for (int e = 0; e < P->n_edges; ++e)
          if (P->edge_dst[e] == s) try_queue(&g, T_B, P->edge_src[e], j);
        if (g.ntypes == 3) try_queue(&g, T_W, s, j);
      }
    }
    /* (diagnostic for the tests: per type and stage, scheduled items and queued items together
     * always form a prefix of the micro-batches) */
    for (int t = 0; t < g.ntypes; ++t)
      for (int s = 0; s < g.S; ++s) {
        int seen_gap = 0;
        for (int j = 0; j < g.m; ++j) {
          const size_t i = item(&g, t, s, j);
          if (!g.scheduled[i] && !g.queued[i]) seen_gap = 1;
          else if (seen_gap) ++violations;
        }
      }
  }
  free(g.scheduled);
  free(g.queued);
  *out_steps = steps;
  *out_status = (uint8_t)(status | (overflow ? 2 : 0));
  if (out_prefix_violations) *out_prefix_violations = violations;
  return 0;
}

/* n parameter sets: policy [n][D][POLICY_INTS], inflight [n][S] -> words [n][D][stride]. */
int fpgen_oracle_generate(const fpgen_problem *P, const int32_t *policy, const int32_t *inflight, int64_t n,
                          int32_t stride, uint16_t *out_words, int32_t *out_steps, uint8_t *out_status) {
  for (int64_t i = 0; i < n; ++i) {
    const int rc = fpgen_oracle_one(P, policy + (size_t)i * P->n_devices * POLICY_INTS,
                                    inflight + (size_t)i * P->n_stages, stride,
                                    out_words + (size_t)i * P->n_devices * stride, out_steps + i, out_status + i,
                                    NULL);
    if (rc) return rc;
  }
  return 0;
}

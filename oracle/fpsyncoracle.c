/*
 * fpsyncoracle.c -- CPU oracle of schedule evaluation with synchronisation stages and user
 * dependency pairs.
 *
 * TEST INFRASTRUCTURE ONLY.  A plain, slow, single-threaded event loop in int64; a file of its own that
 * shares no code with the plain evaluation oracle (fporacle.c), with the HIP sources or with the input
 * generators.  Nothing in the product path may call it.
 *
 * What the paper says (Section 4.2, "Registration of new instructions"; Section 2.2 and Section 7.2 on
 * multimodal models; Section 5.1, "Data dependency"):
 *   - a user can register a new instruction, e.g. the synchronisation that exchanges the output states
 *     of the submodules of a multimodal model; the instruction is attached to a stage registered for
 *     it, and its scheduling attributes say how many of the instructions it depends on must have been
 *     scheduled before it, and when the instructions that depend on it may follow (the comparison
 *     system synchronises once every few micro-batches);
 *   - dependencies between instructions are given as pairs ((type1, stage_i), (type2, stage_j)):
 *     type1 of stage_i comes before type2 of stage_j; they are added to those of the stage DAG.
 *
 * The model evaluated here:
 *   G1  every stage s has a group size group[s] >= 1.  A stage with group n has ceil(m / n) items per
 *       instruction type; item g stands for the micro-batches g n .. min(m, (g + 1) n) - 1, and the
 *       micro-batch field of its op words holds g.  An ordinary stage has group 1; a synchronisation
 *       every n micro-batches is a stage with group n whose forward item is the synchronisation.
 *   G2  an item of stage b depends, along a DAG edge or a dependency pair from stage a, on EVERY item
 *       of a whose micro-batches overlap its own:  items floor(lo / n_a) .. floor(hi / n_a) of a, where
 *       lo .. hi are the micro-batches of the item of b.  (n_a = n_b = 1: the same micro-batch.)
 *   G3  DAG edges: forward items (F, FD) wait for the forward items of the predecessor stages, backward
 *       items (B) for the backward items of the successor stages, as in the plain model.
 *   G4  a pair (kind_from, stage_from, kind_to, stage_to, latency): an item of kind_to on stage_to
 *       starts no earlier than the finish of the items of kind_from on stage_from that G2 names, plus
 *       the latency if the two stages sit on different devices.  kind_from is F (which also stands
 *       for FD: whichever ran), B or W; kind_to any kind (F also constrains FD).
 *   G5  everything else is the plain model: a device runs its list in order, one item at a time;
 *       start = max(device free, every dependency's finish + latency); the activation state machine per
 *       (stage, item); memory +units at the start of F, FD, R, L, -units at the end of FD, O and of W
 *       (or of B without split backward); idle, flags and sentinels.  A word whose micro-batch field is
 *       not below the item count of its stage is malformed.  Pairs that close a cycle make candidates
 *       deadlock; that is a property of the candidate, reported in its flags.
 *
 * Pins (tests/test_oracle_sync.py): group 1 and no pairs against the plain oracle (two files, two
 * loops); a pair that doubles a DAG edge; a hand-worked timeline with a synchronisation every two
 * micro-batches; the GPipe order with one synchronisation after all forward passes in closed form; an
 * independent critical-path checker (tests/sync_checker.py) on random problems, groups and pairs;
 * monotonicity.  Parity UNPINNED by the paper: it prints no timeline of a schedule with a registered
 * instruction; G1, G2 and G4 are this build's reading of Section 4.2.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { K_END = 0, K_F = 1, K_B = 2, K_W = 3, K_R = 4, K_O = 5, K_L = 6, K_FD = 7, NKINDS = 8 };
enum { ST_ABSENT = 0, ST_RES = 1, ST_DISC = 2, ST_OFF = 3, ST_BDONE = 4, ST_DONE = 5 };
enum { FLAG_DEADLOCK = 1, FLAG_INCOMPLETE = 2, FLAG_OVER_CAP = 4 };
#define MAX_CHUNKS 4

typedef struct {
  int32_t n_devices, n_stages, n_microbatches, has_w;
  const int32_t *stage_device; /* [S] */
  int32_t n_edges;
  const int32_t *edge_src, *edge_dst, *edge_comm; /* [E] */
  const int32_t *dur;       /* [NKINDS][S] */
  const int32_t *mem_units; /* [S] */
  const int32_t *mem_cap;   /* [D] */
  const int32_t *group;     /* [S] >= 1 */
  int32_t n_pairs;
  const int32_t *pairs;     /* [n_pairs][5]: kind_from, stage_from, kind_to, stage_to, latency */
} fpsync_problem;

static int items_of(const fpsync_problem *P, int s) {
  return (P->n_microbatches + P->group[s] - 1) / P->group[s];
}

/* finish times of the items other items can wait for: forward (F or FD), backward, weight gradient */
enum { T_FWD = 0, T_BWD = 1, T_WGT = 2, NTABLES = 3 };

/* Earliest time at which item g of stage s may start as far as the items of `table` on stage a are
 * concerned (G2), or -1 if one of them has not finished yet. */
static int64_t wait_for(const fpsync_problem *P, const int64_t *fin, int table, int a, int s, int g, int64_t lat) {
  const int m = P->n_microbatches;
  const int64_t lo = (int64_t)g * P->group[s];
  int64_t hi = lo + P->group[s] - 1;
  if (hi > m - 1) hi = m - 1;
  int64_t ready = 0;
  for (int64_t ga = lo / P->group[a]; ga <= hi / P->group[a]; ++ga) {
    const int64_t t = fin[((size_t)table * P->n_stages + a) * m + ga];
    if (t < 0) return -1;
    if (t + lat > ready) ready = t + lat;
  }
  return ready;
}

/* One candidate.  words: [D][stride].  Returns 0, or -1 for an invalid description. */
int fpsync_eval_one(const fpsync_problem *P, const uint16_t *words, int32_t stride, int64_t *makespan,
                    int64_t *idle, int32_t *peak, uint8_t *flags, int64_t *op_start, int64_t *op_finish) {
  const int D = P->n_devices, S = P->n_stages, m = P->n_microbatches, E = P->n_edges;
  if (D < 1 || S < 1 || m < 1) return -1;
  for (int s = 0; s < S; ++s) if (P->group[s] < 1) return -1;
  for (int i = 0; i < P->n_pairs; ++i) {
    const int32_t *q = P->pairs + 5 * i;
    if ((q[0] != K_F && q[0] != K_B && q[0] != K_W) || q[2] < K_F || q[2] > K_FD || q[1] < 0 || q[1] >= S ||
        q[3] < 0 || q[3] >= S || q[4] < 0) return -1;
  }
  int32_t local_stage[64 * MAX_CHUNKS], n_chunks[64];
  if (D > 64) return -1;
  for (int d = 0; d < D; ++d) n_chunks[d] = 0;
  for (int s = 0; s < S; ++s) {
    const int d = P->stage_device[s];
    if (d < 0 || d >= D || n_chunks[d] >= MAX_CHUNKS) return -1;
    local_stage[d * MAX_CHUNKS + n_chunks[d]++] = s;
  }
  int64_t *fin = malloc(sizeof(int64_t) * NTABLES * (size_t)S * m);
  uint8_t *state = calloc((size_t)S * m, 1);
  int32_t *cursor = calloc(D, sizeof(int32_t)), *len = calloc(D, sizeof(int32_t));
  int64_t *free_at = calloc(D, sizeof(int64_t)), *busy = calloc(D, sizeof(int64_t));
  int64_t *mem = calloc(D, sizeof(int64_t)), *pk = calloc(D, sizeof(int64_t));
  for (size_t i = 0; i < NTABLES * (size_t)S * m; ++i) fin[i] = -1;
  for (int d = 0; d < D; ++d) {
    int n = 0;
    while (n < stride && (words[(size_t)d * stride + n] >> 13) != K_END) ++n;
    len[d] = n;
  }
  if (op_start) for (int64_t i = 0; i < (int64_t)D * stride; ++i) op_start[i] = op_finish[i] = -1;

  int malformed_head = 0;
  for (;;) {
    int issued_any = 0;
    malformed_head = 0;
    for (int d = 0; d < D; ++d) {
      if (cursor[d] >= len[d]) continue;
      const uint16_t w = words[(size_t)d * stride + cursor[d]];
      const int kind = w >> 13, c = (w >> 11) & 3, g = w & 0x7ff;
      if (c >= n_chunks[d] || (kind == K_W && !P->has_w)) { malformed_head = 1; continue; }
      const int s = local_stage[d * MAX_CHUNKS + c];
      if (g >= items_of(P, s)) { malformed_head = 1; continue; }
      uint8_t *st = &state[(size_t)s * m + g];
      /* the activation state machine of the item's (stage, item) */
      int need, next;
      switch (kind) {
        case K_F:  need = ST_ABSENT; next = ST_RES; break;
        case K_FD: need = ST_ABSENT; next = ST_DISC; break;
        case K_R:  need = ST_DISC;   next = ST_RES; break;
        case K_O:  need = ST_RES;    next = ST_OFF; break;
        case K_L:  need = ST_OFF;    next = ST_RES; break;
        case K_B:  need = ST_RES;    next = ST_BDONE; break;
        default:   need = ST_BDONE;  next = ST_DONE; break; /* K_W */
      }
      if (*st != need) continue;
      /* dependencies: the stage DAG (G3), then the pairs (G4) */
      int64_t ready = 0;
      int blocked = 0;
      for (int e = 0; e < E && !blocked; ++e) {
        int a = -1, table = 0;
        if ((kind == K_F || kind == K_FD) && P->edge_dst[e] == s) { a = P->edge_src[e]; table = T_FWD; }
        if (kind == K_B && P->edge_src[e] == s) { a = P->edge_dst[e]; table = T_BWD; }
        if (a < 0) continue;
        const int64_t r = wait_for(P, fin, table, a, s, g, P->stage_device[a] != d ? P->edge_comm[e] : 0);
        if (r < 0) blocked = 1;
        else if (r > ready) ready = r;
      }
      for (int i = 0; i < P->n_pairs && !blocked; ++i) {
        const int32_t *q = P->pairs + 5 * i;
        const int to_kind = q[2];
        if (q[3] != s || !(to_kind == kind || (to_kind == K_F && kind == K_FD))) continue;
        const int table = q[0] == K_F ? T_FWD : (q[0] == K_B ? T_BWD : T_WGT);
        const int64_t r = wait_for(P, fin, table, q[1], s, g, P->stage_device[q[1]] != d ? q[4] : 0);
        if (r < 0) blocked = 1;
        else if (r > ready) ready = r;
      }
      if (blocked) continue;
      /* issue */
      const int64_t dt = P->dur[kind * S + s], u = P->mem_units[s];
      const int64_t start = free_at[d] > ready ? free_at[d] : ready;
      const int64_t finish = start + dt;
      if (kind == K_F || kind == K_FD || kind == K_R || kind == K_L) {
        mem[d] += u;
        if (mem[d] > pk[d]) pk[d] = mem[d];
      }
      if (kind == K_FD || kind == K_O || kind == K_W || (kind == K_B && !P->has_w)) mem[d] -= u;
      *st = (uint8_t)next;
      if (kind == K_F || kind == K_FD) fin[((size_t)T_FWD * S + s) * m + g] = finish;
      if (kind == K_B) fin[((size_t)T_BWD * S + s) * m + g] = finish;
      if (kind == K_W) fin[((size_t)T_WGT * S + s) * m + g] = finish;
      if (op_start) {
        op_start[(size_t)d * stride + cursor[d]] = start;
        op_finish[(size_t)d * stride + cursor[d]] = finish;
      }
      free_at[d] = finish;
      busy[d] += dt;
      cursor[d] += 1;
      issued_any = 1;
    }
    if (!issued_any) break;
  }

  uint8_t fl = 0;
  for (int d = 0; d < D; ++d) if (cursor[d] < len[d]) fl |= FLAG_DEADLOCK;
  if (fl && malformed_head) fl |= FLAG_INCOMPLETE;
  if (!fl) {
    const int terminal = P->has_w ? ST_DONE : ST_BDONE;
    for (int s = 0; s < S; ++s)
      for (int g = 0; g < items_of(P, s); ++g)
        if (state[(size_t)s * m + g] != terminal) fl |= FLAG_INCOMPLETE;
  }
  if (fl) {
    *makespan = INT64_MAX;
    for (int d = 0; d < D; ++d) { idle[d] = -1; peak[d] = -1; }
  } else {
    int64_t ms = 0;
    for (int d = 0; d < D; ++d) if (free_at[d] > ms) ms = free_at[d];
    *makespan = ms;
    for (int d = 0; d < D; ++d) {
      idle[d] = ms - busy[d];
      peak[d] = (int32_t)pk[d];
      if (pk[d] > P->mem_cap[d]) fl |= FLAG_OVER_CAP;
    }
  }
  *flags = fl;
  free(fin); free(state); free(cursor); free(len); free(free_at); free(busy); free(mem); free(pk);
  return 0;
}

/* Candidates [0, n_cand) of a batch laid out [C][D][stride]. */
int fpsync_evaluate(const fpsync_problem *P, const uint16_t *words, int64_t n_cand, int32_t stride,
                    int64_t *makespan, int64_t *idle, int32_t *peak, uint8_t *flags) {
  const int D = P->n_devices;
  for (int64_t c = 0; c < n_cand; ++c) {
    const int rc = fpsync_eval_one(P, words + (size_t)c * D * stride, stride, &makespan[c], &idle[c * D],
                                   &peak[c * D], &flags[c], NULL, NULL);
    if (rc) return rc;
  }
  return 0;
}

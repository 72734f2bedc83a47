/*
 * fporacle.c -- CPU oracle for batched pipeline-schedule evaluation.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, single-threaded
 * definition that the GPU library is checked against.  Nothing in the product
 * path may call it; it shares no code, header, table or helper with the HIP
 * sources.  Times are int64 throughout.
 *
 * What is evaluated (paper, Section 3 "Overview", the auto-tuner paragraph:
 * the offline tuner picks the most suitable schedule out of the enumerated
 * ones; Section 7.1: the winners are the schedules whose bubble ratio is lowest;
 * the estimator sketch that follows Section 6: a schedule becomes an
 * execution graph of tasks labelled with start time, end time and cost):
 *
 *   A schedule is, per device ("actor"), a sequence of instructions (Section 4,
 *   "FlexPipe's Instructions"); an instruction item is (type, micro-batch,
 *   stage) (Section 5.1, "Instruction Item").  Forward items depend on the
 *   forward items of the predecessor stages in the stage DAG, backward items
 *   on the backward items of the successor stages (Section 5.1, "Data
 *   dependency").  Each device executes its list strictly in order, one item
 *   at a time.  An item starts as soon as its device is free and all its
 *   dependencies have finished (plus the edge's communication latency when
 *   the two stages sit on different devices) and runs for the profiled cost
 *   of its (type, stage).
 *
 * Readings of points the paper leaves open:
 *   - evaluation is time-based on integer times; all devices are free at 0;
 *   - communication is a pure latency on cross-device DAG edges, the same
 *     value for activations and gradients;
 *   - same-device ordering rules are a per-(stage, micro-batch) activation
 *     state machine:  ABSENT -F-> RES,  ABSENT -FD-> DISC,  DISC -R-> RES,
 *     RES -O-> OFF,  OFF -L-> RES,  RES -B-> BDONE,  BDONE -W-> DONE;
 *     an item whose (stage, micro-batch) is not in the required source state
 *     cannot issue (and, its device being stuck behind it, never will);
 *   - activation memory: +units at the START of F, FD, R, L; -units at the END
 *     of FD and O; -units at the end of W (split backward) or of B (has_w=0);
 *   - idle[d] = makespan - (sum of durations of the items on d): head, middle
 *     and tail waiting all count (Section 2, bubbles = device idle time;
 *     Section 7.1 breakdown, device waiting time);
 *   - ranking key is (makespan ascending, candidate index ascending): total
 *     work is fixed per problem, so least bubble ratio == least makespan.
 *
 * Layout of this file: eval_one is the definition above and nothing else.  The two variants of the
 * cost model (costs per micro-batch, link occupancy) are a loop of their own further down,
 * eval_one_variants, which repeats the definition with the two switches; with both off it must give
 * what eval_one gives, and the tests compare the two loops.
 *
 * Parity pins (tests/, -m "not gpu"): GPipe and 1F1B closed forms, an
 * independent longest-path + Kahn checker, brute force over all order pairs
 * for p=2, m<=3, order-only memory scan, monotonicity, and the input
 * generator's own list-scheduling clock.  Parity UNPINNED by the paper: the
 * R / O / L / FD semantics and the sentinel values (the paper names neither);
 * they are pinned only by the independent checker and the invariants.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { K_END = 0, K_F = 1, K_B = 2, K_W = 3, K_R = 4, K_O = 5, K_L = 6, K_FD = 7, NKINDS = 8 };
enum { ST_ABSENT = 0, ST_RES = 1, ST_DISC = 2, ST_OFF = 3, ST_BDONE = 4, ST_DONE = 5 };
enum { FLAG_DEADLOCK = 1, FLAG_INCOMPLETE = 2, FLAG_OVER_CAP = 4 };
#define MAX_CHUNKS 4

typedef struct {
  int32_t n_devices;       /* D */
  int32_t n_stages;        /* S */
  int32_t n_microbatches;  /* m */
  int32_t has_w;           /* 1: B then W, W frees; 0: B frees, W illegal */
  const int32_t *stage_device; /* [S] */
  int32_t n_edges;
  const int32_t *edge_src;  /* [E] */
  const int32_t *edge_dst;  /* [E] */
  const int32_t *edge_comm; /* [E] */
  const int32_t *dur;       /* [NKINDS][S] */
  const int32_t *mem_units; /* [S] */
  const int32_t *mem_cap;   /* [D] */
} fporacle_problem;

/* Word layout (unsigned 16 bit): kind in bits 15..13, the device-local chunk
 * in bits 12..11, the micro-batch in bits 10..0.  The all-zero kind ends a
 * device's list. */
static int word_kind(uint16_t w) { return w >> 13; }
static int word_chunk(uint16_t w) { return (w >> 11) & 3; }
static int word_mb(uint16_t w) { return w & 0x7ff; }

void fporacle_decode(const uint16_t *words, int64_t n, int32_t *kind, int32_t *chunk, int32_t *mb) {
  for (int64_t i = 0; i < n; ++i) {
    kind[i] = word_kind(words[i]);
    chunk[i] = word_chunk(words[i]);
    mb[i] = word_mb(words[i]);
  }
}

/* chunk c of device d = the c-th of d's stages in ascending stage id. */
static int build_local_stage(const fporacle_problem *P, int32_t *local_stage, int32_t *n_chunks) {
  for (int d = 0; d < P->n_devices; ++d) n_chunks[d] = 0;
  for (int s = 0; s < P->n_stages; ++s) {
    int d = P->stage_device[s];
    if (d < 0 || d >= P->n_devices) return -1;
    if (n_chunks[d] >= MAX_CHUNKS) return -1;
    local_stage[d * MAX_CHUNKS + n_chunks[d]++] = s;
  }
  return 0;
}

/*
 * Evaluate one candidate.  words: [D][stride].  Outputs: makespan, idle[D],
 * peak[D], flags; optional per-op traces op_start/op_finish [D][stride]
 * (-1 where the op never issued or past the end of the list).
 * Returns 0, or -1 for an invalid problem.
 */
static int eval_one(const fporacle_problem *P, const uint16_t *words, int32_t stride,
                    int64_t *makespan, int64_t *idle, int32_t *peak, uint8_t *flags,
                    int64_t *op_start, int64_t *op_finish) {
  const int D = P->n_devices, S = P->n_stages, m = P->n_microbatches;
  int32_t *local_stage = malloc(sizeof(int32_t) * D * MAX_CHUNKS);
  int32_t *n_chunks = malloc(sizeof(int32_t) * D);
  if (build_local_stage(P, local_stage, n_chunks)) { free(local_stage); free(n_chunks); return -1; }

  int64_t *fin_fwd = malloc(sizeof(int64_t) * S * m);   /* finish of F/FD(s,j), -1 = not yet */
  int64_t *fin_bwd = malloc(sizeof(int64_t) * S * m);   /* finish of B(s,j) */
  uint8_t *state = calloc((size_t)S * m, 1);
  int32_t *cursor = calloc(D, sizeof(int32_t));
  int32_t *len = calloc(D, sizeof(int32_t));
  int64_t *free_at = calloc(D, sizeof(int64_t));
  int64_t *busy = calloc(D, sizeof(int64_t));
  int64_t *mem = calloc(D, sizeof(int64_t));
  int64_t *pk = calloc(D, sizeof(int64_t));
  for (int i = 0; i < S * m; ++i) fin_fwd[i] = fin_bwd[i] = -1;
  for (int d = 0; d < D; ++d) {
    int n = 0;
    while (n < stride && word_kind(words[(size_t)d * stride + n]) != K_END) ++n;
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
      const int kind = word_kind(w), c = word_chunk(w), j = word_mb(w);
      if (c >= n_chunks[d] || j >= m || (kind == K_W && !P->has_w)) { malformed_head = 1; continue; }
      const int s = local_stage[d * MAX_CHUNKS + c];
      uint8_t *st = &state[(size_t)s * m + j];

      /* same-device rule: required source state */
      int need;
      switch (kind) {
        case K_F: case K_FD: need = ST_ABSENT; break;
        case K_R: need = ST_DISC; break;
        case K_O: need = ST_RES; break;
        case K_L: need = ST_OFF; break;
        case K_B: need = ST_RES; break;
        default:  need = ST_BDONE; break; /* K_W */
      }
      if (*st != need) continue;

      /* cross-stage rule */
      int64_t ready = 0;
      int blocked = 0;
      if (kind == K_F || kind == K_FD) {
        for (int e = 0; e < P->n_edges && !blocked; ++e) {
          if (P->edge_dst[e] != s) continue;
          const int sp = P->edge_src[e];
          const int64_t t = fin_fwd[(size_t)sp * m + j];
          if (t < 0) { blocked = 1; break; }
          const int64_t r = t + (P->stage_device[sp] != d ? P->edge_comm[e] : 0);
          if (r > ready) ready = r;
        }
      } else if (kind == K_B) {
        for (int e = 0; e < P->n_edges && !blocked; ++e) {
          if (P->edge_src[e] != s) continue;
          const int sn = P->edge_dst[e];
          const int64_t t = fin_bwd[(size_t)sn * m + j];
          if (t < 0) { blocked = 1; break; }
          const int64_t r = t + (P->stage_device[sn] != d ? P->edge_comm[e] : 0);
          if (r > ready) ready = r;
        }
      }
      if (blocked) continue;

      /* issue */
      const int64_t dt = P->dur[kind * S + s];
      const int64_t u = P->mem_units[s];
      const int64_t start = free_at[d] > ready ? free_at[d] : ready;
      const int64_t finish = start + dt;
      if (kind == K_F || kind == K_FD || kind == K_R || kind == K_L) {
        mem[d] += u;
        if (mem[d] > pk[d]) pk[d] = mem[d];
      }
      if (kind == K_FD || kind == K_O) mem[d] -= u;
      if (kind == K_W || (kind == K_B && !P->has_w)) mem[d] -= u;
      switch (kind) {
        case K_F:  *st = ST_RES;  fin_fwd[(size_t)s * m + j] = finish; break;
        case K_FD: *st = ST_DISC; fin_fwd[(size_t)s * m + j] = finish; break;
        case K_R:  *st = ST_RES; break;
        case K_O:  *st = ST_OFF; break;
        case K_L:  *st = ST_RES; break;
        case K_B:  *st = ST_BDONE; fin_bwd[(size_t)s * m + j] = finish; break;
        default:   *st = ST_DONE; break;
      }
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
    for (int i = 0; i < S * m; ++i) if (state[i] != terminal) { fl |= FLAG_INCOMPLETE; break; }
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

  free(local_stage); free(n_chunks); free(fin_fwd); free(fin_bwd); free(state);
  free(cursor); free(len); free(free_at); free(busy); free(mem); free(pk);
  return 0;
}

int fporacle_eval_one(const fporacle_problem *P, const uint16_t *words, int32_t stride,
                      int64_t *makespan, int64_t *idle, int32_t *peak, uint8_t *flags,
                      int64_t *op_start, int64_t *op_finish) {
  return eval_one(P, words, stride, makespan, idle, peak, flags, op_start, op_finish);
}

/*
 * The variants of the cost model (costs per micro-batch, link occupancy; see the entry points below),
 * as a loop of their own: the plain definition above, written out again with the two switches.  With
 * dur_mb == NULL and links == 0 it must give what eval_one gives (tests/test_oracle_mbdur.py,
 * tests/test_oracle_links.py compare the two loops).
 */
static int eval_one_variants(const fporacle_problem *P, const int32_t *dur_mb, int links, const uint16_t *words, int32_t stride,
                    int64_t *makespan, int64_t *idle, int32_t *peak, uint8_t *flags,
                    int64_t *op_start, int64_t *op_finish) {
  const int D = P->n_devices, S = P->n_stages, m = P->n_microbatches, E = P->n_edges;
  /* links != 0 (see fporacle_evaluate_links): when each value sent over a cross-device edge arrives,
   * per edge and micro-batch (-1 = not sent yet), and until when each device-to-device link is busy */
  int64_t *arr_fwd = NULL, *arr_bwd = NULL, *link_free = NULL;
  if (links) {
    arr_fwd = malloc(sizeof(int64_t) * (size_t)(E > 0 ? E : 1) * m);
    arr_bwd = malloc(sizeof(int64_t) * (size_t)(E > 0 ? E : 1) * m);
    link_free = calloc((size_t)D * D, sizeof(int64_t));
    for (int64_t i = 0; i < (int64_t)E * m; ++i) arr_fwd[i] = arr_bwd[i] = -1;
  }
  int32_t *local_stage = malloc(sizeof(int32_t) * D * MAX_CHUNKS);
  int32_t *n_chunks = malloc(sizeof(int32_t) * D);
  if (build_local_stage(P, local_stage, n_chunks)) { free(local_stage); free(n_chunks); return -1; }

  int64_t *fin_fwd = malloc(sizeof(int64_t) * S * m);   /* finish of F/FD(s,j), -1 = not yet */
  int64_t *fin_bwd = malloc(sizeof(int64_t) * S * m);   /* finish of B(s,j) */
  uint8_t *state = calloc((size_t)S * m, 1);
  int32_t *cursor = calloc(D, sizeof(int32_t));
  int32_t *len = calloc(D, sizeof(int32_t));
  int64_t *free_at = calloc(D, sizeof(int64_t));
  int64_t *busy = calloc(D, sizeof(int64_t));
  int64_t *mem = calloc(D, sizeof(int64_t));
  int64_t *pk = calloc(D, sizeof(int64_t));
  for (int i = 0; i < S * m; ++i) fin_fwd[i] = fin_bwd[i] = -1;
  for (int d = 0; d < D; ++d) {
    int n = 0;
    while (n < stride && word_kind(words[(size_t)d * stride + n]) != K_END) ++n;
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
      const int kind = word_kind(w), c = word_chunk(w), j = word_mb(w);
      if (c >= n_chunks[d] || j >= m || (kind == K_W && !P->has_w)) { malformed_head = 1; continue; }
      const int s = local_stage[d * MAX_CHUNKS + c];
      uint8_t *st = &state[(size_t)s * m + j];

      /* same-device rule: required source state */
      int need;
      switch (kind) {
        case K_F: case K_FD: need = ST_ABSENT; break;
        case K_R: need = ST_DISC; break;
        case K_O: need = ST_RES; break;
        case K_L: need = ST_OFF; break;
        case K_B: need = ST_RES; break;
        default:  need = ST_BDONE; break; /* K_W */
      }
      if (*st != need) continue;

      /* cross-stage rule */
      int64_t ready = 0;
      int blocked = 0;
      if (kind == K_F || kind == K_FD) {
        for (int e = 0; e < P->n_edges && !blocked; ++e) {
          if (P->edge_dst[e] != s) continue;
          const int sp = P->edge_src[e];
          const int64_t t = links ? arr_fwd[(size_t)e * m + j] : fin_fwd[(size_t)sp * m + j];
          if (t < 0) { blocked = 1; break; }
          const int64_t r = links ? t : t + (P->stage_device[sp] != d ? P->edge_comm[e] : 0);
          if (r > ready) ready = r;
        }
      } else if (kind == K_B) {
        for (int e = 0; e < P->n_edges && !blocked; ++e) {
          if (P->edge_src[e] != s) continue;
          const int sn = P->edge_dst[e];
          const int64_t t = links ? arr_bwd[(size_t)e * m + j] : fin_bwd[(size_t)sn * m + j];
          if (t < 0) { blocked = 1; break; }
          const int64_t r = links ? t : t + (P->stage_device[sn] != d ? P->edge_comm[e] : 0);
          if (r > ready) ready = r;
        }
      }
      if (blocked) continue;

      /* issue */
      /* cost of the item: per (type, stage), or per (type, stage, micro-batch) if such a table is given */
      const int64_t dt = dur_mb ? dur_mb[((size_t)kind * S + s) * m + j] : P->dur[kind * S + s];
      const int64_t u = P->mem_units[s];
      const int64_t start = free_at[d] > ready ? free_at[d] : ready;
      const int64_t finish = start + dt;
      if (kind == K_F || kind == K_FD || kind == K_R || kind == K_L) {
        mem[d] += u;
        if (mem[d] > pk[d]) pk[d] = mem[d];
      }
      if (kind == K_FD || kind == K_O) mem[d] -= u;
      if (kind == K_W || (kind == K_B && !P->has_w)) mem[d] -= u;
      switch (kind) {
        case K_F:  *st = ST_RES;  fin_fwd[(size_t)s * m + j] = finish; break;
        case K_FD: *st = ST_DISC; fin_fwd[(size_t)s * m + j] = finish; break;
        case K_R:  *st = ST_RES; break;
        case K_O:  *st = ST_OFF; break;
        case K_L:  *st = ST_RES; break;
        case K_B:  *st = ST_BDONE; fin_bwd[(size_t)s * m + j] = finish; break;
        default:   *st = ST_DONE; break;
      }
      if (links && (kind == K_F || kind == K_FD || kind == K_B)) {
        /* send the result over every outgoing edge, in the order of the edge list: activations to the
         * successor stages, gradients to the predecessor stages.  A transfer starts when the item has
         * finished and the link from this device to the receiving one is free, and keeps the link busy for
         * the edge's latency; on the same device the value is there at once. */
        const int fwd = kind != K_B;
        for (int e = 0; e < E; ++e) {
          if ((fwd ? P->edge_src[e] : P->edge_dst[e]) != s) continue;
          const int to = P->stage_device[fwd ? P->edge_dst[e] : P->edge_src[e]];
          int64_t arrival = finish;
          if (to != d) {
            int64_t *busy_until = &link_free[(size_t)d * D + to];
            const int64_t depart = finish > *busy_until ? finish : *busy_until;
            arrival = depart + P->edge_comm[e];
            *busy_until = arrival;
          }
          (fwd ? arr_fwd : arr_bwd)[(size_t)e * m + j] = arrival;
        }
      }
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
    for (int i = 0; i < S * m; ++i) if (state[i] != terminal) { fl |= FLAG_INCOMPLETE; break; }
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

  free(arr_fwd); free(arr_bwd); free(link_free);
  free(local_stage); free(n_chunks); free(fin_fwd); free(fin_bwd); free(state);
  free(cursor); free(len); free(free_at); free(busy); free(mem); free(pk);
  return 0;
}


/*
 * Variant of the cost model: micro-batches of unequal size.  The paper profiles one cost per
 * (type, stage) (estimator sketch after Section 6); its related-work section (Section 8,
 * "Frameworks") names dynamic micro-batching, where the micro-batches of one iteration differ in
 * length and so in cost.  dur_mb[NKINDS][S][m] then replaces dur[NKINDS][S] in the start rule
 * (finish = start + dur_mb[type][stage][micro-batch]) and in the busy time; nothing else changes.
 * Pins: tests/test_oracle_mbdur.py (proportionate flow shop closed form, a timeline worked by hand,
 * the critical-path checker with per-item weights, a constant table against the plain model).
 */
int fporacle_eval_one_mb(const fporacle_problem *P, const int32_t *dur_mb, const uint16_t *words,
                         int32_t stride, int64_t *makespan, int64_t *idle, int32_t *peak, uint8_t *flags,
                         int64_t *op_start, int64_t *op_finish) {
  return eval_one_variants(P, dur_mb, 0, words, stride, makespan, idle, peak, flags, op_start, op_finish);
}

/* Evaluate candidates [0, n_cand) of a batch laid out [C][D][stride]; dur_mb may be NULL. */
int fporacle_evaluate_mb(const fporacle_problem *P, const int32_t *dur_mb, const uint16_t *words,
                         int64_t n_cand, int32_t stride, int64_t *makespan, int64_t *idle, int32_t *peak,
                         uint8_t *flags) {
  const int D = P->n_devices;
  for (int64_t c = 0; c < n_cand; ++c) {
    int rc = eval_one_variants(P, dur_mb, 0, words + (size_t)c * D * stride, stride, &makespan[c],
                      &idle[c * D], &peak[c * D], &flags[c], NULL, NULL);
    if (rc) return rc;
  }
  return 0;
}

/*
 * Variant of the cost model: links that carry one value at a time.  The paper lists P2P send / receive
 * among its instructions (Section 4, "FlexPipe's Instructions") and leaves out how they are overlapped
 * (Section 5.2, end); the plain model above reads a transfer as a pure latency.  Here every ordered pair
 * of devices (from, to) is a link of its own: a value (the activation of a forward item for a successor
 * stage on another device, the gradient of a backward item for a predecessor stage on another device)
 * leaves when its item has finished and the link is free, occupies the link for the edge's latency and
 * arrives at its end.  Values of one device leave in the order its items run (several values of one item:
 * in the order of the edge list).  A consumer is ready when all its inputs have arrived.  Everything else
 * (order rules, memory, idle, flags) is as in the plain model; with latencies of zero the two coincide.
 * Pins: tests/test_oracle_links.py.
 */
int fporacle_eval_one_links(const fporacle_problem *P, const int32_t *dur_mb, const uint16_t *words, int32_t stride,
                            int64_t *makespan, int64_t *idle, int32_t *peak, uint8_t *flags, int64_t *op_start,
                            int64_t *op_finish) {
  return eval_one_variants(P, dur_mb, 1, words, stride, makespan, idle, peak, flags, op_start, op_finish);
}

/* dur_mb: NULL, or costs per micro-batch as in fporacle_evaluate_mb (the two variants are independent: one
 * says what an item costs, the other when its result arrives). */
int fporacle_evaluate_links(const fporacle_problem *P, const int32_t *dur_mb, const uint16_t *words, int64_t n_cand,
                            int32_t stride, int64_t *makespan, int64_t *idle, int32_t *peak, uint8_t *flags) {
  const int D = P->n_devices;
  for (int64_t c = 0; c < n_cand; ++c) {
    int rc = eval_one_variants(P, dur_mb, 1, words + (size_t)c * D * stride, stride, &makespan[c],
                      &idle[c * D], &peak[c * D], &flags[c], NULL, NULL);
    if (rc) return rc;
  }
  return 0;
}

/* The plain model: candidates [0, n_cand) of a batch laid out [C][D][stride], each by eval_one. */
int fporacle_evaluate(const fporacle_problem *P, const uint16_t *words, int64_t n_cand, int32_t stride,
                      int64_t *makespan, int64_t *idle, int32_t *peak, uint8_t *flags) {
  const int D = P->n_devices;
  for (int64_t c = 0; c < n_cand; ++c) {
    int rc = eval_one(P, words + (size_t)c * D * stride, stride, &makespan[c], &idle[c * D], &peak[c * D],
                      &flags[c], NULL, NULL);
    if (rc) return rc;
  }
  return 0;
}

typedef struct { int64_t makespan, idx; } rank_key;
static int rank_cmp(const void *a, const void *b) {
  const rank_key *x = a, *y = b;
  if (x->makespan != y->makespan) return x->makespan < y->makespan ? -1 : 1;
  if (x->idx != y->idx) return x->idx < y->idx ? -1 : 1;
  return 0;
}

/* Top-k: feasible = flags == 0; ascending (makespan, index); unused slots get
 * idx -1 and makespan INT64_MAX; *count = min(k, #feasible). */
int fporacle_topk(const int64_t *makespan, const uint8_t *flags, int64_t n_cand, int32_t k,
                  int64_t *out_idx, int64_t *out_makespan, int32_t *count) {
  rank_key *keys = malloc(sizeof(rank_key) * (n_cand > 0 ? n_cand : 1));
  int64_t n = 0;
  for (int64_t c = 0; c < n_cand; ++c)
    if (flags[c] == 0) { keys[n].makespan = makespan[c]; keys[n].idx = c; ++n; }
  qsort(keys, n, sizeof(rank_key), rank_cmp);
  for (int32_t i = 0; i < k; ++i) {
    if (i < n) { out_idx[i] = keys[i].idx; out_makespan[i] = keys[i].makespan; }
    else { out_idx[i] = -1; out_makespan[i] = INT64_MAX; }
  }
  *count = (int32_t)(n < k ? n : k);
  free(keys);
  return 0;
}

/* Ranking by a two-part key (an extension of the paper's ranking by bubble ratio, Section 7.1,
 * by the memory footprint, Section 2): mode 0 (makespan), 1 (makespan, largest peak), 2 (largest
 * peak, makespan), 3 (sum of idle).  Failed candidates never rank; over-cap ones only if
 * include_over_cap.  Ties by candidate index.  out_k1/out_k2: the key parts of the winners
 * (k2 = 0 where the mode has one part); unused slots idx -1, parts INT64_MAX. */
typedef struct { int64_t k1, k2, idx; } rank3_key;
static int rank3_cmp(const void *a, const void *b) {
  const rank3_key *x = a, *y = b;
  if (x->k1 != y->k1) return x->k1 < y->k1 ? -1 : 1;
  if (x->k2 != y->k2) return x->k2 < y->k2 ? -1 : 1;
  if (x->idx != y->idx) return x->idx < y->idx ? -1 : 1;
  return 0;
}

int fporacle_rank(const int64_t *makespan, const int64_t *idle, const int32_t *peak, const uint8_t *flags,
                  int64_t n_cand, int32_t n_devices, int32_t k, int32_t mode, int32_t include_over_cap,
                  int64_t *out_idx, int64_t *out_k1, int64_t *out_k2, int32_t *count) {
  if (mode < 0 || mode > 3) return -1;
  rank3_key *keys = malloc(sizeof(rank3_key) * (n_cand > 0 ? n_cand : 1));
  int64_t n = 0;
  for (int64_t c = 0; c < n_cand; ++c) {
    if (flags[c] & (FLAG_DEADLOCK | FLAG_INCOMPLETE)) continue;
    if ((flags[c] & FLAG_OVER_CAP) && !include_over_cap) continue;
    int64_t max_peak = 0, sum_idle = 0;
    for (int d = 0; d < n_devices; ++d) {
      if (peak[c * n_devices + d] > max_peak) max_peak = peak[c * n_devices + d];
      sum_idle += idle[c * n_devices + d];
    }
    keys[n].idx = c;
    keys[n].k1 = mode == 0 || mode == 1 ? makespan[c] : (mode == 2 ? max_peak : sum_idle);
    keys[n].k2 = mode == 1 ? max_peak : (mode == 2 ? makespan[c] : 0);
    ++n;
  }
  qsort(keys, n, sizeof(rank3_key), rank3_cmp);
  for (int32_t i = 0; i < k; ++i) {
    if (i < n) { out_idx[i] = keys[i].idx; out_k1[i] = keys[i].k1; out_k2[i] = keys[i].k2; }
    else { out_idx[i] = -1; out_k1[i] = INT64_MAX; out_k2[i] = INT64_MAX; }
  }
  *count = (int32_t)(n < k ? n : k);
  free(keys);
  return 0;
}

/* Pareto front of (makespan, largest peak[d]) over the candidates that completed (neither
 * DEADLOCK nor INCOMPLETE; the cap plays no part: the front replaces a hard cap by the whole
 * trade-off between the two properties a schedule has in the paper, bubble ratio (Section 7.1)
 * and memory footprint (Section 2)).  Written as the definition: candidate c is on the front
 * iff no other completed candidate is at most as large in both values and smaller in one, and
 * no completed candidate with a smaller index has the same pair.  Quadratic on purpose.
 * The front is returned by ascending makespan (hence descending peak), at most kmax entries;
 * *count = number of entries written; unused slots idx -1, makespan INT64_MAX, peak -1. */
typedef struct { int64_t ms, pk, idx; } front_pt;
static int front_cmp(const void *a, const void *b) {
  const front_pt *x = a, *y = b;
  if (x->ms != y->ms) return x->ms < y->ms ? -1 : 1;
  return 0;
}

int fporacle_pareto(const int64_t *makespan, const int32_t *peak, const uint8_t *flags, int64_t n_cand,
                    int32_t n_devices, int32_t kmax, int64_t *out_idx, int64_t *out_makespan,
                    int32_t *out_peak, int32_t *count) {
  int64_t *mp = malloc(sizeof(int64_t) * (n_cand > 0 ? n_cand : 1));
  front_pt *front = malloc(sizeof(front_pt) * (n_cand > 0 ? n_cand : 1));
  for (int64_t c = 0; c < n_cand; ++c) {
    mp[c] = 0;
    for (int d = 0; d < n_devices; ++d)
      if (peak[c * n_devices + d] > mp[c]) mp[c] = peak[c * n_devices + d];
  }
  int64_t nf = 0;
  for (int64_t c = 0; c < n_cand; ++c) {
    if (flags[c] & (FLAG_DEADLOCK | FLAG_INCOMPLETE)) continue;
    int on_front = 1;
    for (int64_t o = 0; o < n_cand && on_front; ++o) {
      if (o == c || (flags[o] & (FLAG_DEADLOCK | FLAG_INCOMPLETE))) continue;
      const int no_worse = makespan[o] <= makespan[c] && mp[o] <= mp[c];
      const int better = makespan[o] < makespan[c] || mp[o] < mp[c];
      if (no_worse && (better || o < c)) on_front = 0;
    }
    if (on_front) { front[nf].ms = makespan[c]; front[nf].pk = mp[c]; front[nf].idx = c; ++nf; }
  }
  qsort(front, nf, sizeof(front_pt), front_cmp);   /* makespans on the front are distinct */
  for (int32_t i = 0; i < kmax; ++i) {
    if (i < nf) { out_idx[i] = front[i].idx; out_makespan[i] = front[i].ms; out_peak[i] = (int32_t)front[i].pk; }
    else { out_idx[i] = -1; out_makespan[i] = INT64_MAX; out_peak[i] = -1; }
  }
  *count = (int32_t)(nf < kmax ? nf : kmax);
  free(mp);
  free(front);
  return 0;
}

/* OVER_CAP recomputed from the peaks for other memory caps than the problem's (the same
 * schedules judged for devices with less or more memory: Section 2, memory footprint against
 * device capacity).  caps: [n_devices] when per_candidate == 0, else [n_cand][n_devices].
 * The other flag bits are kept; a failed candidate (DEADLOCK or INCOMPLETE: no peaks) never gets OVER_CAP. */
int fporacle_apply_caps(const int32_t *peak, const int32_t *caps, int32_t per_candidate, int64_t n_cand,
                        int32_t n_devices, uint8_t *flags) {
  for (int64_t c = 0; c < n_cand; ++c) {
    int over = 0;
    for (int d = 0; d < n_devices; ++d) {
      const int32_t cap = per_candidate ? caps[c * n_devices + d] : caps[d];
      if (peak[c * n_devices + d] > cap) over = 1;
    }
    flags[c] = (uint8_t)((flags[c] & ~FLAG_OVER_CAP) | (over && !(flags[c] & (FLAG_DEADLOCK | FLAG_INCOMPLETE)) ? FLAG_OVER_CAP : 0));
  }
  return 0;
}

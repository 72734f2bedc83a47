/*
 * fpcopyoracle.c -- CPU oracle of schedule evaluation with a copy engine for offload and reload items.
 *
 * TEST INFRASTRUCTURE ONLY.  A plain, slow, single-threaded event loop in int64; a file of its own that
 * shares no code with the other oracles, with the HIP sources or with the input generators.  Nothing in
 * the product path may call it.
 *
 * The paper names CPU offloading among the memory optimisations of pipeline schedules and among the
 * frameworks it relates to (Section 8) and says nothing about how an offload is timed.  The plain model
 * (fporacle.c) runs offload (O) and reload (L) items on the device's compute timeline like any other
 * item.  This file is the other reading: transfers run on a copy engine beside the computation.
 *
 *   C1  every device has a compute timeline and a copy timeline.  O and L items run on the copy
 *       timeline, all other kinds on the compute timeline; each timeline is serial and keeps the order
 *       of the device's list.
 *   C2  the device walks its list.  A compute item holds the walk until it has finished (as in the
 *       plain model).  A copy item is handed to the copy engine when the walk reaches it -- every
 *       compute item in front of it has finished -- and the walk goes on at once.  The engine holds at
 *       most `depth` transfers, running or waiting: a walk that reaches a copy item while `depth` are
 *       unfinished waits until the oldest of them has finished.
 *   C3  a copy item starts at max(hand-over time, finish of the copy item before it) and runs for
 *       dur[kind][stage].
 *   C4  the activation state machine follows the list order as before (a copy item changes the state
 *       when it is handed over).  A backward item whose activation was reloaded starts no earlier than
 *       the finish of that reload.  Everything a copy item needs is there when it is handed over: the
 *       forward or recompute item in front of an offload has finished, an offload in front of a reload
 *       precedes it on the copy timeline.
 *   C5  memory: +units at the start of F, FD, R and L, -units at the end of FD, O and W (B without split
 *       backward), now at the TIMES these happen: the peak is the largest running sum over all events of
 *       the device in time order; at equal times the compute timeline's events come first, and each
 *       timeline's events keep their own order.
 *   C6  makespan = the latest finish on either timeline; idle[d] = makespan - the costs of d's compute
 *       items (transfers do not keep the compute units busy).  Dependencies across stages, flags and
 *       sentinels are those of the plain model.
 *
 * Pins (tests/test_oracle_copy.py): lists without O and L items against the plain oracle; a timeline
 * worked out by hand; every finish time at most the plain model's; an independent checker
 * (tests/copy_checker.py: topological order + recurrences, events sorted by key) on random candidates;
 * depth 1 with a closed form.  Parity UNPINNED by the paper: C1-C6 are this build's reading.
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
} fpcopy_problem;

typedef struct { int64_t time, delta; } mem_event;

/* One candidate.  words: [D][stride]; depth >= 1: transfers the copy engine holds at most.
 * Returns 0, or -1 for an invalid description. */
int fpcopy_eval_one(const fpcopy_problem *P, int32_t depth, const uint16_t *words, int32_t stride,
                    int64_t *makespan, int64_t *idle, int32_t *peak, uint8_t *flags,
                    int64_t *op_start, int64_t *op_finish) {
  const int D = P->n_devices, S = P->n_stages, m = P->n_microbatches, E = P->n_edges;
  if (D < 1 || D > 64 || S < 1 || m < 1 || depth < 1) return -1;
  int32_t local_stage[64 * MAX_CHUNKS], n_chunks[64];
  for (int d = 0; d < D; ++d) n_chunks[d] = 0;
  for (int s = 0; s < S; ++s) {
    const int d = P->stage_device[s];
    if (d < 0 || d >= D || n_chunks[d] >= MAX_CHUNKS) return -1;
    local_stage[d * MAX_CHUNKS + n_chunks[d]++] = s;
  }
  int64_t *fin_fwd = malloc(sizeof(int64_t) * (size_t)S * m), *fin_bwd = malloc(sizeof(int64_t) * (size_t)S * m);
  int64_t *resident_at = calloc((size_t)S * m, sizeof(int64_t));   /* finish of the last reload, else 0 */
  uint8_t *state = calloc((size_t)S * m, 1);
  int32_t *cursor = calloc(D, sizeof(int32_t)), *len = calloc(D, sizeof(int32_t));
  int64_t *free_at = calloc(D, sizeof(int64_t)), *copy_free = calloc(D, sizeof(int64_t));
  int64_t *busy = calloc(D, sizeof(int64_t));
  /* per device: finish of every copy item in hand-over order; the memory events of either timeline */
  int64_t *copy_fin = malloc(sizeof(int64_t) * (size_t)D * (stride > 0 ? stride : 1));
  int32_t *n_copy = calloc(D, sizeof(int32_t));
  mem_event *ev_compute = malloc(sizeof(mem_event) * 2 * (size_t)D * (stride > 0 ? stride : 1));
  mem_event *ev_copy = malloc(sizeof(mem_event) * (size_t)D * (stride > 0 ? stride : 1));
  int32_t *n_ev_compute = calloc(D, sizeof(int32_t)), *n_ev_copy = calloc(D, sizeof(int32_t));
  for (int i = 0; i < S * m; ++i) fin_fwd[i] = fin_bwd[i] = -1;
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
      const int kind = w >> 13, c = (w >> 11) & 3, j = w & 0x7ff;
      if (c >= n_chunks[d] || j >= m || (kind == K_W && !P->has_w)) { malformed_head = 1; continue; }
      const int s = local_stage[d * MAX_CHUNKS + c];
      const size_t at = (size_t)s * m + j;
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
      if (state[at] != need) continue;
      const int64_t dt = P->dur[kind * S + s], u = P->mem_units[s];
      int64_t start, finish;
      if (kind == K_O || kind == K_L) {
        /* C2, C3: hand-over (waiting for room in the engine if need be), then the copy timeline */
        int64_t handover = free_at[d];
        if (n_copy[d] >= depth) {
          const int64_t oldest = copy_fin[(size_t)d * stride + n_copy[d] - depth];
          if (oldest > handover) handover = oldest;
        }
        start = handover > copy_free[d] ? handover : copy_free[d];
        finish = start + dt;
        copy_free[d] = finish;
        copy_fin[(size_t)d * stride + n_copy[d]++] = finish;
        free_at[d] = handover;
        mem_event *e = &ev_copy[(size_t)d * stride + n_ev_copy[d]++];
        if (kind == K_L) { e->time = start; e->delta = u; resident_at[at] = finish; }
        else { e->time = finish; e->delta = -u; }
      } else {
        int64_t ready = 0;
        int blocked = 0;
        for (int e = 0; e < E && !blocked; ++e) {
          int64_t t = 0, lat = 0;
          if ((kind == K_F || kind == K_FD) && P->edge_dst[e] == s) {
            t = fin_fwd[(size_t)P->edge_src[e] * m + j];
            lat = P->stage_device[P->edge_src[e]] != d ? P->edge_comm[e] : 0;
          } else if (kind == K_B && P->edge_src[e] == s) {
            t = fin_bwd[(size_t)P->edge_dst[e] * m + j];
            lat = P->stage_device[P->edge_dst[e]] != d ? P->edge_comm[e] : 0;
          } else continue;
          if (t < 0) blocked = 1;
          else if (t + lat > ready) ready = t + lat;
        }
        if (blocked) continue;
        if (kind == K_B && resident_at[at] > ready) ready = resident_at[at];   /* C4 */
        start = free_at[d] > ready ? free_at[d] : ready;
        finish = start + dt;
        free_at[d] = finish;
        busy[d] += dt;
        mem_event *e = &ev_compute[2 * (size_t)d * stride + n_ev_compute[d]];
        if (kind == K_F || kind == K_FD || kind == K_R) { e->time = start; e->delta = u; ++e; ++n_ev_compute[d]; }
        if (kind == K_FD || kind == K_W || (kind == K_B && !P->has_w)) { e->time = finish; e->delta = -u; ++n_ev_compute[d]; }
        if (kind == K_F || kind == K_FD) fin_fwd[at] = finish;
        if (kind == K_B) fin_bwd[at] = finish;
      }
      state[at] = (uint8_t)next;
      if (op_start) {
        op_start[(size_t)d * stride + cursor[d]] = start;
        op_finish[(size_t)d * stride + cursor[d]] = finish;
      }
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
    for (int d = 0; d < D; ++d) {
      if (free_at[d] > ms) ms = free_at[d];
      if (copy_free[d] > ms) ms = copy_free[d];
    }
    *makespan = ms;
    for (int d = 0; d < D; ++d) {
      /* C5: the two event sequences of the device, each already in time order, merged; ties: compute first */
      const mem_event *a = &ev_compute[2 * (size_t)d * stride], *b = &ev_copy[(size_t)d * stride];
      int ia = 0, ib = 0;
      int64_t mem = 0, pk = 0;
      while (ia < n_ev_compute[d] || ib < n_ev_copy[d]) {
        const int take_copy = ia >= n_ev_compute[d] || (ib < n_ev_copy[d] && b[ib].time < a[ia].time);
        mem += take_copy ? b[ib++].delta : a[ia++].delta;
        if (mem > pk) pk = mem;
      }
      idle[d] = ms - busy[d];
      peak[d] = (int32_t)pk;
      if (pk > P->mem_cap[d]) fl |= FLAG_OVER_CAP;
    }
  }
  *flags = fl;
  free(fin_fwd); free(fin_bwd); free(resident_at); free(state); free(cursor); free(len); free(free_at);
  free(copy_free); free(busy); free(copy_fin); free(n_copy); free(ev_compute); free(ev_copy);
  free(n_ev_compute); free(n_ev_copy);
  return 0;
}

/* Candidates [0, n_cand) of a batch laid out [C][D][stride]. */
int fpcopy_evaluate(const fpcopy_problem *P, int32_t depth, const uint16_t *words, int64_t n_cand, int32_t stride,
                    int64_t *makespan, int64_t *idle, int32_t *peak, uint8_t *flags) {
  const int D = P->n_devices;
  for (int64_t c = 0; c < n_cand; ++c) {
    const int rc = fpcopy_eval_one(P, depth, words + (size_t)c * D * stride, stride, &makespan[c], &idle[c * D],
                                   &peak[c * D], &flags[c], NULL, NULL);
    if (rc) return rc;
  }
  return 0;
}

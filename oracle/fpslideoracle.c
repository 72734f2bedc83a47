/*
 * fpslideoracle.c -- CPU oracle of the weight-gradient sliding pass.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, single-threaded; nothing in the
 * product path may call it, and it shares no code with the HIP sources nor
 * with the other oracle files (the few declarations it needs are repeated
 * here).  Times are int64.
 *
 * What the pass does (paper, Section 5.2, "Bubble optimizations": the
 * backward pass is separated into the part that the upstream stage waits for
 * and the weight-gradient part; the weight-gradient computations are stashed
 * and put into later bubbles of the same actor, so that the items others wait
 * for run as early as possible).  The paper describes the idea on a figure
 * and gives no rule for which bubble takes which stashed item; the rule below
 * is this library's reading:
 *
 *   Input: per device an ordered list of op words of a problem with split
 *   backward (kinds F, B, W, R, O, L, FD).  W words of the input are dropped:
 *   only the order of the other items is taken from it.
 *
 *   Every device walks its list in order under the evaluator's start rule
 *   (start = max(device free, inputs' finish + latency), finish = start +
 *   dur[kind][stage]; activation state machine as in the evaluator).  A B
 *   item that issues puts its weight-gradient item W(stage, micro-batch) at
 *   the back of the device's stash, a first-in first-out queue.
 *
 *   Before an item X of the list issues at its start time t, the device runs
 *   stashed W items in the idle time in front of it: as long as the stash is
 *   not empty and its oldest item ends no later than t when started now
 *   (device free + dur[W][its stage] <= t), that item issues at the time the
 *   device is free.  X is never delayed.  Only the oldest item is tried.
 *
 *   When the list ends, the items still stashed issue back to back.
 *
 *   Output: per device the new list (the order in which its items issued,
 *   END-padded to stride_out) and the evaluation of that list: makespan,
 *   idle, peak, flags, with the evaluator's meaning and sentinels.  A row of
 *   stride_out words that cannot hold all items of its device keeps the
 *   first stride_out of them; nothing else changes for the other devices
 *   (where the W items go never moves an item of the list), and the
 *   candidate is reported as DEADLOCK | INCOMPLETE with the sentinels.
 *
 * Parity pins (tests/test_slideoracle.py): the output list evaluated by the
 * evaluation oracle reproduces the results; the new list is the old order of
 * the non-W items with one W behind each B; weight-gradient items of zero
 * cost end up directly behind their B; one device alone has no idle time and
 * gets all W at the end; a hand-worked timeline on two devices.
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
} fpslide_problem;

typedef struct {
  const fpslide_problem *P;
  int d;                 /* the device */
  uint16_t *out;         /* its output row */
  int32_t cap, len;      /* words the row holds, words written */
  int64_t free_at, busy, mem, peak;
  int halted;            /* stopped at a malformed word */
  int overflow;          /* some item found the row full */
} device_t;

/* One item issues on its device at `start`; its word joins the row while there is room. */
static void issue(device_t *dev, int kind, int chunk, int s, int j, int64_t start, uint8_t *state) {
  const fpslide_problem *P = dev->P;
  if (dev->len < dev->cap) dev->out[dev->len++] = (uint16_t)((kind << 13) | (chunk << 11) | j);
  else dev->overflow = 1;
  const int64_t dt = P->dur[kind * P->n_stages + s], u = P->mem_units[s];
  if (kind == K_F || kind == K_FD || kind == K_R || kind == K_L) {
    dev->mem += u;
    if (dev->mem > dev->peak) dev->peak = dev->mem;
  }
  if (kind == K_FD || kind == K_O || kind == K_W) dev->mem -= u;
  switch (kind) {
    case K_F:  *state = ST_RES; break;
    case K_FD: *state = ST_DISC; break;
    case K_R:  *state = ST_RES; break;
    case K_O:  *state = ST_OFF; break;
    case K_L:  *state = ST_RES; break;
    case K_B:  *state = ST_BDONE; break;
    default:   *state = ST_DONE; break;
  }
  dev->free_at = start + dt;
  dev->busy += dt;
}

/*
 * links != 0: the pass under the link-occupancy variant of the cost model (every ordered pair of devices
 * is a link that carries one value at a time: a value leaves when its item has finished and the link is
 * free, keeps the link busy for the edge's latency and arrives at its end; values of a device leave in the
 * order its items run, two values of one item in the order of the edge list).  Weight-gradient items send
 * nothing, so the sliding rule itself is the same; only the times the list items are ready at change.
 */
static int slide_one(const fpslide_problem *P, int links, const uint16_t *words, int32_t stride, uint16_t *out_words,
                     int32_t stride_out, int64_t *makespan, int64_t *idle, int32_t *peak, uint8_t *flags) {
  const int D = P->n_devices, S = P->n_stages, m = P->n_microbatches, E = P->n_edges;
  if (!P->has_w) return -1;
  /* links: arrival of the value sent over edge e for micro-batch j, forward and backward (-1 = not sent),
   * and until when the link from device a to device b is busy */
  int64_t *arr_fwd = malloc(sizeof(int64_t) * (size_t)(E > 0 ? E : 1) * m);
  int64_t *arr_bwd = malloc(sizeof(int64_t) * (size_t)(E > 0 ? E : 1) * m);
  int64_t *busy_until = calloc((size_t)D * D, sizeof(int64_t));
  for (int64_t i = 0; i < (int64_t)E * m; ++i) arr_fwd[i] = arr_bwd[i] = -1;
  int32_t *local_stage = malloc(sizeof(int32_t) * D * MAX_CHUNKS), *n_chunks = calloc(D, sizeof(int32_t));
  for (int s = 0; s < S; ++s) {   /* chunk c of device d = the c-th of d's stages in ascending stage id */
    const int d = P->stage_device[s];
    if (d < 0 || d >= D || n_chunks[d] >= MAX_CHUNKS) { free(local_stage); free(n_chunks); return -1; }
    local_stage[d * MAX_CHUNKS + n_chunks[d]++] = s;
  }
  int64_t *fin_fwd = malloc(sizeof(int64_t) * S * m), *fin_bwd = malloc(sizeof(int64_t) * S * m);
  uint8_t *state = calloc((size_t)S * m, 1);
  for (int i = 0; i < S * m; ++i) fin_fwd[i] = fin_bwd[i] = -1;
  device_t *dev = calloc(D, sizeof(device_t));
  int32_t *cursor = calloc(D, sizeof(int32_t)), *len = calloc(D, sizeof(int32_t));
  int *finished = calloc(D, sizeof(int));
  /* stash: per device a queue of (chunk, micro-batch), at most one entry per B item */
  int32_t *stash = malloc(sizeof(int32_t) * 2 * (size_t)D * MAX_CHUNKS * m);
  int32_t *stash_head = calloc(D, sizeof(int32_t)), *stash_tail = calloc(D, sizeof(int32_t));
  memset(out_words, 0, sizeof(uint16_t) * (size_t)D * stride_out);
  for (int d = 0; d < D; ++d) {
    dev[d].P = P; dev[d].d = d; dev[d].out = out_words + (size_t)d * stride_out; dev[d].cap = stride_out;
    while (len[d] < stride && (words[(size_t)d * stride + len[d]] >> 13) != K_END) ++len[d];
  }

  for (int moved = 1; moved;) {
    moved = 0;
    for (int d = 0; d < D; ++d) {
      if (finished[d] || dev[d].halted) continue;
      int32_t *q = stash + 2 * (size_t)d * MAX_CHUNKS * m;
      if (cursor[d] >= len[d]) {
        /* the list is over: what is still stashed runs back to back */
        while (stash_head[d] < stash_tail[d]) {
          const int c = q[2 * stash_head[d]], j = q[2 * stash_head[d] + 1], s = local_stage[d * MAX_CHUNKS + c];
          issue(&dev[d], K_W, c, s, j, dev[d].free_at, &state[(size_t)s * m + j]);
          ++stash_head[d];
        }
        finished[d] = 1;
        moved = 1;
        continue;
      }
      const uint16_t w = words[(size_t)d * stride + cursor[d]];
      const int kind = w >> 13, c = (w >> 11) & 3, j = w & 0x7ff;
      if (c >= n_chunks[d] || j >= m) { dev[d].halted = 1; continue; }
      if (kind == K_W) { ++cursor[d]; moved = 1; continue; }   /* the input's own placement of W is not used */
      const int s = local_stage[d * MAX_CHUNKS + c];
      uint8_t *st = &state[(size_t)s * m + j];
      const int need = (kind == K_F || kind == K_FD) ? ST_ABSENT : kind == K_R ? ST_DISC
                     : kind == K_L ? ST_OFF : ST_RES /* O, B */;
      if (*st != need) continue;
      int64_t ready = 0;
      int blocked = 0;
      for (int e = 0; e < P->n_edges; ++e) {
        int other;
        const int64_t *fin;
        if ((kind == K_F || kind == K_FD) && P->edge_dst[e] == s) { other = P->edge_src[e]; fin = fin_fwd; }
        else if (kind == K_B && P->edge_src[e] == s) { other = P->edge_dst[e]; fin = fin_bwd; }
        else continue;
        int64_t r;
        if (links) {
          r = (fin == fin_fwd ? arr_fwd : arr_bwd)[(size_t)e * m + j];
          if (r < 0) { blocked = 1; break; }
        } else {
          const int64_t t = fin[(size_t)other * m + j];
          if (t < 0) { blocked = 1; break; }
          r = t + (P->stage_device[other] != d ? P->edge_comm[e] : 0);
        }
        if (r > ready) ready = r;
      }
      if (blocked) continue;
      const int64_t start = dev[d].free_at > ready ? dev[d].free_at : ready;
      /* idle time in front of the item: the oldest stashed W runs if it is over by `start` */
      while (stash_head[d] < stash_tail[d]) {
        const int cq = q[2 * stash_head[d]], jq = q[2 * stash_head[d] + 1], sq = local_stage[d * MAX_CHUNKS + cq];
        if (dev[d].free_at + P->dur[K_W * S + sq] > start) break;
        issue(&dev[d], K_W, cq, sq, jq, dev[d].free_at, &state[(size_t)sq * m + jq]);
        ++stash_head[d];
      }
      issue(&dev[d], kind, c, s, j, start, st);
      if (kind == K_F || kind == K_FD) fin_fwd[(size_t)s * m + j] = dev[d].free_at;
      if (kind == K_B) {
        fin_bwd[(size_t)s * m + j] = dev[d].free_at;
        q[2 * stash_tail[d]] = c; q[2 * stash_tail[d] + 1] = j; ++stash_tail[d];
      }
      if (links && (kind == K_F || kind == K_FD || kind == K_B)) {
        /* the result goes out over every edge to another stage: activations downstream, gradients upstream */
        const int fwd = kind != K_B;
        const int64_t finish = dev[d].free_at;
        for (int e = 0; e < E; ++e) {
          if ((fwd ? P->edge_src[e] : P->edge_dst[e]) != s) continue;
          const int to = P->stage_device[fwd ? P->edge_dst[e] : P->edge_src[e]];
          int64_t arrival = finish;
          if (to != d) {
            int64_t *link = &busy_until[(size_t)d * D + to];
            arrival = (finish > *link ? finish : *link) + P->edge_comm[e];
            *link = arrival;
          }
          (fwd ? arr_fwd : arr_bwd)[(size_t)e * m + j] = arrival;
        }
      }
      ++cursor[d];
      moved = 1;
    }
  }

  uint8_t fl = 0;
  for (int d = 0; d < D; ++d) {
    if (!finished[d]) fl |= FLAG_DEADLOCK;
    if (dev[d].halted || dev[d].overflow) fl |= FLAG_DEADLOCK | FLAG_INCOMPLETE;
  }
  if (!fl)
    for (int i = 0; i < S * m; ++i) if (state[i] != ST_DONE) { fl = FLAG_INCOMPLETE; break; }
  if (fl) {
    *makespan = INT64_MAX;
    for (int d = 0; d < D; ++d) { idle[d] = -1; peak[d] = -1; }
  } else {
    int64_t ms = 0;
    for (int d = 0; d < D; ++d) if (dev[d].free_at > ms) ms = dev[d].free_at;
    *makespan = ms;
    for (int d = 0; d < D; ++d) {
      idle[d] = ms - dev[d].busy;
      peak[d] = (int32_t)dev[d].peak;
      if (dev[d].peak > P->mem_cap[d]) fl |= FLAG_OVER_CAP;
    }
  }
  *flags = fl;
  free(arr_fwd); free(arr_bwd); free(busy_until);
  free(local_stage); free(n_chunks); free(fin_fwd); free(fin_bwd); free(state); free(dev); free(cursor);
  free(len); free(finished); free(stash); free(stash_head); free(stash_tail);
  return 0;
}

int fpslide_oracle_one(const fpslide_problem *P, const uint16_t *words, int32_t stride, uint16_t *out_words,
                       int32_t stride_out, int64_t *makespan, int64_t *idle, int32_t *peak, uint8_t *flags) {
  return slide_one(P, 0, words, stride, out_words, stride_out, makespan, idle, peak, flags);
}

/* Candidates [0, n_cand) of a batch laid out [C][D][stride] -> [C][D][stride_out]; links: see slide_one. */
int fpslide_oracle_batch_links(const fpslide_problem *P, int32_t links, const uint16_t *words, int64_t n_cand,
                               int32_t stride, uint16_t *out_words, int32_t stride_out, int64_t *makespan,
                               int64_t *idle, int32_t *peak, uint8_t *flags) {
  const int D = P->n_devices;
  for (int64_t c = 0; c < n_cand; ++c) {
    const int rc = slide_one(P, links, words + (size_t)c * D * stride, stride,
                             out_words + (size_t)c * D * stride_out, stride_out, &makespan[c],
                             &idle[c * D], &peak[c * D], &flags[c]);
    if (rc) return rc;
  }
  return 0;
}

int fpslide_oracle_batch(const fpslide_problem *P, const uint16_t *words, int64_t n_cand, int32_t stride,
                         uint16_t *out_words, int32_t stride_out, int64_t *makespan, int64_t *idle,
                         int32_t *peak, uint8_t *flags) {
  return fpslide_oracle_batch_links(P, 0, words, n_cand, stride, out_words, stride_out, makespan, idle, peak, flags);
}

/*
 * fpgen.c -- seeded synthetic candidate schedules (input generator).
 *
 * Produces per-device op orders, packed as 16-bit op words, by randomized
 * list scheduling over the stage DAG.  It serves the tests, the benchmark,
 * the CPU oracle's callers and the GPU library's callers alike and contains
 * none of the evaluator: it emits ORDERS only.  Its private clock exists to
 * make the orders look like schedules a search would propose (and is handed
 * out, optionally, so that a test can compare it with the oracle).
 *
 * Recipe (paper, Section 5.2: every actor keeps fetching dependency-free items
 * in a priority order; Section 4.2: an in-flight micro-batch limit; Section 6:
 * the tuner enumerates priority settings):
 *   - per candidate, draw weights  prio = w_kind[k] + w_chunk[k][c] - w_mb*j
 *     + noise, and an open-micro-batch limit K per device;
 *   - repeat: take the device that can start something earliest; among its
 *     ops that are startable by then, append the one with the highest
 *     priority to that device's list;
 *   - within one (kind, stage) micro-batches are emitted in ascending order
 *     (paper, Section 5.1, "Data dependency": the default rule);
 *   - optional recompute marks (forward becomes FD, an R op is inserted just
 *     before the backward can run) or offload marks (O after the forward,
 *     L just before the backward);
 *   - a stated fraction of candidates is then perturbed so that it deadlocks
 *     (half same-device, half a two-device cycle), another small fraction
 *     gets a harmless delay of one W (or B/F swap).  What a perturbed candidate
 *     really does is decided by whoever evaluates it, never by this label.
 * All random numbers are splitmix64 of (seed, candidate index, counter), so a
 * candidate can be regenerated alone.
 */
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { K_END = 0, K_F = 1, K_B = 2, K_W = 3, K_R = 4, K_O = 5, K_L = 6, K_FD = 7, NKINDS = 8 };
#define MAX_CHUNKS 4
#define T_INF INT64_MAX

/* stream ids per stage */
enum { Q_FWD = 0, Q_B = 1, Q_W = 2, Q_R = 3, Q_O = 4, Q_L = 5, NQ = 6 };
enum { DONE_FWD = 1, DONE_R = 2, DONE_O = 4, DONE_L = 8, DONE_B = 16, DONE_W = 32 };

typedef struct {
  int32_t n_devices, n_stages, n_microbatches, has_w;
  const int32_t *stage_device;
  int32_t n_edges;
  const int32_t *edge_src, *edge_dst, *edge_comm;
  const int32_t *dur; /* [NKINDS][S] */
  int32_t recompute;  /* 1: draw recompute marks */
  int32_t offload;    /* 1: draw offload marks */
  int32_t max_marks_per_device; /* bound on R (or O/L pairs) per device list */
  int32_t cap_units;  /* memory cap the in-flight limit is centred on */
  uint64_t seed;
  int32_t deadlock_per_mille; /* candidates perturbed to deadlock, in 1/1000 */
  int32_t benign_per_mille;   /* candidates given a harmless reorder, in 1/1000 */
} fpgen_params;

static uint64_t mix64(uint64_t x) {
  x += 0x9E3779B97F4A7C15ull;
  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
  x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
  return x ^ (x >> 31);
}
typedef struct { uint64_t key, ctr; } rng_t;
static rng_t rng_make(uint64_t seed, uint64_t cand, uint64_t stream) {
  rng_t r = { mix64(mix64(seed) ^ mix64(cand * 0xD1342543DE82EF95ull + stream)), 0 };
  return r;
}
static uint64_t rng_next(rng_t *r) { return mix64(r->key + (r->ctr++) * 0x2545F4914F6CDD1Dull); }
static uint32_t rng_below(rng_t *r, uint32_t n) { return (uint32_t)((rng_next(r) >> 32) * (uint64_t)n >> 32); }

typedef struct {
  const fpgen_params *P;
  int D, S, m;
  int32_t *local_stage;  /* [D][MAX_CHUNKS] */
  int32_t *n_chunks;     /* [D] */
  int32_t *chunk_of;     /* [S] */
  int32_t *pred_off, *pred_s, *pred_c; /* CSR by dst */
  int32_t *succ_off, *succ_s, *succ_c; /* CSR by src */
  /* per candidate */
  uint8_t *mark;     /* [S*m] 1 = recompute or offload mark */
  uint8_t *done;     /* [S*m] DONE_* bits */
  int64_t *fin_fwd, *fin_bwd; /* [S*m] generator clock */
  int32_t *head;     /* [S][NQ] */
  int64_t *free_at, *t_dev; /* [D] */
  int32_t *open;     /* [D] */
  int32_t *limit;    /* [D] */
  int32_t *len;      /* [D] */
  int32_t *marks_on_dev; /* [D] */
  int64_t w_kind[NKINDS], w_chunk[NKINDS][MAX_CHUNKS], w_mb, noise;
} gen_t;

static int kind_of_stream(const gen_t *g, int q, int s, int j) {
  switch (q) {
    case Q_FWD: return (g->P->recompute && g->mark[s * g->m + j]) ? K_FD : K_F;
    case Q_B: return K_B;
    case Q_W: return K_W;
    case Q_R: return K_R;
    case Q_O: return K_O;
    default: return K_L;
  }
}

/* Is the head op of stream q of stage s startable given what is already listed?
 * Returns 1 and the earliest start contribution of its cross-stage inputs. */
static int stream_available(gen_t *g, int s, int q, int *out_j, int64_t *out_ready) {
  const int m = g->m, d = g->P->stage_device[s];
  int j = g->head[s * NQ + q];
  if (q == Q_R || q == Q_O || q == Q_L) {
    while (j < m && !g->mark[s * m + j]) ++j;
    g->head[s * NQ + q] = j;
  }
  if (j >= m) return 0;
  const uint8_t dn = g->done[s * m + j];
  int64_t ready = 0;
  switch (q) {
    case Q_FWD:
      if (g->chunk_of[s] == 0 && g->open[d] >= g->limit[d]) return 0;
      for (int e = g->pred_off[s]; e < g->pred_off[s + 1]; ++e) {
        const int sp = g->pred_s[e];
        if (!(g->done[sp * m + j] & DONE_FWD)) return 0;
        const int64_t r = g->fin_fwd[sp * m + j] + (g->P->stage_device[sp] != d ? g->pred_c[e] : 0);
        if (r > ready) ready = r;
      }
      break;
    case Q_B:
      if (!(dn & DONE_FWD)) return 0;
      if (g->mark[s * m + j]) {
        if (g->P->recompute && !(dn & DONE_R)) return 0;
        if (g->P->offload && !(dn & DONE_L)) return 0;
      }
      /* fall through: B, and the just-in-time R and L, wait for the downstream backward */
    case Q_R:
    case Q_L:
      if (q == Q_R && (!(dn & DONE_FWD) || (dn & DONE_R))) return 0;
      if (q == Q_L && (!(dn & DONE_O) || (dn & DONE_L))) return 0;
      for (int e = g->succ_off[s]; e < g->succ_off[s + 1]; ++e) {
        const int sn = g->succ_s[e];
        if (!(g->done[sn * m + j] & DONE_B)) return 0;
        const int64_t r = g->fin_bwd[sn * m + j] + (g->P->stage_device[sn] != d ? g->succ_c[e] : 0);
        if (r > ready) ready = r;
      }
      if (q != Q_B) ready = 0; /* R and L have no cross-stage input of their own */
      break;
    case Q_W:
      if (!(dn & DONE_B)) return 0;
      break;
    case Q_O:
      if (!(dn & DONE_FWD) || (dn & DONE_O)) return 0;
      break;
  }
  *out_j = j;
  *out_ready = ready;
  return 1;
}

static int stream_enabled(const gen_t *g, int q) {
  if (q == Q_W) return g->P->has_w;
  if (q == Q_R) return g->P->recompute;
  if (q == Q_O || q == Q_L) return g->P->offload;
  return 1;
}

/* earliest time device d could start anything (T_INF: nothing startable yet) */
static int64_t device_time(gen_t *g, int d) {
  int64_t best = T_INF;
  for (int c = 0; c < g->n_chunks[d]; ++c) {
    const int s = g->local_stage[d * MAX_CHUNKS + c];
    for (int q = 0; q < NQ; ++q) {
      if (!stream_enabled(g, q)) continue;
      int j; int64_t r;
      if (stream_available(g, s, q, &j, &r) && r < best) best = r;
    }
  }
  if (best == T_INF) return T_INF;
  return best > g->free_at[d] ? best : g->free_at[d];
}

static void gen_one(gen_t *g, int64_t cand, int32_t stride, uint16_t *out, int64_t *gen_makespan) {
  const fpgen_params *P = g->P;
  const int D = g->D, S = g->S, m = g->m;
  rng_t rw = rng_make(P->seed, (uint64_t)cand, 1);
  /* priority weights */
  for (int k = 0; k < NKINDS; ++k) {
    g->w_kind[k] = rng_below(&rw, 1000);
    for (int c = 0; c < MAX_CHUNKS; ++c) g->w_chunk[k][c] = rng_below(&rw, 400);
  }
  if (rng_below(&rw, 4) != 0) g->w_kind[K_B] += 600;       /* mostly backward-first */
  g->w_kind[K_FD] = g->w_kind[K_F];
  for (int c = 0; c < MAX_CHUNKS; ++c) g->w_chunk[K_FD][c] = g->w_chunk[K_F][c];
  g->w_kind[K_O] += 500;
  g->w_mb = rng_below(&rw, 40);
  { static const int64_t scales[4] = { 0, 8, 64, 512 }; g->noise = scales[rng_below(&rw, 4)]; }

  /* marks */
  memset(g->mark, 0, (size_t)S * m);
  memset(g->marks_on_dev, 0, sizeof(int32_t) * D);
  if (P->recompute || P->offload) {
    static const uint32_t rho_rec[4] = { 0, 128, 256, 512 };  /* of 1024 */
    static const uint32_t rho_off[4] = { 0, 128, 256, 0 };
    const uint32_t rho = P->recompute ? rho_rec[rng_below(&rw, 4)] : rho_off[rng_below(&rw, 3)];
    rng_t rm = rng_make(P->seed, (uint64_t)cand, 2);
    for (int s = 0; s < S; ++s)
      for (int j = 0; j < m; ++j) {
        const int d = P->stage_device[s];
        if (rng_below(&rm, 1024) < rho && g->marks_on_dev[d] < P->max_marks_per_device) {
          g->mark[s * m + j] = 1;
          g->marks_on_dev[d] += 1;
        }
      }
  }
  /* open-micro-batch limit per device, centred on cap / chunks */
  {
    const uint32_t u = rng_below(&rw, 1024);
    for (int d = 0; d < D; ++d) {
      const int v = g->n_chunks[d] > 0 ? g->n_chunks[d] : 1;
      int64_t k = ((int64_t)P->cap_units * (512 + 1280 * (int64_t)u / 1024)) / (1024 * (int64_t)v);
      if (k < 1) k = 1;
      if (k > m) k = m;
      g->limit[d] = (int32_t)k;
    }
  }

  memset(g->done, 0, (size_t)S * m);
  memset(g->head, 0, sizeof(int32_t) * S * NQ);
  for (int d = 0; d < D; ++d) { g->free_at[d] = 0; g->open[d] = 0; g->len[d] = 0; }
  memset(out, 0, sizeof(uint16_t) * (size_t)D * stride);
  for (int d = 0; d < D; ++d) g->t_dev[d] = device_time(g, d);

  rng_t rn = rng_make(P->seed, (uint64_t)cand, 3);
  for (;;) {
    int d = -1;
    int64_t t = T_INF;
    for (int i = 0; i < D; ++i) if (g->t_dev[i] < t) { t = g->t_dev[i]; d = i; }
    if (d < 0) break;
    /* highest-priority op of d that is startable by t */
    int best_s = -1, best_q = 0, best_j = 0;
    int64_t best_prio = INT64_MIN, best_ready = 0;
    for (int c = 0; c < g->n_chunks[d]; ++c) {
      const int s = g->local_stage[d * MAX_CHUNKS + c];
      for (int q = 0; q < NQ; ++q) {
        if (!stream_enabled(g, q)) continue;
        int j; int64_t r;
        if (!stream_available(g, s, q, &j, &r) || r > t) continue;
        const int k = kind_of_stream(g, q, s, j);
        int64_t prio = g->w_kind[k] + g->w_chunk[k][c] - g->w_mb * j;
        if (g->noise) prio += (int64_t)rng_below(&rn, (uint32_t)g->noise);
        if (prio > best_prio) { best_prio = prio; best_s = s; best_q = q; best_j = j; best_ready = r; }
      }
    }
    /* list it */
    const int s = best_s, j = best_j, q = best_q;
    const int k = kind_of_stream(g, q, s, j);
    const int64_t start = best_ready > g->free_at[d] ? best_ready : g->free_at[d];
    const int64_t finish = start + P->dur[k * S + s];
    g->free_at[d] = finish;
    if (g->len[d] < stride)
      out[(size_t)d * stride + g->len[d]] = (uint16_t)((k << 13) | (g->chunk_of[s] << 11) | j);
    g->len[d] += 1;
    uint8_t *dn = &g->done[s * m + j];
    switch (q) {
      case Q_FWD: *dn |= DONE_FWD; g->fin_fwd[s * m + j] = finish; g->head[s * NQ + Q_FWD] = j + 1;
                  if (g->chunk_of[s] == 0) g->open[d] += 1; break;
      case Q_B:   *dn |= DONE_B; g->fin_bwd[s * m + j] = finish; g->head[s * NQ + Q_B] = j + 1;
                  if (!P->has_w && g->chunk_of[s] == 0) g->open[d] -= 1; break;
      case Q_W:   *dn |= DONE_W; g->head[s * NQ + Q_W] = j + 1;
                  if (g->chunk_of[s] == 0) g->open[d] -= 1; break;
      case Q_R:   *dn |= DONE_R; g->head[s * NQ + Q_R] = j + 1; break;
      case Q_O:   *dn |= DONE_O; g->head[s * NQ + Q_O] = j + 1; break;
      default:    *dn |= DONE_L; g->head[s * NQ + Q_L] = j + 1; break;
    }
    /* refresh the devices whose options changed */
    g->t_dev[d] = device_time(g, d);
    if (q == Q_FWD)
      for (int e = g->succ_off[s]; e < g->succ_off[s + 1]; ++e) {
        const int dd = P->stage_device[g->succ_s[e]];
        if (dd != d) g->t_dev[dd] = device_time(g, dd);
      }
    if (q == Q_B)
      for (int e = g->pred_off[s]; e < g->pred_off[s + 1]; ++e) {
        const int dd = P->stage_device[g->pred_s[e]];
        if (dd != d) g->t_dev[dd] = device_time(g, dd);
      }
  }
  int64_t ms = 0;
  for (int d = 0; d < D; ++d) if (g->free_at[d] > ms) ms = g->free_at[d];
  int perturbed = 0;

  /* perturbations */
  rng_t rp = rng_make(P->seed, (uint64_t)cand, 4);
  const uint32_t roll = rng_below(&rp, 1000);
  if ((int32_t)roll < P->deadlock_per_mille) {
    perturbed = 1;
    if (rng_below(&rp, 2) == 0 || S < 2) {
      /* same-device: move an op in front of the op of the same (stage, micro-batch) it needs */
      for (int tries = 0; tries < 64; ++tries) {
        const int d = (int)rng_below(&rp, (uint32_t)D);
        const int n = g->len[d] < stride ? g->len[d] : stride;
        if (n < 2) continue;
        uint16_t *row = out + (size_t)d * stride;
        const int i = 1 + (int)rng_below(&rp, (uint32_t)(n - 1));
        const int k = row[i] >> 13;
        if (k == K_F || k == K_FD) continue;
        const uint16_t key = row[i] & 0x1FFF; /* chunk + micro-batch */
        int i0 = -1;
        for (int a = 0; a < i; ++a) if ((row[a] & 0x1FFF) == key) { i0 = a; }
        if (i0 < 0) continue;
        const uint16_t w = row[i];
        memmove(row + i0 + 1, row + i0, sizeof(uint16_t) * (size_t)(i - i0));
        row[i0] = w;
        break;
      }
    } else {
      /* two-device cycle: on A put B(s,j) before F(s,j2); on the device of a successor
       * stage put F(s+,j2) before B(s+,j) */
      for (int tries = 0; tries < 64; ++tries) {
        const int s = (int)rng_below(&rp, (uint32_t)S);
        if (g->succ_off[s + 1] == g->succ_off[s]) continue;
        const int sn = g->succ_s[g->succ_off[s]];
        const int da = P->stage_device[s], db = P->stage_device[sn];
        if (da == db || m < 2) continue;
        const int j = (int)rng_below(&rp, (uint32_t)(m - 1));
        const int j2 = j + 1 + (int)rng_below(&rp, (uint32_t)(m - 1 - j));
        uint16_t *ra = out + (size_t)da * stride, *rb = out + (size_t)db * stride;
        const int na = g->len[da] < stride ? g->len[da] : stride;
        const int nb = g->len[db] < stride ? g->len[db] : stride;
        const uint16_t ca = (uint16_t)(g->chunk_of[s] << 11), cb = (uint16_t)(g->chunk_of[sn] << 11);
        int pa_b = -1, pa_f = -1, pb_b = -1, pb_f = -1;
        for (int a = 0; a < na; ++a) {
          if (ra[a] == (uint16_t)((K_B << 13) | ca | j)) pa_b = a;
          if ((ra[a] & 0x1FFF) == (ca | j2) && ((ra[a] >> 13) == K_F || (ra[a] >> 13) == K_FD)) pa_f = a;
        }
        for (int a = 0; a < nb; ++a) {
          if (rb[a] == (uint16_t)((K_B << 13) | cb | j)) pb_b = a;
          if ((rb[a] & 0x1FFF) == (cb | j2) && ((rb[a] >> 13) == K_F || (rb[a] >> 13) == K_FD)) pb_f = a;
        }
        if (pa_b < 0 || pa_f < 0 || pb_b < 0 || pb_f < 0) continue;
        if (pa_b > pa_f) { const uint16_t w = ra[pa_b];
          memmove(ra + pa_f + 1, ra + pa_f, sizeof(uint16_t) * (size_t)(pa_b - pa_f)); ra[pa_f] = w; }
        if (pb_f > pb_b) { const uint16_t w = rb[pb_f];
          memmove(rb + pb_b + 1, rb + pb_b, sizeof(uint16_t) * (size_t)(pb_f - pb_b)); rb[pb_b] = w; }
        break;
      }
    }
  } else if ((int32_t)roll < P->deadlock_per_mille + P->benign_per_mille) {
    perturbed = 1;
    /* harmless: delay one op that nothing else waits for (a W, or a B on a source-stage
     * device when backward is not split) by up to three places */
    for (int tries = 0; tries < 64; ++tries) {
      const int d = (int)rng_below(&rp, (uint32_t)D);
      const int n = g->len[d] < stride ? g->len[d] : stride;
      if (n < 2) continue;
      uint16_t *row = out + (size_t)d * stride;
      const int i = (int)rng_below(&rp, (uint32_t)(n - 1));
      if ((row[i] >> 13) != K_W) continue;
      int hop = 1 + (int)rng_below(&rp, 3);
      if (i + hop > n - 1) hop = n - 1 - i;
      const uint16_t w = row[i];
      memmove(row + i, row + i + 1, sizeof(uint16_t) * (size_t)hop);
      row[i + hop] = w;
      break;
    }
  }
  if (gen_makespan) *gen_makespan = perturbed ? -1 : ms;
}

typedef struct {
  const fpgen_params *P;
  int64_t first, count;
  int32_t stride;
  uint16_t *out;
  int64_t *gen_makespan;
  int rc;
} job_t;

static void *xcalloc(size_t n, size_t sz) { return calloc(n ? n : 1, sz); }

static int gen_init(gen_t *g, const fpgen_params *P) {
  memset(g, 0, sizeof(*g));
  g->P = P;
  const int D = g->D = P->n_devices, S = g->S = P->n_stages, m = g->m = P->n_microbatches;
  g->local_stage = xcalloc((size_t)D * MAX_CHUNKS, sizeof(int32_t));
  g->n_chunks = xcalloc(D, sizeof(int32_t));
  g->chunk_of = xcalloc(S, sizeof(int32_t));
  for (int s = 0; s < S; ++s) {
    const int d = P->stage_device[s];
    if (d < 0 || d >= D || g->n_chunks[d] >= MAX_CHUNKS) return -1;
    g->chunk_of[s] = g->n_chunks[d];
    g->local_stage[d * MAX_CHUNKS + g->n_chunks[d]++] = s;
  }
  const int E = P->n_edges;
  g->pred_off = xcalloc(S + 1, sizeof(int32_t)); g->succ_off = xcalloc(S + 1, sizeof(int32_t));
  g->pred_s = xcalloc(E, sizeof(int32_t)); g->pred_c = xcalloc(E, sizeof(int32_t));
  g->succ_s = xcalloc(E, sizeof(int32_t)); g->succ_c = xcalloc(E, sizeof(int32_t));
  for (int e = 0; e < E; ++e) { g->pred_off[P->edge_dst[e] + 1]++; g->succ_off[P->edge_src[e] + 1]++; }
  for (int s = 0; s < S; ++s) { g->pred_off[s + 1] += g->pred_off[s]; g->succ_off[s + 1] += g->succ_off[s]; }
  int32_t *pf = xcalloc(S, sizeof(int32_t)), *sf = xcalloc(S, sizeof(int32_t));
  for (int e = 0; e < E; ++e) {
    const int a = P->edge_src[e], b = P->edge_dst[e];
    g->pred_s[g->pred_off[b] + pf[b]] = a; g->pred_c[g->pred_off[b] + pf[b]++] = P->edge_comm[e];
    g->succ_s[g->succ_off[a] + sf[a]] = b; g->succ_c[g->succ_off[a] + sf[a]++] = P->edge_comm[e];
  }
  free(pf); free(sf);
  g->mark = xcalloc((size_t)S * m, 1); g->done = xcalloc((size_t)S * m, 1);
  g->fin_fwd = xcalloc((size_t)S * m, sizeof(int64_t)); g->fin_bwd = xcalloc((size_t)S * m, sizeof(int64_t));
  g->head = xcalloc((size_t)S * NQ, sizeof(int32_t));
  g->free_at = xcalloc(D, sizeof(int64_t)); g->t_dev = xcalloc(D, sizeof(int64_t));
  g->open = xcalloc(D, sizeof(int32_t)); g->limit = xcalloc(D, sizeof(int32_t));
  g->len = xcalloc(D, sizeof(int32_t)); g->marks_on_dev = xcalloc(D, sizeof(int32_t));
  return 0;
}
static void gen_free(gen_t *g) {
  free(g->local_stage); free(g->n_chunks); free(g->chunk_of);
  free(g->pred_off); free(g->succ_off); free(g->pred_s); free(g->pred_c); free(g->succ_s); free(g->succ_c);
  free(g->mark); free(g->done); free(g->fin_fwd); free(g->fin_bwd); free(g->head);
  free(g->free_at); free(g->t_dev); free(g->open); free(g->limit); free(g->len); free(g->marks_on_dev);
}

static void *job_main(void *arg) {
  job_t *J = arg;
  gen_t g;
  if (gen_init(&g, J->P)) { J->rc = -1; gen_free(&g); return NULL; }
  const size_t per = (size_t)J->P->n_devices * J->stride;
  for (int64_t i = 0; i < J->count; ++i) {
    gen_one(&g, J->first + i, J->stride, J->out + per * (size_t)i,
            J->gen_makespan ? &J->gen_makespan[i] : NULL);
    for (int d = 0; d < g.D; ++d) if (g.len[d] > J->stride) J->rc = -2; /* stride too small */
  }
  gen_free(&g);
  return NULL;
}

/* Candidates [first, first+count) -> out[count][D][stride]; gen_makespan (optional,
 * [count]): the generator's own clock for unperturbed candidates, -1 otherwise.
 * Returns 0, -1 (bad problem), -2 (stride too small for some list). */
int fpgen_generate(const fpgen_params *P, int64_t first, int64_t count, int32_t stride,
                   uint16_t *out, int64_t *gen_makespan, int32_t n_threads) {
  if (n_threads < 1) n_threads = 1;
  if (n_threads > 64) n_threads = 64;
  if ((int64_t)n_threads > count) n_threads = count > 0 ? (int32_t)count : 1;
  pthread_t th[64];
  job_t jobs[64];
  const size_t per = (size_t)P->n_devices * stride;
  for (int t = 0; t < n_threads; ++t) {
    const int64_t lo = count * t / n_threads, hi = count * (t + 1) / n_threads;
    jobs[t] = (job_t){ P, first + lo, hi - lo, stride, out + per * (size_t)lo,
                       gen_makespan ? gen_makespan + lo : NULL, 0 };
    if (n_threads == 1) job_main(&jobs[t]);
    else pthread_create(&th[t], NULL, job_main, &jobs[t]);
  }
  int rc = 0;
  for (int t = 0; t < n_threads; ++t) {
    if (n_threads > 1) pthread_join(th[t], NULL);
    if (jobs[t].rc) rc = jobs[t].rc;
  }
  return rc;
}

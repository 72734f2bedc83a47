/*
 * fpsyncgen.c -- seeded candidate schedules for problems with synchronisation stages and dependency
 * pairs (input generator).
 *
 * It emits ORDERS only and holds none of the evaluator: no costs, no latencies, no clock.  The recipe
 * follows the paper's scheduler in spirit (Section 5.2: in every scheduling step each actor fetches one
 * dependency-free item in a priority order; Section 4.2: an in-flight micro-batch limit; Section 6: the
 * tuner enumerates priority settings), with the priorities randomised per candidate:
 *   - a stage with group n has ceil(m / n) items per kind; item g stands for micro-batches
 *     g n .. min(m, (g + 1) n) - 1, and waits, along a DAG edge or a pair, for every item of the other
 *     stage whose micro-batches overlap its own (forward items along the DAG, backward items against
 *     it, pairs as given);
 *   - per candidate: a weight per kind (backward-first mostly), a weight per stage of a device, a
 *     preference for early micro-batches, noise, and an in-flight limit per device for the forward
 *     items of its first stage (never below the widest group: a synchronisation over n micro-batches
 *     needs n of them in flight in front of it);
 *   - in every step each device lists, among its items whose prerequisites were listed in EARLIER
 *     steps, the one of highest priority (items of one kind and stage in ascending order); a step in
 *     which nothing can be listed ends the candidate (cyclic pairs: the lists stay short);
 *   - a stated fraction of the candidates then gets two entries of one row swapped; whether such a
 *     candidate still runs is for whoever evaluates it to say.
 * All random numbers are splitmix64 of (seed, candidate, counter): a candidate can be regenerated alone.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { K_F = 1, K_B = 2, K_W = 3 };
#define MAX_CHUNKS 4
#define MAX_D 64
#define MAX_S 256

typedef struct {
  int32_t n_devices, n_stages, n_microbatches, has_w;
  const int32_t *stage_device;                 /* [S] */
  int32_t n_edges;
  const int32_t *edge_src, *edge_dst;          /* [E] */
  const int32_t *group;                        /* [S] */
  int32_t n_pairs;
  const int32_t *pairs;                        /* [n_pairs][5]: kind_from, stage_from, kind_to, stage_to, (latency) */
  uint64_t seed;
  int32_t swap_per_mille;                      /* candidates with two entries of a row swapped, in 1/1000 */
} fpsyncgen_params;

static uint64_t mix64(uint64_t x) {
  x += 0x9E3779B97F4A7C15ull;
  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
  x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
  return x ^ (x >> 31);
}
typedef struct { uint64_t key, ctr; } rng_t;
static uint64_t rng_next(rng_t *r) { return mix64(r->key + (r->ctr++) * 0x2545F4914F6CDD1Dull); }
static int32_t rng_below(rng_t *r, int32_t n) { return (int32_t)((rng_next(r) >> 32) * (uint64_t)n >> 32); }

static int items_of(const fpsyncgen_params *P, int s) {
  return (P->n_microbatches + P->group[s] - 1) / P->group[s];
}

/* were all items of (kind a_kind, stage a) that overlap item g of stage s listed before step t? */
static int listed_before(const fpsyncgen_params *P, const int32_t *step_of, int a_kind, int a, int s, int g, int t) {
  const int m = P->n_microbatches;
  const int lo = g * P->group[s];
  int hi = lo + P->group[s] - 1;
  if (hi > m - 1) hi = m - 1;
  for (int ga = lo / P->group[a]; ga <= hi / P->group[a]; ++ga) {
    const int32_t at = step_of[((size_t)a_kind * P->n_stages + a) * m + ga];
    if (at < 0 || at >= t) return 0;
  }
  return 1;
}

static int generate_one(const fpsyncgen_params *P, int64_t cand, int32_t stride, uint16_t *out) {
  const int D = P->n_devices, S = P->n_stages, m = P->n_microbatches;
  const int nk = P->has_w ? 3 : 2;
  rng_t rng = { mix64(mix64(P->seed) ^ mix64((uint64_t)cand * 0xD1342543DE82EF95ull + 7)), 0 };
  int32_t stages_of[MAX_D][MAX_CHUNKS], n_chunks[MAX_D], chunk_of[MAX_S];
  for (int d = 0; d < D; ++d) n_chunks[d] = 0;
  for (int s = 0; s < S; ++s) {
    const int d = P->stage_device[s];
    chunk_of[s] = n_chunks[d];
    stages_of[d][n_chunks[d]++] = s;
  }
  /* priorities of this candidate */
  int64_t w_kind[4], w_stage[MAX_S], w_mb, noise;
  const int style = rng_below(&rng, 10);            /* 0-6 backward first, 7-8 interleaved-like, 9 forward first */
  w_kind[K_B] = style <= 6 ? 4000 : (style <= 8 ? 2000 : 0);
  w_kind[K_F] = style <= 6 ? 0 : (style <= 8 ? 2000 : 4000);
  w_kind[K_W] = rng_below(&rng, 3) == 0 ? 3000 : -1000;   /* weight gradients early, or only to fill */
  for (int s = 0; s < S; ++s) w_stage[s] = rng_below(&rng, 600);
  w_mb = 20 + rng_below(&rng, 60);
  noise = rng_below(&rng, 4) == 0 ? 1 + rng_below(&rng, 1500) : 1 + rng_below(&rng, 100);
  /* a synchronisation over n micro-batches needs n of them in flight on the stages in front of it */
  int32_t limit[MAX_D], open[MAX_D], len[MAX_D], widest = 1;
  for (int s = 0; s < S; ++s) if (P->group[s] > widest) widest = P->group[s] < m ? P->group[s] : m;
  const int32_t spread = 1 + rng_below(&rng, 2 * D);
  for (int d = 0; d < D; ++d) {
    limit[d] = widest + rng_below(&rng, spread);
    open[d] = 0;
    len[d] = 0;
  }
  /* step at which each item was listed, -1 = not yet; next item of each (kind, stage) */
  int32_t *step_of = malloc(sizeof(int32_t) * 4 * (size_t)S * m);
  int32_t *next = calloc((size_t)4 * S, sizeof(int32_t));
  for (size_t i = 0; i < 4 * (size_t)S * m; ++i) step_of[i] = -1;
  memset(out, 0, sizeof(uint16_t) * (size_t)D * stride);
  int64_t left = 0;
  for (int s = 0; s < S; ++s) left += (int64_t)nk * items_of(P, s);
  for (int t = 0; left > 0; ++t) {
    int pick_k[MAX_D], pick_s[MAX_D], any = 0;
    for (int d = 0; d < D; ++d) {
      int64_t best = INT64_MIN;
      pick_k[d] = 0;
      for (int c = 0; c < n_chunks[d]; ++c) {
        const int s = stages_of[d][c];
        for (int k = K_F; k <= nk; ++k) {
          const int g = next[k * S + s];
          if (g >= items_of(P, s) || len[d] >= stride) continue;
          int ok = 1;
          if (k == K_B) ok = step_of[((size_t)K_F * S + s) * m + g] >= 0 && step_of[((size_t)K_F * S + s) * m + g] < t;
          if (k == K_W) ok = step_of[((size_t)K_B * S + s) * m + g] >= 0 && step_of[((size_t)K_B * S + s) * m + g] < t;
          if (k == K_F && c == 0 && open[d] >= limit[d]) ok = 0;
          for (int e = 0; e < P->n_edges && ok; ++e) {
            if (k == K_F && P->edge_dst[e] == s) ok = listed_before(P, step_of, K_F, P->edge_src[e], s, g, t);
            if (k == K_B && P->edge_src[e] == s) ok = listed_before(P, step_of, K_B, P->edge_dst[e], s, g, t);
          }
          for (int i = 0; i < P->n_pairs && ok; ++i) {
            const int32_t *q = P->pairs + 5 * i;
            if (q[2] == k && q[3] == s && q[0] >= K_F && q[0] <= K_W) ok = listed_before(P, step_of, q[0], q[1], s, g, t);
          }
          if (!ok) continue;
          const int64_t prio = w_kind[k] + w_stage[s] - w_mb * (int64_t)g * P->group[s] + rng_below(&rng, (int32_t)noise);
          if (prio > best) { best = prio; pick_k[d] = k; pick_s[d] = s; }
        }
      }
      any |= pick_k[d] != 0;
    }
    if (!any) break;
    for (int d = 0; d < D; ++d) {
      const int k = pick_k[d], s = pick_s[d];
      if (!k) continue;
      const int g = next[k * S + s]++;
      step_of[((size_t)k * S + s) * m + g] = t;
      out[(size_t)d * stride + len[d]++] = (uint16_t)((k << 13) | (chunk_of[s] << 11) | g);
      if (chunk_of[s] == 0 && k == K_F) open[d] += 1;
      if (chunk_of[s] == 0 && k == K_B) open[d] -= 1;
      left -= 1;
    }
  }
  if (P->swap_per_mille > 0 && rng_below(&rng, 1000) < P->swap_per_mille) {
    const int d = rng_below(&rng, D);
    if (len[d] >= 2) {
      const int a = rng_below(&rng, len[d]), span = 1 + rng_below(&rng, 12);
      const int b = a + span < len[d] ? a + span : len[d] - 1;
      const uint16_t x = out[(size_t)d * stride + a];
      out[(size_t)d * stride + a] = out[(size_t)d * stride + b];
      out[(size_t)d * stride + b] = x;
    }
  }
  free(step_of);
  free(next);
  return 0;
}

/* candidates [first, first + n) -> out[n][D][stride].  Returns 0, or -1 for a bad description. */
int fpsyncgen_generate(const fpsyncgen_params *P, int64_t first, int64_t n, int32_t stride, uint16_t *out) {
  if (P->n_devices < 1 || P->n_devices > MAX_D || P->n_stages < 1 || P->n_stages > MAX_S ||
      P->n_microbatches < 1 || P->n_microbatches > 2048 || stride < 1) return -1;
  int32_t cnt[MAX_D] = {0};
  for (int s = 0; s < P->n_stages; ++s) {
    const int d = P->stage_device[s];
    if (d < 0 || d >= P->n_devices || ++cnt[d] > MAX_CHUNKS || P->group[s] < 1) return -1;
  }
  for (int64_t i = 0; i < n; ++i)
    if (generate_one(P, first + i, stride, out + (size_t)i * P->n_devices * stride)) return -1;
  return 0;
}

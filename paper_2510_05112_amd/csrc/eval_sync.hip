// Evaluation with synchronisation stages and dependency pairs.
//
// Paper basis: a user may register a new instruction -- the synchronisation that exchanges the output
// states of the submodules of a multimodal model -- attached to a stage registered for it, say how many
// of the instructions it depends on must come first (one synchronisation every few micro-batches), and
// add dependencies as pairs ((type1, stage_i), (type2, stage_j)) (Section 4.2, registration of new
// instructions; Sections 2.2 and 7.2).  Here a stage has a group size n: it has ceil(m / n) items per
// kind, item g stands for the micro-batches g n .. min(m, (g + 1) n) - 1, and an item waits, along a DAG
// edge or a pair, for every item of the other stage whose micro-batches overlap its own.
//
// The kernel is the table form of the evaluator: one wavefront per workgroup, `cands_per_wave`
// candidates per wavefront, lane = device; the finish times of forward, backward (and, if a pair asks
// for them, weight-gradient) items per (stage, item) and the activation states live in LDS; a lane whose
// next op cannot issue waits for a later round; a round in which no lane of a candidate moves ends it.
// All dependencies of an item, DAG edges and pairs alike, are one list per (kind, stage).  Op words
// reach a lane eight at a time (one 16-byte load, the next one requested while these are used).
//
// Start rule: start = max(device free, finish of every item waited for + latency if it ran on another
// device); finish = start + dur[kind][stage].
//
// COPY = true is the copy-engine form of the cost model (the paper names CPU offloading without saying
// how an offload is timed; in the plain model offload and reload items run on the compute timeline):
// offload (O) and reload (L) items run on a copy timeline of their own.  The walk through the list hands
// such an item to the engine when it reaches it and goes on at once, unless `copy_depth` transfers are
// still unfinished: then it waits for the oldest of them.  A transfer starts at max(hand-over, finish of
// the transfer before it); a backward item waits for the reload of its activation (a table of its own);
// the makespan covers both timelines; the costs of transfers are not busy time.  Memory becomes a sum over
// events in time order (allocations at the start of F, FD, R, L; releases at the end of FD, O, W or B);
// at equal times the compute timeline's events come first.  The walk produces compute events in time
// order and knows every transfer's event time at hand-over, so a lane keeps the transfer events that lie
// ahead of the walk in a small ring (at most copy_depth + 1: transfers cost at least 1) and applies them
// as the walk passes their time.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

namespace fpsched {

template <bool COPY>
__global__ __launch_bounds__(64) void eval_sync_kernel(
    SyncTables T, const uint16_t* __restrict__ ops, long long n_cand, int stride,
    long long* __restrict__ out_makespan, long long* __restrict__ out_idle,
    int* __restrict__ out_peak, unsigned char* __restrict__ out_flags) {
  extern __shared__ int32_t lds[];
  const int lane = threadIdx.x;
  const int S = T.S, m = T.m, SM = S * m;
  const int fin_ints = T.n_fin_tables * SM;
  // COPY: behind the finish times, the time each activation became resident again (0 = never reloaded)
  const int per_cand_ints = fin_ints + (COPY ? SM : 0) + ((SM + 3) >> 2);
  const int cpw = T.cands_per_wave;
  const int lpc = T.lanes_per_cand;
  const int lpc_shift = __ffs(lpc) - 1;

  for (int i = lane; i < T.n_table_ints; i += 64) lds[i] = T.ints[i];
  int32_t* cand_base = lds + T.n_table_ints;
  for (int c = 0; c < cpw; ++c) {
    int32_t* p = cand_base + c * per_cand_ints;
    for (int i = lane; i < fin_ints; i += 64) p[i] = -1;
    for (int i = fin_ints + lane; i < per_cand_ints; i += 64) p[i] = 0;   // reload times, states
  }
  __syncthreads();

  const int32_t* tab = lds;
  const int seg = lane >> lpc_shift;
  const int d = lane & (lpc - 1);
  const long long cand = (long long)blockIdx.x * cpw + seg;
  const bool active = (seg < cpw) && (d < T.D) && (cand < n_cand);
  int32_t* fin = cand_base + (seg < cpw ? seg : 0) * per_cand_ints;   // [table][stage][item]
  int32_t* resident_at = fin + fin_ints;
  unsigned char* state = reinterpret_cast<unsigned char*>(fin + fin_ints + (COPY ? SM : 0));
  // COPY: per lane, behind all candidates' tables: the finish times of the last eight transfers and a ring
  // of eight pending memory events (time, units), each [entry][lane]
  int32_t* copy_fin = cand_base + cpw * per_cand_ints + lane;
  int32_t* ev_time = copy_fin + 8 * 64;
  int32_t* ev_units = ev_time + 8 * 64;
  int copy_free = 0, n_copy = 0;
  unsigned ev_head = 0, ev_tail = 0;

  const int dd = active ? d : 0;
  const int nch = tab[T.off_n_chunks + dd];
  const int cap = tab[T.off_mem_cap + dd];
  const uint16_t* row = ops + ((size_t)(active ? cand : 0) * T.D + dd) * (size_t)stride;
  const unsigned long long seg_mask = (lpc == 64 ? ~0ull : ((1ull << lpc) - 1ull)) << (seg * lpc);
  const unsigned free_mask = (1u << kFD) | (1u << kO) | (T.has_w ? (1u << kW) : (1u << kB));
  const int terminal_kind = T.has_w ? kW : kB;
  // items this device has to take to their last state
  int n_expected = 0;
  for (int c = 0; c < nch; ++c) n_expected += tab[T.off_items + tab[T.off_local_stage + dd * kMaxChunks + c]];

  // op words: eight in registers (stride is a multiple of 8, rows are 16-byte aligned), the next eight on
  // their way
  uint4 cur = make_uint4(0, 0, 0, 0), nxt = make_uint4(0, 0, 0, 0);
  if (active) {
    cur = *reinterpret_cast<const uint4*>(row);
    if (stride > 8) nxt = *reinterpret_cast<const uint4*>(row + 8);
  }
  auto word_at = [&](int k) -> unsigned {   // word k & 7 of `cur`
    // (two selects and a 64-bit shift: as a select among the four dwords the compiler moves `cur` to scratch
    // memory and loads the dword from there)
    const unsigned lo = (k & 4) ? cur.z : cur.x, hi = (k & 4) ? cur.w : cur.y;
    const unsigned long long half = ((unsigned long long)hi << 32) | lo;
    return (unsigned)(half >> ((k & 3) << 4)) & 0xffffu;
  };

  int cursor = 0, free_at = 0, busy = 0, mem = 0, pk = 0, n_term = 0;
  bool done = !active, bad = false, seg_live = true;
  unsigned w = active ? word_at(0) : 0u;
  // COPY: apply the pending transfer events that come before a compute event at time `limit`
  auto pass_time = [&](int limit) {
    while (ev_head != ev_tail && ev_time[(ev_head & 7u) * 64] < limit) {
      mem += ev_units[(ev_head & 7u) * 64];
      pk = max(pk, mem);
      ++ev_head;
    }
  };

  for (;;) {
    bool progressed = false;
    if (!done && seg_live) {
      const int kind = w >> 13;
      if (kind == kEnd) {
        done = true;
        progressed = true;
        if (COPY) pass_time(0x7fffffff);
      } else {
        const int c = (w >> 11) & 3, g = w & 0x7ff;
        const int s = c < nch ? tab[T.off_local_stage + d * kMaxChunks + c] : 0;
        if (c >= nch || g >= tab[T.off_items + s] || (kind == kW && !T.has_w)) {
          bad = true;
        } else {
          const int idx = s * m + g;
          const int st = state[idx];
          const int need = (0x03124100u >> (4 * kind)) & 0xf;
          if (st == need) {
            int ready = 0;
            bool blocked = false;
            const int e1 = tab[T.off_dep_off + kind * S + s + 1];
            int e = tab[T.off_dep_off + kind * S + s];
            if (e < e1) {
              // the micro-batches of this item (g < items of s, so lo < m)
              const int ns = tab[T.off_group + s];
              const int lo = g * ns, hi = min(m, lo + ns) - 1;
              for (; e < e1; ++e) {
                const int32_t* dep = tab + T.off_dep + 3 * e;
                const int a = dep[1], lat = dep[2];
                const int na = tab[T.off_group + a];
                const int32_t* from = fin + dep[0] * SM + a * m;
                // (hi <= m - 1, so every index stays below the item count of stage a)
                for (int ga = lo / na; ga <= hi / na; ++ga) {
                  const int t = from[ga];
                  if (t < 0) blocked = true;
                  ready = max(ready, t + lat);
                }
              }
            }
            if (COPY && kind == kB) ready = max(ready, resident_at[idx]);
            if (!blocked && COPY && (kind == kO || kind == kL)) {
              // a transfer: hand it over (waiting for room in the engine), time it on the copy timeline
              const int dt = tab[T.off_dur + kind * S + s];
              const int u = tab[T.off_mem_units + s];
              int handover = free_at;
              if (n_copy >= T.copy_depth) handover = max(handover, copy_fin[((unsigned)(n_copy - T.copy_depth) & 7u) * 64]);
              const int start = max(handover, copy_free);
              copy_free = start + dt;
              copy_fin[((unsigned)n_copy & 7u) * 64] = copy_free;
              ++n_copy;
              free_at = handover;
              pass_time(handover);
              ev_time[(ev_tail & 7u) * 64] = kind == kL ? start : copy_free;
              ev_units[(ev_tail & 7u) * 64] = kind == kL ? u : -u;
              ++ev_tail;
              if (kind == kL) resident_at[idx] = copy_free;
              state[idx] = (unsigned char)((0x21315410u >> (4 * kind)) & 0xf);
            } else if (!blocked) {
              const int dt = tab[T.off_dur + kind * S + s];
              const int u = tab[T.off_mem_units + s];
              const int finish = max(free_at, ready) + dt;
              if ((0xD2u >> kind) & 1u) {  // F, R, L, FD allocate at their start
                if (COPY) pass_time(finish - dt);
                mem += u;
                pk = max(pk, mem);
              }
              if ((free_mask >> kind) & 1u) {
                if (COPY) pass_time(finish);
                mem -= u;
              }
              state[idx] = (unsigned char)((0x21315410u >> (4 * kind)) & 0xf);
              if (kind == kF || kind == kFD) fin[idx] = finish;
              else if (kind == kB) fin[SM + idx] = finish;
              else if (kind == kW && T.n_fin_tables > 2) fin[2 * SM + idx] = finish;
              free_at = finish;
              busy += dt;
              if (COPY) pass_time(finish);
            }
            if (!blocked) {
              n_term += (kind == terminal_kind);
              ++cursor;
              if ((cursor & 7) == 0) {
                cur = nxt;
                if (cursor + 8 < stride) nxt = *reinterpret_cast<const uint4*>(row + cursor + 8);
              }
              w = (cursor < stride) ? word_at(cursor) : 0u;
              progressed = true;
            }
          }
        }
      }
    }
    __builtin_amdgcn_wave_barrier();
    const unsigned long long moved = __ballot(progressed);
    if ((moved & seg_mask) == 0ull) seg_live = false;
    if (moved == 0ull) break;
  }

  const unsigned long long stuck = __ballot(active && !done) & seg_mask;
  const unsigned long long stuck_bad = __ballot(active && !done && bad) & seg_mask;
  const unsigned long long unfinished = __ballot(active && n_term != n_expected) & seg_mask;
  const unsigned long long over = __ballot(active && pk > cap) & seg_mask;
  int ms = active ? (COPY ? max(free_at, copy_free) : free_at) : 0;
  for (int off = 1; off < lpc; off <<= 1) ms = max(ms, __shfl_xor(ms, off, 64));

  unsigned fl = 0;
  if (stuck) fl = kDeadlock | (stuck_bad ? kIncomplete : 0);
  else if (unfinished) fl = kIncomplete;
  else if (over) fl = kOverCap;
  if (active) {
    const bool failed = (fl & (kDeadlock | kIncomplete)) != 0;
    out_idle[cand * T.D + d] = failed ? -1ll : (long long)(ms - busy);
    out_peak[cand * T.D + d] = failed ? -1 : pk;
    if (d == 0) {
      out_makespan[cand] = failed ? 0x7fffffffffffffffll : (long long)ms;
      out_flags[cand] = (unsigned char)fl;
    }
  }
}

template __global__ void eval_sync_kernel<false>(SyncTables, const uint16_t*, long long, int, long long*, long long*,
                                                 int*, unsigned char*);
template __global__ void eval_sync_kernel<true>(SyncTables, const uint16_t*, long long, int, long long*, long long*,
                                                int*, unsigned char*);

}  // namespace fpsched

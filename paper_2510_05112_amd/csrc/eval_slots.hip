// Slot evaluation kernel: the main path.  Any per-device op order, any stage DAG,
// with a few KB of LDS per candidate instead of a finish-time table.
//
// Mapping: one wavefront owns `slot_cands_per_wave` candidates, lane = device inside
// a candidate; four independent wavefronts share a workgroup (and one LDS copy of
// the problem tables).  Each lane walks its device's list with a cursor in
// registers; a lane whose next op cannot issue yet waits for a later round, and a
// round in which no lane of a candidate moves ends that candidate (lists
// exhausted, or deadlock).
//
// Cross-stage finish times travel through per-micro-batch mail slots.  The edges
// of the stage DAG are split on the host into classes (chains of edges in which
// each edge starts at, or downstream of, the stage the previous one ends in; a
// plain pipeline is one class).  For one micro-batch at most one edge of a class
// carries a live value at a time -- the value of F(a,j) on edge a->b is dead once
// F(b,j) has issued, and only then can anything further down the class be produced --
// so a class needs ONE slot per micro-batch and direction, tagged with the stage
// that produced it: slot[dir][class][j] = (finish, producer stage).  A consumer
// finds its input iff the tag names its upstream stage.  No order of micro-batches
// is assumed and a producer never has to wait for room.
//
// Same-device ordering rules are the activation state machine of one
// (stage, micro-batch), 4 bits per entry, in lane-private LDS words.  Op words are
// staged through a lane-private 32-word LDS ring that the whole wavefront tops up
// with 16-byte global loads every eighth round; the load issued at one top-up is
// only written to LDS at the next, so its latency is off the critical path.
//
// Start rule (paper Section 5.1 "Data dependency"; estimator sketch after Section
// 6): start = max(device free, finish of each cross-stage input + latency if the
// input ran on another device); finish = start + dur[kind][stage].
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

namespace fpsched {

namespace {

template <int V>
__device__ __forceinline__ int pick(const int (&a)[V], int c) {
  int r = a[0];
#pragma unroll
  for (int i = 1; i < V; ++i) r = (c == i) ? a[i] : r;
  return r;
}

}  // namespace

template <int V>
__global__ __launch_bounds__(kSlotThreads) void eval_slot_kernel(
    DevTables T, const uint16_t* __restrict__ ops, long long n_cand, int stride,
    long long* __restrict__ out_makespan, long long* __restrict__ out_idle,
    int* __restrict__ out_peak, unsigned char* __restrict__ out_flags) {
  extern __shared__ int32_t lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int S = T.S, m = T.m, ncls = T.n_classes;
  const int cpw = T.slot_cands_per_wave;
  const int lpc = T.lanes_per_cand;
  const int lpc_shift = __ffs(lpc) - 1;

  for (int i = tid; i < T.n_table_ints; i += kSlotThreads) lds[i] = T.ints[i];
  uint32_t* win = reinterpret_cast<uint32_t*>(lds + T.table_ints_padded + wave * T.wave_ints);
  uint32_t* stt = win + 16 * 64;
  int2* slots = reinterpret_cast<int2*>(stt + T.state_words * 64);
  const int slots_per_cand = 2 * ncls * m;
  for (int i = lane; i < T.state_words * 64; i += 64) stt[i] = 0u;
  for (int i = lane; i < cpw * slots_per_cand; i += 64) slots[i] = make_int2(0, -1);
  __syncthreads();

  const int32_t* tab = lds;
  const int seg = lane >> lpc_shift;
  const int d = lane & (lpc - 1);
  const long long cand = ((long long)blockIdx.x * kSlotWaves + wave) * cpw + seg;
  const bool active = (seg < cpw) && (d < T.D) && (cand < n_cand);
  int2* fwd_slot = slots + (seg < cpw ? seg : 0) * slots_per_cand;
  int2* bwd_slot = fwd_slot + ncls * m;

  const int dd = active ? d : 0;
  const int nch = tab[T.off_n_chunks + dd];
  const int cap = tab[T.off_mem_cap + dd];
  int stage_of[V], units_of[V];
#pragma unroll
  for (int c = 0; c < V; ++c) {
    const int s = tab[T.off_local_stage + dd * kMaxChunks + c];
    stage_of[c] = s < 0 ? 0 : s;
    units_of[c] = tab[T.off_mem_units + stage_of[c]];
  }
  const uint16_t* row = ops + ((size_t)(active ? cand : 0) * T.D + dd) * (size_t)stride;
  const unsigned long long seg_mask =
      (lpc == 64 ? ~0ull : ((1ull << lpc) - 1ull)) << (seg * lpc);
  const unsigned free_mask = (1u << kFD) | (1u << kO) | (T.has_w ? (1u << kW) : (1u << kB));
  const int terminal_kind = T.has_w ? kW : kB;

  // prime the op window with the first 16 words of the row
  int loaded = 0;  // words of this row already in the window ring
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    if (active && loaded < stride) {
      const uint4 v = *reinterpret_cast<const uint4*>(row + loaded);
      win[(q * 4 + 0) * 64 + lane] = v.x;
      win[(q * 4 + 1) * 64 + lane] = v.y;
      win[(q * 4 + 2) * 64 + lane] = v.z;
      win[(q * 4 + 3) * 64 + lane] = v.w;
      loaded += 8;
    }
  }
  uint4 pend = make_uint4(0, 0, 0, 0);
  bool has_pend = false;

  int cursor = 0, free_at = 0, busy = 0, mem = 0, pk = 0, n_term = 0;
  bool done = !active, bad = false, seg_live = true;

  for (unsigned round = 0;; ++round) {
    if ((round & 7u) == 0u) {
      // wave-wide top-up: land the chunk requested eight rounds ago, request the next
      if (has_pend) {
        const int q = (loaded >> 3) & 3;
        win[(q * 4 + 0) * 64 + lane] = pend.x;
        win[(q * 4 + 1) * 64 + lane] = pend.y;
        win[(q * 4 + 2) * 64 + lane] = pend.z;
        win[(q * 4 + 3) * 64 + lane] = pend.w;
        loaded += 8;
        has_pend = false;
      }
      if (!done && loaded - cursor <= 16 && loaded < stride) {
        pend = *reinterpret_cast<const uint4*>(row + loaded);
        has_pend = true;
      }
    }
    bool progressed = false;
    if (!done && seg_live) {
      unsigned w = 0u;
      if (cursor < stride) {
        const unsigned x = win[((cursor >> 1) & 15) * 64 + lane];
        w = (cursor & 1) ? (x >> 16) : (x & 0xffffu);
      }
      const int kind = w >> 13;
      if (kind == kEnd) {
        done = true;
        progressed = true;
      } else {
        const int c = (w >> 11) & 3, j = w & 0x7ff;
        if (c >= nch || j >= m || (kind == kW && !T.has_w)) {
          bad = true;
        } else {
          const int s = pick<V>(stage_of, c);
          const int idx = c * m + j;
          const int sw = (idx >> 3) * 64 + lane;
          const int sh = (idx & 7) * 4;
          const unsigned sx = stt[sw];
          const unsigned st = (sx >> sh) & 15u;
          const unsigned need = (0x03124100u >> (4 * kind)) & 15u;
          if (st == need) {
            int ready = 0;
            bool blocked = false;
            if (kind == kF || kind == kFD) {
              const int e1 = tab[T.off_pred_off + s + 1];
              for (int e = tab[T.off_pred_off + s]; e < e1; ++e) {
                const int2 v = fwd_slot[tab[T.off_pred_cls + e] * m + j];
                if (v.y != tab[T.off_pred_stage + e]) blocked = true;
                ready = max(ready, v.x + tab[T.off_pred_comm + e]);
              }
            } else if (kind == kB) {
              const int e1 = tab[T.off_succ_off + s + 1];
              for (int e = tab[T.off_succ_off + s]; e < e1; ++e) {
                const int2 v = bwd_slot[tab[T.off_succ_cls + e] * m + j];
                if (v.y != tab[T.off_succ_stage + e]) blocked = true;
                ready = max(ready, v.x + tab[T.off_succ_comm + e]);
              }
            }
            if (!blocked) {
              const int dt = tab[T.off_dur + kind * S + s];
              const int u = pick<V>(units_of, c);
              const int fin = max(free_at, ready) + dt;
              if ((0xD2u >> kind) & 1u) {  // F, R, L, FD allocate at their start
                mem += u;
                pk = max(pk, mem);
              }
              if ((free_mask >> kind) & 1u) mem -= u;
              const unsigned next = (0x21315410u >> (4 * kind)) & 15u;
              stt[sw] = sx ^ ((st ^ next) << sh);
              if (kind == kF || kind == kFD) {
                const int e1 = tab[T.off_succ_off + s + 1];
                for (int e = tab[T.off_succ_off + s]; e < e1; ++e)
                  fwd_slot[tab[T.off_succ_cls + e] * m + j] = make_int2(fin, s);
              } else if (kind == kB) {
                const int e1 = tab[T.off_pred_off + s + 1];
                for (int e = tab[T.off_pred_off + s]; e < e1; ++e)
                  bwd_slot[tab[T.off_pred_cls + e] * m + j] = make_int2(fin, s);
              }
              n_term += (kind == terminal_kind);
              free_at = fin;
              busy += dt;
              ++cursor;
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
  const unsigned long long unfinished = __ballot(active && n_term != nch * m) & seg_mask;
  const unsigned long long over = __ballot(active && pk > cap) & seg_mask;
  int ms = active ? free_at : 0;
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

template __global__ void eval_slot_kernel<1>(DevTables, const uint16_t*, long long, int, long long*,
                                             long long*, int*, unsigned char*);
template __global__ void eval_slot_kernel<2>(DevTables, const uint16_t*, long long, int, long long*,
                                             long long*, int*, unsigned char*);
template __global__ void eval_slot_kernel<4>(DevTables, const uint16_t*, long long, int, long long*,
                                             long long*, int*, unsigned char*);

}  // namespace fpsched

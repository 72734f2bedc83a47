// Slot evaluation kernel: the main path.  Any per-device op order, any stage DAG with
// at most two inputs and two outputs per stage, a few KB of LDS per candidate.
//
// Mapping: one wavefront owns `slot_cands_per_wave` candidates, lane = device inside a
// candidate; four independent wavefronts share a workgroup (and one LDS copy of the
// op-metadata table).  Each lane walks its device's list with a cursor in registers; a
// lane whose next op cannot issue yet waits for a later round, and a round in which no
// lane of a candidate moves ends that candidate (lists exhausted, or deadlock).
//
// Cross-stage finish times travel through per-micro-batch mail slots.  The edges of
// the stage DAG are split on the host into classes (chains of edges in which each edge
// starts at the stage the previous one ends in; a plain pipeline is one class).  For
// one micro-batch at most one edge of a class carries a live value at a time -- the
// value of F(a,j) on edge a->b is dead once F(b,j) has issued, and only then can the
// next edge of the class be produced -- so a class needs ONE slot per micro-batch and
// direction, tagged with the stage that produced it: slot[dir][class][j] = (finish,
// producer stage).  A consumer finds its input iff the tag names its upstream stage.
// No order of micro-batches is assumed and a producer never has to wait for room.
//
// Same-device ordering rules are the activation state machine of one (stage,
// micro-batch), 4 bits per entry, in lane-private LDS words.  Op words are staged
// through a lane-private 32-word LDS ring that the whole wavefront tops up with
// 16-byte global loads every eighth round; the load issued at one top-up is only
// written to LDS at the next, so its latency is off the critical path.
//
// A round is straight-line code: the LDS reads of a round (next op word, op metadata,
// state word, input slots) depend only on registers and are issued together, so a
// round costs one LDS round trip.
//
// Start rule (paper Section 5.1 "Data dependency"; estimator sketch after Section 6):
// start = max(device free, finish of each cross-stage input + latency if the input ran
// on another device); finish = start + dur[kind][stage].
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

template <int V, bool DEG2>
__global__ __launch_bounds__(kSlotThreads) void eval_slot_kernel(
    SlotTables T, const uint16_t* __restrict__ ops, long long n_cand, int stride,
    long long* __restrict__ out_makespan, long long* __restrict__ out_idle,
    int* __restrict__ out_peak, unsigned char* __restrict__ out_flags) {
  extern __shared__ int32_t lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m = T.m;
  const int cpw = T.cands_per_wave;
  const int lpc = T.lanes_per_cand;
  const int lpc_shift = __ffs(lpc) - 1;

  // shared: op metadata (+ second-edge metadata); per wave: window, state words, slots
  for (int i = tid; i < T.n_shared_ints; i += kSlotThreads) lds[i] = T.ints[i];
  const int4* meta = reinterpret_cast<const int4*>(lds);
  const int2* meta2 = reinterpret_cast<const int2*>(lds + T.off_meta2);
  uint32_t* win = reinterpret_cast<uint32_t*>(lds + T.n_shared_ints + wave * T.wave_ints);
  uint32_t* stt = win + 16 * 64;
  int2* slots = reinterpret_cast<int2*>(stt + T.state_words * 64);
  const int slots_per_cand = 2 * T.n_classes * m;
  for (int i = lane; i < T.state_words * 64; i += 64) stt[i] = 0u;
  for (int i = lane; i < cpw * slots_per_cand; i += 64) slots[i] = make_int2(0, -1);
  __syncthreads();

  const int seg = lane >> lpc_shift;
  const int d = lane & (lpc - 1);
  const long long cand = ((long long)blockIdx.x * kSlotWaves + wave) * cpw + seg;
  const bool active = (seg < cpw) && (d < T.D) && (cand < n_cand);
  int2* my_slots = slots + (seg < cpw ? seg : 0) * slots_per_cand;

  // per-device constants: chunk count, cap, slot offsets of the inputs of each chunk
  const int32_t* dev = T.ints + T.off_dev + d * T.dev_ints;
  const int nch = dev[0];
  const int cap = dev[1];
  int cons_f[V], cons_b[V], cons_f2[V], cons_b2[V];
#pragma unroll
  for (int c = 0; c < V; ++c) {
    cons_f[c] = dev[2 + c];
    cons_b[c] = dev[2 + V + c];
    cons_f2[c] = DEG2 ? dev[2 + 2 * V + c] : 0;
    cons_b2[c] = DEG2 ? dev[2 + 3 * V + c] : 0;
  }
  const int dd = active ? d : 0;
  const uint16_t* row = ops + ((size_t)(active ? cand : 0) * T.D + dd) * (size_t)stride;
  const unsigned long long seg_mask =
      (lpc == 64 ? ~0ull : ((1ull << lpc) - 1ull)) << (seg * lpc);

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
  unsigned w = (active && stride > 0) ? (win[lane] & 0xffffu) : 0u;

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
      if (!done && loaded - cursor <= 17 && loaded < stride) {
        pend = *reinterpret_cast<const uint4*>(row + loaded);
        has_pend = true;
      }
    }
    // ---- decode the current word (already in a register) and issue this round's reads
    const int kind = w >> 13;
    const int c = (w >> 11) & 3;
    const int j = w & 0x7ff;
    const bool is_b = kind == kB;
    const int nxt = cursor + 1;
    const unsigned nx = win[((nxt >> 1) & 15) * 64 + lane];
    const int cc = c < V ? c : 0;
    const int4 M = meta[(kind * V + cc) * lpc + d];
    const int jj = j < m ? j : 0;
    const int idx = cc * m + jj;
    const int sw = (idx >> 3) * 64 + lane;
    const int sh = (idx & 7) * 4;
    const unsigned sx = stt[sw];
    const int coff = is_b ? pick<V>(cons_b, c) : pick<V>(cons_f, c);
    const int2 in1 = my_slots[coff + jj];
    int2 M2 = make_int2(0, 0), in2 = make_int2(0, 0);
    if (DEG2) {
      M2 = meta2[((is_b ? V : 0) + cc) * lpc + d];
      const int coff2 = is_b ? pick<V>(cons_b2, c) : pick<V>(cons_f2, c);
      in2 = my_slots[coff2 + jj];
    }
    // ---- decide
    const unsigned fl = (unsigned)M.z;
    const bool live = !done && seg_live;
    const bool is_end = kind == kEnd;
    const bool wellformed = !(fl & kMetaInvalid) && j < m && c < nch;
    const unsigned st = (sx >> sh) & 15u;
    bool ok = live && !is_end && wellformed && st == ((unsigned)M.w & 15u);
    int ready = 0;
    if (fl & kMetaHasCons) {
      ok = ok && in1.y == (int)((fl >> 16) & 0xffu);
      ready = in1.x + M.y;
    }
    if (DEG2) {
      if ((unsigned)M2.y & kMetaHasCons) {
        ok = ok && in2.y == (int)(((unsigned)M2.y >> 16) & 0xffu);
        ready = max(ready, in2.x + M2.x);
      }
    }
    const bool newly_done = live && is_end;
    done = done || newly_done;
    bad = bad || (live && !is_end && !wellformed);
    // ---- issue
    if (ok) {
      const int dt = M.x;
      const int u = (int)((unsigned)M.w >> 16);
      const int self = (int)(((unsigned)M.w >> 8) & 0xffu);
      const int fin = max(free_at, ready) + dt;
      mem += (fl & kMetaAlloc) ? u : 0;
      pk = max(pk, mem);
      mem -= (fl & kMetaFree) ? u : 0;
      stt[sw] = sx ^ ((st ^ (((unsigned)M.w >> 4) & 15u)) << sh);
      if (fl & kMetaHasProd) my_slots[(fl & 0xffffu) + j] = make_int2(fin, self);
      if (DEG2) {
        if ((unsigned)M2.y & kMetaHasProd) my_slots[((unsigned)M2.y & 0xffffu) + j] = make_int2(fin, self);
      }
      n_term += (fl & kMetaTerminal) ? 1 : 0;
      free_at = fin;
      busy += dt;
      cursor = nxt;
      w = nxt < stride ? ((nxt & 1) ? (nx >> 16) : (nx & 0xffffu)) : 0u;
    }
    __builtin_amdgcn_wave_barrier();
    const unsigned long long moved = __ballot(ok || newly_done);
    if ((moved & seg_mask) == 0ull) seg_live = false;
    if (moved == 0ull) break;
  }

  const unsigned long long stuck = __ballot(active && !done) & seg_mask;
  const unsigned long long stuck_bad = __ballot(active && !done && bad) & seg_mask;
  const unsigned long long unfinished = __ballot(active && n_term != nch * m) & seg_mask;
  const unsigned long long over = __ballot(active && pk > cap) & seg_mask;
  int ms = active ? free_at : 0;
  for (int off = 1; off < lpc; off <<= 1) ms = max(ms, __shfl_xor(ms, off, 64));

  unsigned flg = 0;
  if (stuck) flg = kDeadlock | (stuck_bad ? kIncomplete : 0);
  else if (unfinished) flg = kIncomplete;
  else if (over) flg = kOverCap;
  if (active) {
    const bool failed = (flg & (kDeadlock | kIncomplete)) != 0;
    out_idle[cand * T.D + d] = failed ? -1ll : (long long)(ms - busy);
    out_peak[cand * T.D + d] = failed ? -1 : pk;
    if (d == 0) {
      out_makespan[cand] = failed ? 0x7fffffffffffffffll : (long long)ms;
      out_flags[cand] = (unsigned char)flg;
    }
  }
}

#define FPSCHED_INSTANTIATE(V, G)                                                               \
  template __global__ void eval_slot_kernel<V, G>(SlotTables, const uint16_t*, long long, int,  \
                                                  long long*, long long*, int*, unsigned char*);
FPSCHED_INSTANTIATE(1, false)
FPSCHED_INSTANTIATE(2, false)
FPSCHED_INSTANTIATE(4, false)
FPSCHED_INSTANTIATE(1, true)
FPSCHED_INSTANTIATE(2, true)
FPSCHED_INSTANTIATE(4, true)
#undef FPSCHED_INSTANTIATE

}  // namespace fpsched

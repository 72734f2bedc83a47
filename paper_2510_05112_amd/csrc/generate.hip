// Schedule generator kernel: the actor-aware schedule of the paper's Section 5 for a batch of
// parameter sets, one schedule per set.
//
// The scheduling process is step-synchronous by definition (Section 5.2, Steps 2-5: in a step
// every actor runs the step function of Algorithm 1 on the state the previous step left, and
// what an actor schedules stays in its local buffer until the step is over), which is the shape
// of a wavefront: lane = actor, `64 / pow2(D)` parameter sets per wavefront, one step = one pass
// of straight-line code with a read phase and a write phase.
//
// State.  Items of one instruction type and stage are scheduled in ascending micro-batch order
// and become dependency-free in that order as well (a forward item needs the same micro-batch
// of the upstream stages, a backward item the same micro-batch of the own forward pass and of
// the downstream backward passes, a weight-gradient item its backward item), so the instruction
// pool and the reorder queues of Section 5.1 reduce to one counter per (type, stage): the number
// of micro-batches scheduled so far.  The next item of (type, stage) is in its reorder queue iff
// every counter it depends on is ahead of its own.  The counters of a parameter set live in LDS;
// a lane reads those of its stages' neighbours in the read phase and bumps at most one of its
// own in the write phase.
//
// Priorities (Section 5.2; Table of built-in values): computation type traversal priority
// bwdpass-first / fwdpass-first / interleaved(unit1, unit2); stage traversal priority
// breadth-first / depth-first with an optional interval, separately for forward and backward
// items; the check function is the per-stage limit of in-flight micro-batches (Section 4.2,
// config_inflight_micros).  How the corners are read (type fallback, when an interval position
// moves, weight-gradient items last) is stated with the host declaration of fpsched_generate.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

namespace fpsched {

namespace {

enum GenType : int { kGenF = 0, kGenB = 1, kGenW = 2 };

// lowest / highest set bit of a non-zero 4-bit mask
__device__ __forceinline__ int low_bit(unsigned x) { return __ffs(x) - 1; }
__device__ __forceinline__ int high_bit(unsigned x) { return 31 - __clz(x); }

}  // namespace

template <int V>
__global__ __launch_bounds__(64) void generate_kernel(DevTables T, const int32_t* __restrict__ policy,
                                                      const int32_t* __restrict__ inflight, long long n_sets,
                                                      int stride, uint16_t* __restrict__ ops,
                                                      int32_t* __restrict__ out_steps,
                                                      unsigned char* __restrict__ out_status) {
  extern __shared__ int32_t lds[];
  const int lane = threadIdx.x;
  const int S = T.S, m = T.m, D = T.D;
  const int lpc = T.lanes_per_cand;
  const int lpc_shift = __ffs(lpc) - 1;
  const int cpw = 64 >> lpc_shift;
  const int ntypes = T.has_w ? 3 : 2;
  // LDS: [problem tables][sets of the wavefront: counters [3][S]]
  for (int i = lane; i < T.n_table_ints; i += 64) lds[i] = T.ints[i];
  int32_t* counts = lds + T.n_table_ints;
  for (int i = lane; i < cpw * 3 * S; i += 64) counts[i] = 0;
  __syncthreads();
  const int32_t* pred_off = lds + T.off_pred_off;
  const int32_t* pred_stage = lds + T.off_pred_stage;
  const int32_t* succ_off = lds + T.off_succ_off;
  const int32_t* succ_stage = lds + T.off_succ_stage;

  const int seg = lane >> lpc_shift;
  const int d = lane & (lpc - 1);
  const long long set = (long long)blockIdx.x * cpw + seg;
  const bool has_row = set < n_sets && d < D;
  const unsigned long long seg_mask = (lpc == 64 ? ~0ull : ((1ull << lpc) - 1ull)) << (seg * lpc);
  int32_t* cnt = counts + seg * 3 * S;   // cnt[type * S + stage]

  const int nch = has_row ? lds[T.off_n_chunks + d] : 0;
  int stage[V], limit[V];
#pragma unroll
  for (int c = 0; c < V; ++c) {
    stage[c] = c < nch ? lds[T.off_local_stage + d * kMaxChunks + c] : 0;
    limit[c] = c < nch ? inflight[set * S + stage[c]] : 1;
  }
  int cttp = 0, unit_f = 1, unit_b = 1, f_dir = 0, f_int = 0, b_dir = 0, b_int = 0;
  if (has_row) {
    const int32_t* pol = policy + (set * D + d) * 8;
    cttp = pol[0]; unit_f = pol[1]; unit_b = pol[2];
    f_dir = pol[3]; f_int = pol[4]; b_dir = pol[5]; b_int = pol[6];
  }
  // a parameter set with a value outside its domain generates nothing (status 4)
  bool bad = cttp < 0 || cttp > 2 || unit_f < 1 || unit_b < 1 || f_dir < 0 || f_dir > 1 || f_int < 0 ||
             b_dir < 0 || b_dir > 1 || b_int < 0 || (cttp != 2 && (unit_f != 1 || unit_b != 1));
#pragma unroll
  for (int c = 0; c < V; ++c) bad = bad || limit[c] < 1;
  const bool set_bad = (__ballot(bad && has_row) & seg_mask) != 0ull;

  int turn_type = kGenF, turn_run = 0;
  int pos_f = f_dir == 0 ? 0 : (nch > 0 ? nch - 1 : 0), pos_b = b_dir == 0 ? 0 : (nch > 0 ? nch - 1 : 0);
  int stepped_f = 0, stepped_b = 0;
  int left = set_bad ? 0 : nch * m * ntypes;   // items this actor still has to schedule
  bool live = (__ballot(left > 0) & seg_mask) != 0ull;   // the set's process is still running
  int steps = 0, status = set_bad ? 4 : 0;
  int len = 0;
  unsigned buf0 = 0u, buf1 = 0u;   // up to four op words waiting for their 8-byte store
  uint16_t* row = ops + (size_t)(has_row ? set * D + d : 0) * (size_t)stride;

  // every step but the last of a set schedules at least one of its 3 S m items
  const long long max_steps = 3ll * S * m + 2;
  for (long long step = 0; step < max_steps; ++step) {
    if (__ballot(live) == 0ull) break;
    // ---- read phase: which of this actor's (type, stage) have their next item in the reorder
    // queue, and which of those pass the check function
    unsigned ready[3] = {0u, 0u, 0u}, ok_f = 0u;
    int own[3][V];
#pragma unroll
    for (int c = 0; c < V; ++c) {
      own[0][c] = own[1][c] = own[2][c] = 0;
      if (c < nch && live) {
        const int s = stage[c];
        const int nf = cnt[s], nb = cnt[S + s], nw = cnt[2 * S + s];
        own[0][c] = nf; own[1][c] = nb; own[2][c] = nw;
        int f_ahead = m;
        for (int e = pred_off[s]; e < pred_off[s + 1]; ++e) f_ahead = min(f_ahead, cnt[pred_stage[e]]);
        int b_ahead = nf;
        for (int e = succ_off[s]; e < succ_off[s + 1]; ++e) b_ahead = min(b_ahead, cnt[S + succ_stage[e]]);
        const unsigned bit = 1u << c;
        if (f_ahead > nf) { ready[0] |= bit; if (nf - nb < limit[c]) ok_f |= bit; }
        if (b_ahead > nb) ready[1] |= bit;
        if (ntypes == 3 && nb > nw) ready[2] |= bit;
      }
    }
    // ---- the step function: instruction types in priority order, stages in traversal order
    int pick_t = -1, pick_c = 0;
    const int first = cttp == 0 ? kGenB : (cttp == 1 ? kGenF : turn_type);
#pragma unroll
    for (int oi = 0; oi < 3; ++oi) {
      const int t = oi == 0 ? first : (oi == 1 ? (first == kGenF ? kGenB : kGenF) : kGenW);
      if (pick_t >= 0 || (oi == 2 && ntypes < 3)) continue;
      const unsigned rdy = t == kGenF ? ready[0] : (t == kGenB ? ready[1] : ready[2]);
      if (rdy == 0u) continue;   // this reorder queue is empty
      const unsigned ok = t == kGenF ? ok_f : rdy;
      const int dir = t == kGenF ? f_dir : (t == kGenB ? b_dir : 0);
      const int interval = t == kGenF ? f_int : (t == kGenB ? b_int : 0);
      if (ok == 0u) continue;    // nothing eligible of this type: try the next one
      if (interval > 0) {
        int p = t == kGenF ? pos_f : pos_b;
        int stepped = t == kGenF ? stepped_f : stepped_b;
        if (stepped == interval || !((ok >> p) & 1u)) {
          // move on, in the traversal direction, to the next stage with an eligible item
          for (int k = 0; k < V; ++k) {
            if (k >= nch) break;
            p = dir == 0 ? (p + 1 == nch ? 0 : p + 1) : (p == 0 ? nch - 1 : p - 1);
            if ((ok >> p) & 1u) break;
          }
          stepped = 0;
        }
        pick_t = t; pick_c = p; stepped += 1;
        if (t == kGenF) { pos_f = p; stepped_f = stepped; } else { pos_b = p; stepped_b = stepped; }
      } else {
        pick_t = t;
        pick_c = dir == 0 ? low_bit(ok) : high_bit(ok);
      }
    }
    __syncthreads();   // every lane has read the counters of this step
    // ---- write phase: the choice becomes visible for the next step
    if (pick_t >= 0) {
      int s = stage[0], j = own[0][0];
#pragma unroll
      for (int c = 0; c < V; ++c)
#pragma unroll
        for (int t = 0; t < 3; ++t)
          if (pick_c == c && pick_t == t) { s = stage[c]; j = own[t][c]; }
      cnt[pick_t * S + s] = j + 1;
      left -= 1;
      const unsigned word = ((unsigned)(pick_t + 1) << 13) | ((unsigned)pick_c << 11) | (unsigned)j;
      const int q = len & 3;
      if (q == 0) buf0 = word;
      else if (q == 1) buf0 |= word << 16;
      else if (q == 2) buf1 = word;
      else {
        buf1 |= word << 16;
        *reinterpret_cast<uint2*>(row + (len - 3)) = make_uint2(buf0, buf1);
        buf0 = 0u; buf1 = 0u;
      }
      len += 1;
      if (cttp == 2 && pick_t == turn_type) {
        if (++turn_run >= (pick_t == kGenF ? unit_f : unit_b)) { turn_type = pick_t == kGenF ? kGenB : kGenF; turn_run = 0; }
      }
    }
    const bool any_pick = (__ballot(pick_t >= 0) & seg_mask) != 0ull;
    const bool any_left = (__ballot(left > 0) & seg_mask) != 0ull;
    if (live) {
      if (!any_pick) { status = 1; live = false; }   // items remain and nothing can move
      else { steps += 1; live = any_left; }
    }
    __syncthreads();   // the counters written in this step are in place
  }
  // ---- rows are END-padded to the stride; words still waiting go out with the padding
  if (has_row) {
    int at = len & ~3;
    if (len & 3) {
      if (at < stride) *reinterpret_cast<uint2*>(row + at) = make_uint2(buf0, buf1);
      at += 4;
    }
    for (; at < stride; at += 4) *reinterpret_cast<uint2*>(row + at) = make_uint2(0u, 0u);
    if (d == 0) {
      out_steps[set] = steps;
      out_status[set] = (unsigned char)status;
    }
  }
}

template __global__ void generate_kernel<1>(DevTables, const int32_t*, const int32_t*, long long, int, uint16_t*,
                                            int32_t*, unsigned char*);
template __global__ void generate_kernel<2>(DevTables, const int32_t*, const int32_t*, long long, int, uint16_t*,
                                            int32_t*, unsigned char*);
template __global__ void generate_kernel<4>(DevTables, const int32_t*, const int32_t*, long long, int, uint16_t*,
                                            int32_t*, unsigned char*);

}  // namespace fpsched

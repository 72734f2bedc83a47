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
// a lane reads its own and those of its stages' neighbours in the read phase and bumps at most one
// of its own in the write phase (the old value is the item's micro-batch).
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
// two 16-bit counters side by side: those of an actor's two stages
typedef short pair16 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned bits_of(pair16 v) { return __builtin_bit_cast(unsigned, v); }
constexpr unsigned kBothSigns = 0x80008000u;

// one value per chunk of an actor, as one vector value (an array would be indexed in memory)
template <int V>
struct GenPerChunk { typedef int type __attribute__((ext_vector_type(V))); };
template <int V>
__device__ __forceinline__ int gen_pick(typename GenPerChunk<V>::type a, unsigned c) {
  int r = a[0];
#pragma unroll
  for (int i = 1; i < V; ++i) r = (c == (unsigned)i) ? a[i] : r;
  return r;
}

// a * b + c for a, b below 2^24, b the same in all lanes: one full-rate instruction
__device__ __forceinline__ unsigned mad24(unsigned a, unsigned b_uniform, unsigned c) {
  unsigned r;
  asm("v_mad_u32_u24 %0, %1, %2, %3" : "=v"(r) : "v"(a), "s"(b_uniform), "v"(c));
  return r;
}

}  // namespace

// V = bound on the stages per device (1, 2, 4).  DEG = bound on the DAG in- and out-degree of a
// stage (1 or 2): the LDS addresses of the neighbours' counters are then kept in registers;
// DEG = 0 walks the edge lists in LDS instead (any degree).
//
// The grid is persistent: a segment (the lanes of one parameter set) that finishes its schedule
// writes it out, draws the next set from a global counter and starts over while the other segments
// of the wavefront keep stepping, so that sets that need few and many steps balance out.
//
// TIMED: generator and evaluator in one (fpsched_generate_evaluate).  An item is scheduled only
// after everything it depends on was scheduled in an earlier step, so its start time is known the
// moment it is placed: start = max(the actor's free time, the inputs' finish + latency), exactly
// what fpsched_evaluate computes for the generated lists (Section 5.1 data dependency; the
// estimator's start / end / cost).  The inputs' finish times travel through the mail slots of the
// slot kernel, here plain int32 words without tags (the counters already say that the value is
// there); resident memory is counted as the items are placed.  No op word is formed, nothing but
// the results is written.  Workgroups hold several wavefronts that share the cost rows; each
// wavefront keeps its own counters and slots and never looks at another's, so no barrier is needed
// after the start.
//
// FORM kGenSlide: the timed form with the weight-gradient sliding pass of Section 5.2 (bubble optimizations) in
// it: the results fpsched_wslide_evaluate gives for the generated lists.  A W item that the scheduler places is
// passed over; a B item stashes its W item, and in front of every other item the actor runs the oldest
// stashed items that end before the item starts.  The stash is a queue of log2(V) bits per entry (the chunk):
// a head word and a tail word in registers, full words in between in a ring in LDS (kGenSpillWords per lane).
template <int V, int DEG, int FORM>
__global__ __launch_bounds__(FORM != kGenPlain ? kGenTimedThreads : 64) void generate_kernel(
    DevTables T, const int32_t* __restrict__ policy, const int32_t* __restrict__ inflight,
    const long long* __restrict__ select, long long n_src, long long n_sets, int stride, uint16_t* __restrict__ ops,
    int32_t* __restrict__ out_steps, unsigned char* __restrict__ out_status,
    unsigned long long* __restrict__ next_set, GenResults R) {
  constexpr bool TIMED = FORM != kGenPlain;
  constexpr bool SLIDE = FORM == kGenSlide;
  // SLIDE: bits per queue entry, entries per queue word
  constexpr unsigned kQBits = V == 1 ? 0u : (V == 2 ? 1u : 2u);
  constexpr unsigned kQCap = V == 1 ? 0x7fffffffu : 32u / (kQBits ? kQBits : 1u);
  extern __shared__ int32_t lds[];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6, waves_per_block = blockDim.x >> 6;
  const int S = T.S, m = T.m, D = T.D;
  const int lpc = T.lanes_per_cand;
  const int lpc_shift = __ffs(lpc) - 1;
  const int cpw = 64 >> lpc_shift;
  const bool has_w = T.has_w != 0;
  // LDS: [edge lists, only if DEG == 0 | cost rows, only if TIMED] then per wavefront
  // [sets of the wavefront: counters [3][S]][words holding m]
  // [row staging: 16 op words per lane, as 8 dwords laid out [dword][lane] | TIMED: the sets' slots]
  const int n_tab = TIMED ? 3 * V * D * 8 : (DEG == 0 ? T.n_table_ints : 0);
  if (TIMED) {
    for (int i = threadIdx.x; i < n_tab; i += blockDim.x) lds[i] = T.ints[T.off_gen_rows + i];
  } else if (DEG == 0) {
    for (int i = lane; i < n_tab; i += 64) lds[i] = T.ints[i];
  }
  const int n_count_ints = (cpw * 3 * S + 2 * S + 1 + 3) & ~3;
  const int slot_words = T.gen_slot_words;
  const int spill_words = SLIDE ? T.gen_spill_words : 0;   // per lane, a power of two
  int32_t* counts = lds + n_tab + wave * (n_count_ints + (TIMED ? cpw * slot_words + 64 * spill_words : 8 * 64));
  // counters that are always "done" (value m): at_m stands in for a missing neighbour, and at_m,
  // at_m + S, at_m + 2 S for the three counters of a chunk the actor does not have
  const int at_m = cpw * 3 * S;
  if (lane < 3) counts[at_m + lane * S] = m;
  // a lane collects 16 op words (32 bytes) of its row before it stores them: HBM is written in
  // 32-byte pieces, not a quarter of that
  uint32_t* staging = reinterpret_cast<uint32_t*>(counts + n_count_ints) + lane;   // dword i at + i * 64
  // TIMED: slots never hold anything but finish times (an item without an input reads some word of
  // them and adds -2^30)
  if (TIMED)
    for (int i = lane; i < cpw * slot_words; i += 64) counts[n_count_ints + i] = 0;
  __syncthreads();

  const int seg = lane >> lpc_shift;
  const int d = lane & (lpc - 1);
  const bool has_dev = d < D;
  const int base = seg * 3 * S;   // this segment's counters: counts[base + type * S + stage]
  int32_t* slot = counts + n_count_ints + seg * slot_words;   // TIMED: this segment's slots

  // what depends on the actor only
  const int nch = has_dev ? T.ints[T.off_n_chunks + d] : 0;
  int stage[V];
  int own_at[V];   // LDS index of this actor's forward counter of chunk c (backward at + S, W at + 2 S)
  int pred_at[V][DEG > 0 ? DEG : 1], succ_at[V][DEG > 0 ? DEG : 1];
#pragma unroll
  for (int c = 0; c < V; ++c) {
    stage[c] = c < nch ? T.ints[T.off_local_stage + d * kMaxChunks + c] : 0;
    own_at[c] = c < nch ? base + stage[c] : at_m;
#pragma unroll
    for (int k = 0; k < (DEG > 0 ? DEG : 1); ++k) {
      pred_at[c][k] = at_m;
      succ_at[c][k] = at_m;
      if (DEG > 0 && c < nch) {
        const int s = stage[c];
        const int pe = T.ints[T.off_pred_off + s] + k, se = T.ints[T.off_succ_off + s] + k;
        if (pe < T.ints[T.off_pred_off + s + 1]) pred_at[c][k] = base + T.ints[T.off_pred_stage + pe];
        if (se < T.ints[T.off_succ_off + s + 1]) succ_at[c][k] = base + S + T.ints[T.off_succ_stage + se];
      }
    }
  }

  // TIMED: what the actor's items cost together, and its memory cap
  long long busy_total = 0;
  int cap = 0x7fffffff;
  if (TIMED && has_dev) {
    cap = T.ints[T.off_mem_cap + d];
#pragma unroll
    for (int c = 0; c < V; ++c)
      if (c < nch)
        busy_total += (long long)m * ((long long)T.ints[T.off_dur + kF * S + stage[c]] + T.ints[T.off_dur + kB * S + stage[c]] +
                                      (has_w ? T.ints[T.off_dur + kW * S + stage[c]] : 0));
  }
  int free_at = 0, mem = 0, peak = 0;
  // SLIDE: cost and freed units of the W item of each chunk (the W rows), what all of them cost; the queue
  typename GenPerChunk<V>::type w_dur, w_free;
  int w_total = 0;
#pragma unroll
  for (int c = 0; c < V; ++c) {
    int wd = 0, wf = 0;
    if (SLIDE && has_dev && c < nch) {
      const int32_t* r = lds + ((2 * V + c) * D + d) * 8;   // (read after the barrier above)
      wd = r[0];
      wf = r[2];
    }
    w_dur[c] = wd; w_free[c] = wf;
    w_total += m * wd;
  }
  uint32_t* spill = reinterpret_cast<uint32_t*>(counts + n_count_ints + cpw * slot_words) + lane;   // word i at + i * 64
  unsigned q_h = 0u, h_n = 0u, q_t = 0u, t_n = 0u, s_rd = 0u, s_wr = 0u;
  unsigned q_head_dur = 0xffffffffu;   // cost of the oldest stashed item (all ones: none)
  int q_head_free = 0, w_placed = 0;
  auto new_head = [&]() {
    const unsigned head = V > 1 ? q_h & (unsigned)(V - 1) : 0u;
    q_head_dur = h_n != 0u ? (unsigned)gen_pick<V>(w_dur, head) : 0xffffffffu;
    q_head_free = gen_pick<V>(w_free, head);
  };

  pair16 limit2 = {1, 1};
  int w_at[V];   // the weight-gradient counters; without split backward, a word that holds m
#pragma unroll
  for (int c = 0; c < V; ++c) w_at[c] = has_w ? own_at[c] + 2 * S : at_m;

  // per-set state
  long long set = ((long long)blockIdx.x * waves_per_block + wave) * cpw + seg;   // the first set of a segment is its global index
  bool first_draw = true;
  bool has_set = false;   // the segment is working on a set (possibly finished and not yet written out)
  bool fresh = true;      // the segment wants its next set
  int limit[V];
  int cttp = 0, unit_f = 1, unit_b = 1, f_dir = 0, f_int = 0, b_dir = 0, b_int = 0;
#pragma unroll
  for (int c = 0; c < V; ++c) limit[c] = 1;
  int turn_type = kGenF, turn_run = 0, pos_f = 0, pos_b = 0, stepped_f = 0, stepped_b = 0;
  int first = kGenF;   // the instruction type tried first in a step: fixed, or the interleaved priority's turn
  int left = 0;        // items this actor still has to schedule
  bool live = false;   // the set's process is still running
  int status = 0, len = 0;
  unsigned long long first_step = 0ull;   // the loop's step counter when the set's process began
  int steps = 0;
  int last_pick = -1;   // the step, counted from first_step, in which this actor scheduled its last item so far
  constexpr unsigned long long kEndCheckMask = 7ull;
  uint16_t* row = ops;
  // "does any lane of my segment ...": the ballot against the lanes of the segment
  const unsigned long long seg_lanes = (lpc == 64 ? ~0ull : ((1ull << lpc) - 1ull)) << (seg * lpc);
  const unsigned seg_lo = (unsigned)seg_lanes, seg_hi = (unsigned)(seg_lanes >> 32);
  auto any_in_segment = [&](unsigned long long ballot) -> bool {
    return (((unsigned)ballot & seg_lo) | ((unsigned)(ballot >> 32) & seg_hi)) != 0u;
  };

  // Every step but the last of a set schedules at least one of its 3 S m items, and a segment
  // cannot draw more than all sets: the bound below is never reached, it only makes sure that the
  // wavefront leaves the loop whatever happens.  A workgroup is one wavefront: its LDS instructions
  // execute in program order, so the reads of a step see the counters as the previous step left them
  // and no barrier is needed between the phases.
  const unsigned long long per_set = 3ull * (unsigned)S * (unsigned)m + 16ull;
  const unsigned long long bound = per_set * ((unsigned long long)n_sets + 1ull);
  for (unsigned long long step = 0; step < bound; ++step) {
    if (__ballot(fresh) != 0ull) {
      // ---- segments that finished write their schedule out and start on the next set
      if (fresh) {
        fresh = false;
        if (TIMED) {
          if (has_set) {
            // the segment's results, in the form fpsched_evaluate gives them for the generated lists; a
            // schedule that is not complete (stuck, bad policy) has items that never ran
            // (SLIDE: what is still stashed runs back to back behind the actor's last item)
            int makespan = SLIDE ? free_at + (w_total - w_placed) : free_at;
            bool over = peak > cap;
            for (int off = 1; off < lpc; off <<= 1) makespan = max(makespan, __shfl_xor(makespan, off, 64));
            over = any_in_segment(__ballot(over));
            const bool complete = status == 0;
            if (has_dev) {
              R.idle[set * D + d] = complete ? (long long)makespan - busy_total : -1ll;
              R.peak[set * D + d] = complete ? peak : -1;
            }
            if (d == 0) {
              R.makespan[set] = complete ? (long long)makespan : 0x7fffffffffffffffll;
              R.flags[set] = (unsigned char)(complete ? (over ? kOverCap : 0) : kIncomplete);
              out_steps[set] = steps;
              out_status[set] = (unsigned char)status;
            }
          }
        } else if (has_set && has_dev) {
          // rows are END-padded to the stride; words still staged go out with the padding
          int at = len & ~15;
          if (len & 15) {
            for (int i = len & 15; i < 16; ++i) reinterpret_cast<uint16_t*>(staging + (i >> 1) * 64)[i & 1] = 0;
            if (at < stride)
              *reinterpret_cast<uint4*>(row + at) = make_uint4(staging[0], staging[64], staging[128], staging[192]);
            if (at + 8 < stride)
              *reinterpret_cast<uint4*>(row + at + 8) = make_uint4(staging[256], staging[320], staging[384], staging[448]);
            at += 16;
          }
          for (; at < stride; at += 8) *reinterpret_cast<uint4*>(row + at) = make_uint4(0u, 0u, 0u, 0u);
          if (d == 0) {
            out_steps[set] = steps;
            out_status[set] = (unsigned char)status;
          }
        }
        if (!first_draw) {
          unsigned long long drawn = 0ull;
          if (d == 0 && seg < cpw) drawn = atomicAdd(next_set, 1ull);
          set = (long long)__shfl(drawn, seg << lpc_shift, 64);
        }
        first_draw = false;
        has_set = seg < cpw && set < n_sets;
        const bool has_row = has_set && has_dev;
        if (has_set)
          for (int i = d; i < 3 * S; i += lpc) counts[base + i] = 0;
        cttp = 0; unit_f = 1; unit_b = 1; f_dir = 0; f_int = 0; b_dir = 0; b_int = 0;
        // (with a selection, output row `set` is the schedule of parameter set select[set]; an entry that
        // is negative or not below n_src selects nothing and counts as a bad set)
        const long long src = (has_set && select) ? select[set] : set;
        const bool has_src = has_row && src >= 0 && src < n_src;
        if (has_src) {
          const int32_t* pol = policy + (src * D + d) * 8;
          cttp = pol[0]; unit_f = pol[1]; unit_b = pol[2];
          f_dir = pol[3]; f_int = pol[4]; b_dir = pol[5]; b_int = pol[6];
        }
#pragma unroll
        for (int c = 0; c < V; ++c) limit[c] = (has_src && c < nch) ? inflight[src * S + stage[c]] : 1;
        if constexpr (V == 2) {   // (no stage has more than m <= 2048 micro-batches in flight)
          limit2.x = (short)min(limit[0], 0x7fff);
          limit2.y = (short)min(limit[1], 0x7fff);
        }
        // a parameter set with a value outside its domain generates nothing (status 4)
        bool bad = (has_row && !has_src) || cttp < 0 || cttp > 2 || unit_f < 1 || unit_b < 1 || f_dir < 0 || f_dir > 1 || f_int < 0 ||
                   b_dir < 0 || b_dir > 1 || b_int < 0 || (cttp != 2 && (unit_f != 1 || unit_b != 1));
#pragma unroll
        for (int c = 0; c < V; ++c) bad = bad || limit[c] < 1;
        const bool set_bad = any_in_segment(__ballot(bad && has_row));
        turn_type = kGenF; turn_run = 0;
        first = cttp == 0 ? kGenB : kGenF;
        pos_f = f_dir == 0 ? 0 : (nch > 0 ? nch - 1 : 0);
        pos_b = b_dir == 0 ? 0 : (nch > 0 ? nch - 1 : 0);
        stepped_f = 0; stepped_b = 0;
        left = (has_row && !set_bad) ? nch * m * (has_w ? 3 : 2) : 0;
        live = any_in_segment(__ballot(left > 0));
        first_step = step; steps = 0; last_pick = -1;
        status = set_bad ? 4 : 0; len = 0;
        free_at = 0; mem = 0; peak = 0;
        q_h = 0u; h_n = 0u; q_t = 0u; t_n = 0u; s_rd = 0u; s_wr = 0u; q_head_dur = 0xffffffffu; w_placed = 0;
        if (!TIMED) row = ops + (size_t)(has_row ? set * D + d : 0) * (size_t)stride;
        fresh = has_set && !live;   // nothing to schedule (a bad set, no stages): written out next time round
      }
      if (__ballot(has_set) == 0ull) break;   // every segment of the wavefront is out of work
    }
    // ---- read phase: the counters of this actor's own (type, stage) and of the neighbouring stages;
    // then for which stages the next item of each type is eligible (dependencies resolved, and for
    // forward items the in-flight rule).  A chunk the actor does not have is never eligible.
    int pick_t, pick_c, p1;
    bool is_f, is_b, move;
    int interval, stepped0;
    if constexpr (V == 2) {
      // Two stages per actor: their counters side by side in 16-bit halves (no counter exceeds m <= 2048),
      // every comparison a packed subtraction whose sign bits (bit 15: first stage, bit 31: second) say
      // "eligible".  A missing stage reads words that hold m and is never eligible.
      auto both = [&](int at0, int at1) {
        pair16 v;
        v.x = *reinterpret_cast<const short*>(&counts[at0]);
        v.y = *reinterpret_cast<const short*>(&counts[at1]);
        return v;
      };
      const pair16 nf = both(own_at[0], own_at[1]), nb = both(own_at[0] + S, own_at[1] + S);
      const pair16 nw = both(w_at[0], w_at[1]);
      pair16 f_ahead = both(pred_at[0][0], pred_at[1][0]), b_ahead = both(succ_at[0][0], succ_at[1][0]);
      if (DEG > 1) {
        f_ahead = __builtin_elementwise_min(f_ahead, both(pred_at[0][DEG > 1 ? 1 : 0], pred_at[1][DEG > 1 ? 1 : 0]));
        b_ahead = __builtin_elementwise_min(b_ahead, both(succ_at[0][DEG > 1 ? 1 : 0], succ_at[1][DEG > 1 ? 1 : 0]));
      }
      const unsigned alive = live ? kBothSigns : 0u;
      const unsigned el_f = bits_of(nf - f_ahead) & bits_of(nf - nb - limit2) & alive;
      const unsigned el_b = bits_of(nb - __builtin_elementwise_min(nf, b_ahead)) & alive;
      const unsigned el_w = bits_of(nw - nb) & alive;
      // the step function: the first instruction type, in priority order, with an eligible item ...
      const bool f_first = first == kGenF;
      const unsigned el_first = f_first ? el_f : el_b, el_second = f_first ? el_b : el_f;
      int type = el_w ? (int)kGenW : -1;
      type = el_second ? (first ^ 1) : type;
      type = el_first ? first : type;
      pick_t = type;
      unsigned el = el_second ? el_second : el_w;
      el = el_first ? el_first : el;
      is_f = pick_t == kGenF; is_b = pick_t == kGenB;
      const int dir = is_f ? f_dir : (is_b ? b_dir : 0);
      interval = is_f ? f_int : (is_b ? b_int : 0);
      const int p0 = is_f ? pos_f : pos_b;
      stepped0 = is_f ? stepped_f : stepped_b;
      // ... then the stage: "the next stage with an eligible item" is the other one if it has one, and the
      // first eligible stage in either direction is the only one, or the first / the last of both
      const unsigned p0_bit = 15u | ((unsigned)p0 << 4);
      move = stepped0 == interval || !((el >> p0_bit) & 1u);
      p1 = (move && ((el >> (p0_bit ^ 16u)) & 1u)) ? (p0 ^ 1) : p0;
      const int without_interval = el == kBothSigns ? dir : (int)(el >> 31);
      pick_c = interval > 0 ? p1 : without_interval;
    } else {
    unsigned ok_f = 0u, ok_b = 0u, ok_w = 0u;
#pragma unroll
    for (int c = 0; c < V; ++c) {
      const int nf = counts[own_at[c]], nb = counts[own_at[c] + S], nw = counts[own_at[c] + 2 * S];
      int f_ahead = m, b_ahead = nf;
      if (DEG > 0) {
        // (no counter exceeds m, and a missing neighbour reads a word that holds m)
        f_ahead = counts[pred_at[c][0]];
        b_ahead = min(b_ahead, counts[succ_at[c][0]]);
#pragma unroll
        for (int k = 1; k < (DEG > 0 ? DEG : 1); ++k) {
          f_ahead = min(f_ahead, counts[pred_at[c][k]]);
          b_ahead = min(b_ahead, counts[succ_at[c][k]]);
        }
      } else if (c < nch) {
        const int32_t* pred_off = lds + T.off_pred_off;
        const int32_t* succ_off = lds + T.off_succ_off;
        const int s = stage[c];
        for (int e = pred_off[s]; e < pred_off[s + 1]; ++e) f_ahead = min(f_ahead, counts[base + lds[T.off_pred_stage + e]]);
        for (int e = succ_off[s]; e < succ_off[s + 1]; ++e) b_ahead = min(b_ahead, counts[base + S + lds[T.off_succ_stage + e]]);
      }
      ok_f |= (unsigned)(f_ahead > nf && nf - nb < limit[c]) << c;
      ok_b |= (unsigned)(b_ahead > nb) << c;
      ok_w |= (unsigned)(has_w && nb > nw) << c;
    }
    if (!live) { ok_f = 0u; ok_b = 0u; ok_w = 0u; }
    // ---- the step function, without branches: the first instruction type, in priority order, with an
    // eligible item; then the stage, in traversal order
    const unsigned ok_first = first == kGenF ? ok_f : ok_b, ok_second = first == kGenF ? ok_b : ok_f;
    pick_t = ok_first ? first : (ok_second ? (first ^ 1) : (ok_w ? kGenW : -1));
    const unsigned ok = ok_first ? ok_first : (ok_second ? ok_second : ok_w);
    is_f = pick_t == kGenF; is_b = pick_t == kGenB;
    const int dir = is_f ? f_dir : (is_b ? b_dir : 0);
    interval = is_f ? f_int : (is_b ? b_int : 0);
    const int p0 = is_f ? pos_f : pos_b;
    stepped0 = is_f ? stepped_f : stepped_b;
    move = stepped0 == interval || !((ok >> p0) & 1u);
    if (V <= 2) {
      // at most two stages: "the next stage with an eligible item" is the other one if it has one, and the
      // first eligible stage in either direction is the only one, or the first / the last of both
      const unsigned other = (unsigned)p0 ^ 1u;
      p1 = (move && ((ok >> other) & 1u)) ? (int)other : p0;
      const int without_interval = ok == 3u ? dir : (int)(ok >> 1);
      pick_c = interval > 0 ? p1 : without_interval;
    } else {
      // the next stage after p0, in the traversal direction and cyclically, that has an eligible item:
      // lay the mask out twice, shift it so that the stage after p0 is at bit 0, take the lowest bit
      // (depth-first: the same on the mirrored mask)
      const unsigned mirrored = __brev(ok) >> (32 - nch);   // (nch = 0: ok is 0 and nothing is picked)
      const unsigned walk = dir == 0 ? ok : mirrored;
      const int q0 = dir == 0 ? p0 : nch - 1 - p0;
      const unsigned twice = walk | (walk << nch);
      int q1 = q0 + 1 + low_bit(twice >> (q0 + 1));
      q1 = q1 >= nch ? q1 - nch : q1;
      const int moved_to = dir == 0 ? q1 : nch - 1 - q1;
      p1 = move ? moved_to : p0;
      const int first_c = low_bit(ok), last_c = high_bit(ok);
      pick_c = interval > 0 ? p1 : (dir == 0 ? first_c : last_c);
    }
    }
    const int stepped1 = (move ? 0 : stepped0) + 1;
    if (interval > 0 && is_f) { pos_f = p1; stepped_f = stepped1; }
    if (interval > 0 && is_b) { pos_b = p1; stepped_b = stepped1; }
    if (pick_t >= 0) {
      // ---- write phase: the choice becomes visible for the next step; the counter's old value is
      // the micro-batch of the item
      int at = own_at[0];
#pragma unroll
      for (int c = 1; c < V; ++c) at = pick_c == c ? own_at[c] : at;
      const int j = atomicAdd(&counts[mad24((unsigned)pick_t, (unsigned)S, (unsigned)at)], 1);
      left -= 1;
      last_pick = (int)(step - first_step);
      if (TIMED && (!SLIDE || pick_t != kGenW)) {
        // the item's row: cost, memory, where its inputs' finish times are and where its own goes
        const int4* r = reinterpret_cast<const int4*>(
            reinterpret_cast<const char*>(lds) + __umul24((unsigned)(pick_t * V + pick_c), (unsigned)D * 32u) + d * 32);
        const int4 a = r[0], b = r[1];
        // (slot offsets in the rows are byte offsets)
        char* my_slot = reinterpret_cast<char*>(slot) + j * 4;
        int ready = *reinterpret_cast<const int32_t*>(my_slot + a.w) + b.x;
        if (DEG > 1) ready = max(ready, *reinterpret_cast<const int32_t*>(my_slot + b.y) + b.z);
        const int start = max(free_at, ready);
        if (SLIDE && q_head_dur <= (unsigned)(start - free_at)) {
          // the oldest stashed W items that end before this item starts run in front of it
          do {
            free_at += (int)q_head_dur;
            w_placed += (int)q_head_dur;
            mem -= q_head_free;
            q_h >>= kQBits;
            --h_n;
            if (h_n == 0u) {
              // the head word is used up: the oldest full word of the ring, else what the tail word holds
              if (s_rd != s_wr) {
                q_h = spill[(s_rd & (unsigned)(spill_words - 1)) * 64];
                ++s_rd;
                h_n = kQCap;
              } else {
                q_h = q_t; h_n = t_n;
                q_t = 0u; t_n = 0u;
              }
            }
            new_head();
          } while (q_head_dur <= (unsigned)(start - free_at));
        }
        free_at = start + a.x;
        *reinterpret_cast<int32_t*>(my_slot + (DEG > 1 ? (b.w & 0xffff) : b.w)) = free_at;
        if (DEG > 1) *reinterpret_cast<int32_t*>(my_slot + ((unsigned)b.w >> 16)) = free_at;
        mem += a.y;
        peak = max(peak, mem);
        if (!SLIDE) mem -= a.z;   // (SLIDE: with split backward only W items free, and they do when they are placed)
        if (SLIDE && pick_t == kGenB) {
          // a B item stashes its W item: into the head word while nothing waits behind it, else into the tail
          // word, which moves to the ring when it is full
          if (s_rd == s_wr && t_n == 0u && h_n < kQCap) {
            q_h |= (unsigned)pick_c << (h_n * kQBits);
            ++h_n;
            new_head();
          } else {
            q_t |= (unsigned)pick_c << (t_n * kQBits);
            ++t_n;
            if (t_n == kQCap) {
              spill[(s_wr & (unsigned)(spill_words - 1)) * 64] = q_t;
              ++s_wr;
              q_t = 0u; t_n = 0u;
            }
          }
        }
      } else if (TIMED) {
        // (SLIDE: a W item the scheduler placed is passed over)
      } else {
        const unsigned word = ((unsigned)(pick_t + 1) << 13) | ((unsigned)pick_c << 11) | (unsigned)j;
        // sixteen op words are collected in the lane's staging dwords and stored together
        reinterpret_cast<uint16_t*>(staging + ((len >> 1) & 7) * 64)[len & 1] = (uint16_t)word;
        if ((len & 15) == 15) {
          uint4* dst = reinterpret_cast<uint4*>(row + (len - 15));
          dst[0] = make_uint4(staging[0], staging[64], staging[128], staging[192]);
          dst[1] = make_uint4(staging[256], staging[320], staging[384], staging[448]);
        }
        len += 1;
      }
      if (cttp == 2 && pick_t == turn_type) {
        if (++turn_run >= (is_f ? unit_f : unit_b)) { turn_type = is_f ? kGenB : kGenF; turn_run = 0; first = turn_type; }
      }
    }
    __builtin_amdgcn_wave_barrier();
    // ---- has the set's process ended?  Looked at every eighth step only: a process that has ended stays ended
    // (when every item is scheduled nothing is eligible any more; when a step schedules nothing although items
    // remain, no later step can), so the few steps a segment runs on change nothing, and the number of steps the
    // process took is one more than the step of its last item.
    if ((step & kEndCheckMask) == kEndCheckMask) {
      const bool any_pick = any_in_segment(__ballot(pick_t >= 0));
      const bool any_left = any_in_segment(__ballot(left > 0));
      if (live && (!any_pick || !any_left)) {
        int last = last_pick;
        for (int off = 1; off < lpc; off <<= 1) last = max(last, __shfl_xor(last, off, 64));
        status = any_left ? 1 : status;   // items remain and nothing can move
        steps = last + 1;
        live = false;
        fresh = true;
      }
    }
  }
}

#define FPSCHED_INSTANTIATE(V, G, FORM)                                                                     \
  template __global__ void generate_kernel<V, G, FORM>(DevTables, const int32_t*, const int32_t*,            \
                                                        const long long*, long long, long long, int, uint16_t*, int32_t*, \
                                                        unsigned char*, unsigned long long*, GenResults);
FPSCHED_INSTANTIATE(1, 1, false)
FPSCHED_INSTANTIATE(2, 1, false)
FPSCHED_INSTANTIATE(4, 1, false)
FPSCHED_INSTANTIATE(1, 2, false)
FPSCHED_INSTANTIATE(2, 2, false)
FPSCHED_INSTANTIATE(4, 2, false)
FPSCHED_INSTANTIATE(1, 0, false)
FPSCHED_INSTANTIATE(2, 0, false)
FPSCHED_INSTANTIATE(4, 0, false)
FPSCHED_INSTANTIATE(1, 1, true)
FPSCHED_INSTANTIATE(2, 1, true)
FPSCHED_INSTANTIATE(4, 1, true)
FPSCHED_INSTANTIATE(1, 2, true)
FPSCHED_INSTANTIATE(2, 2, true)
FPSCHED_INSTANTIATE(4, 2, true)
FPSCHED_INSTANTIATE(1, 1, kGenSlide)
FPSCHED_INSTANTIATE(2, 1, kGenSlide)
FPSCHED_INSTANTIATE(4, 1, kGenSlide)
FPSCHED_INSTANTIATE(1, 2, kGenSlide)
FPSCHED_INSTANTIATE(2, 2, kGenSlide)
FPSCHED_INSTANTIATE(4, 2, kGenSlide)
#undef FPSCHED_INSTANTIATE

}  // namespace fpsched

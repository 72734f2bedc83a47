// Weight-gradient sliding pass, second kernel (paper Section 5.2, "Bubble optimizations": the
// weight-gradient part of a backward pass is stashed and run in a later bubble of the same actor,
// so that what other actors wait for runs first).
//
// The rule: the W words of the input are dropped; every device walks its list under the
// evaluator's start rule; a B item that issues stashes its W item (first in, first out); in front
// of the next item of the list, which starts at t, the oldest stashed items run as long as they
// end by t; what is left when the list ends runs back to back.
//
// Because a stashed item only runs where it delays nothing, every item of the list starts exactly
// when it would start if there were no W items at all.  So the pass splits in two:
//   1. the evaluation kernel in its TIMES form (eval_slots.hip) times the lists without their W
//      items -- the only part with dependencies between devices -- and leaves each op's start time
//      and the position at which each list stopped;
//   2. this kernel places the W items: one lane per (candidate, device) row, no interaction
//      between lanes until the final reduction.  A lane walks its row once; the stash is the B
//      words between a second cursor and the first one (every B word before the second cursor has
//      had its W item placed), so it needs no storage.  One step per loop iteration, the same code
//      for all lanes: the oldest stashed item if it fits in front of the item at the list cursor
//      (or the list is over), else that item.  The new row leaves in 16-byte pieces collected in
//      registers; memory is accounted along the new order.
// Rows are read 16 bytes (op words) and 32 bytes (start times) at a time with the loads' latency
// exposed: there are thousands of independent wavefronts to cover it.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

namespace fpsched {

namespace {

// 8 op words in four registers, refilled from a 16-byte aligned row one piece ahead
struct WordReader {
  const uint16_t* row;
  int stride;
  uint4 cur, next;
  __device__ __forceinline__ uint4 piece(int at) const {
    return at < stride ? *reinterpret_cast<const uint4*>(row + at) : make_uint4(0u, 0u, 0u, 0u);
  }
  __device__ __forceinline__ void start(const uint16_t* r, int s) {
    row = r; stride = s;
    cur = piece(0);
    next = piece(8);
  }
  // word at position i (i only ever moves forward by one, starting at 0)
  __device__ __forceinline__ unsigned at(int i) const {
    const unsigned lo = (i & 2) ? cur.y : cur.x, hi = (i & 2) ? cur.w : cur.z;
    const unsigned dw = (i & 4) ? hi : lo;
    return (i & 1) ? dw >> 16 : dw & 0xffffu;
  }
  // call after moving on to position i
  __device__ __forceinline__ void moved_to(int i) {
    if ((i & 7) == 0) {
      cur = next;
      next = piece(i + 8);
    }
  }
};

}  // namespace

__global__ __launch_bounds__(kSlideThreads) void wslide_place_kernel(
    SlotTables T, const uint16_t* __restrict__ ops, long long n_cand, int stride,
    const uint32_t* __restrict__ start8, const int32_t* __restrict__ stop_pos,
    const unsigned char* __restrict__ timed_flags, uint16_t* __restrict__ ops_out, int stride_out,
    long long* __restrict__ out_makespan, long long* __restrict__ out_idle, int* __restrict__ out_peak,
    unsigned char* __restrict__ out_flags) {
  extern __shared__ int32_t lds[];
  const int lpc = T.lanes_per_cand;
  const int lpc_shift = __ffs(lpc) - 1;
  // LDS: the metadata rows, one int4 per (kind * 4 + chunk, device): x = dur << 8,
  // w = units allocated at the start (byte 0) | units freed at the end (byte 1)
  const int n_meta_ints = kNKinds * kMaxChunks * lpc * 4;
  for (int i = threadIdx.x; i < n_meta_ints; i += blockDim.x) lds[i] = T.ints[i];
  const int4* meta = reinterpret_cast<const int4*>(lds);
  __syncthreads();

  const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const long long cand = t >> lpc_shift;
  const int d = (int)(t & (lpc - 1));
  const bool active = cand < n_cand && d < T.D;
  const size_t row_index = (size_t)(active ? cand : 0) * T.D + (active ? d : 0);
  // start times: [candidate][group of four positions][lane of the candidate][4]
  const uint32_t* start_row = start8 + (size_t)(active ? cand : 0) * (size_t)stride * (size_t)lpc + ((size_t)d << 2);
  uint16_t* out_row = ops_out + row_index * (size_t)stride_out;
  const int stop = active ? stop_pos[row_index] : 0;

  WordReader list, scan;   // the list cursor and the stash cursor read the same row
  list.start(ops + row_index * (size_t)stride, active ? stride : 0);
  scan = list;
  int wcur = 0, out_len = 0;
  unsigned t8 = 0u, busy8 = 0u;   // device free time and busy time, << 8
  int mem = 0, pk = 0;
  bool overflow = false;
  // the oldest stashed item: the B word at the stash cursor as a W word, its cost and what it frees
  unsigned q_word = 0u, q_dur8 = 0u;
  int q_free = 0;
  auto stash_head = [&](unsigned b_word) {
    q_word = (b_word & 0x1fffu) | ((unsigned)kW << 13);
    const int4 Mq = meta[(q_word >> 11) * lpc + d];
    q_dur8 = (unsigned)Mq.x;
    q_free = (int)(((unsigned)Mq.w >> 8) & 0xffu);
  };
  // the new row leaves in 16-byte pieces: eight words shifted into four registers
  unsigned acc0 = 0u, acc1 = 0u, acc2 = 0u, acc3 = 0u;
  auto shift_in = [&](unsigned word) {
    acc0 = __builtin_amdgcn_alignbit(acc1, acc0, 16);
    acc1 = __builtin_amdgcn_alignbit(acc2, acc1, 16);
    acc2 = __builtin_amdgcn_alignbit(acc3, acc2, 16);
    acc3 = (acc3 >> 16) | (word << 16);
  };
  auto append = [&](unsigned word) {
    if (out_len < stride_out) {
      shift_in(word);
      if ((out_len & 7) == 7) *reinterpret_cast<uint4*>(out_row + (out_len - 7)) = make_uint4(acc0, acc1, acc2, acc3);
      ++out_len;
    } else {
      overflow = true;   // the row keeps its first stride_out items; the candidate is reported as failed
    }
  };
  // the item at the list cursor: its word, metadata row and start time, fetched when the cursor moves
  int pos = 0;
  unsigned w = 0u, s8 = 0u;
  int4 M = make_int4(0, 0, 0, 0);
  uint4 starts = make_uint4(0u, 0u, 0u, 0u), starts_hi = make_uint4(0u, 0u, 0u, 0u);
  auto fetch = [&]() {
    if ((pos & 7) == 0) {   // the start times of eight positions (strides are multiples of 8)
      starts = *reinterpret_cast<const uint4*>(start_row + ((size_t)(pos >> 2) << (lpc_shift + 2)));
      starts_hi = *reinterpret_cast<const uint4*>(start_row + ((size_t)((pos >> 2) + 1) << (lpc_shift + 2)));
    }
    w = list.at(pos);
    M = meta[(w >> 11) * lpc + d];
    const uint4 half = (pos & 4) ? starts_hi : starts;
    const unsigned s01 = (pos & 1) ? half.y : half.x, s23 = (pos & 1) ? half.w : half.z;
    s8 = (pos & 2) ? s23 : s01;
  };
  if (pos < stop) fetch();
  // a device that reached the end of its list runs what is still stashed back to back
  const bool at_end = active && (stop >= stride || (ops[row_index * (size_t)stride + stop] >> 13) == (unsigned)kEnd);

  // One step per iteration: the oldest stashed item runs if it ends by the start of the item at the
  // list cursor (or the list is over); else that item issues, or a W word of the input is passed over.
  for (;;) {
    const bool have = pos < stop;
    const unsigned kind = w >> 13;
    const bool item = have && kind != (unsigned)kW;   // where the input put its W items is not used
    const bool place = wcur < pos && (have ? (item && t8 + q_dur8 <= s8) : at_end);
    if (!have && !place) break;
    if (place || item) {
      const unsigned dur8 = place ? q_dur8 : (unsigned)M.x;
      const unsigned at8 = place ? t8 : s8;
      append(place ? q_word : w);
      mem += place ? 0 : (int)((unsigned)M.w & 0xffu);
      pk = max(pk, mem);
      mem -= place ? q_free : (int)(((unsigned)M.w >> 8) & 0xffu);
      t8 = at8 + dur8;
      busy8 += dur8;
    }
    if (place) {
      // the stash cursor moves on to the next B word in front of the list cursor
      do {
        ++wcur;
        scan.moved_to(wcur);
      } while (wcur < pos && (scan.at(wcur) >> 13) != (unsigned)kB);
      if (wcur < pos) stash_head(scan.at(wcur));
    } else {
      // the word at the list cursor is done with; the stash cursor follows the list cursor unless it
      // rests on a B word whose W item is due
      if (wcur == pos) {
        if (kind == (unsigned)kB) {
          stash_head(w);
        } else {
          ++wcur;
          scan.moved_to(wcur);
        }
      }
      ++pos;
      list.moved_to(pos);
      if (pos < stop) fetch();
    }
  }

  // ---- the rest of the new row: words still in the registers, then END words up to the stride
  if (active) {
    int at = out_len;
    if (at & 7) {
      for (; at & 7; ++at) shift_in(0u);
      *reinterpret_cast<uint4*>(out_row + (at - 8)) = make_uint4(acc0, acc1, acc2, acc3);
    }
    for (; at < stride_out; at += 8) *reinterpret_cast<uint4*>(out_row + at) = make_uint4(0u, 0u, 0u, 0u);
  }
  // ---- the evaluation of the new lists
  const int seg_base = (threadIdx.x & 63) & ~(lpc - 1);
  const unsigned long long seg_mask = (lpc == 64 ? ~0ull : ((1ull << lpc) - 1ull)) << seg_base;
  const int cap = active ? T.ints[T.off_dev + d * T.dev_ints + 1] : 0;
  const unsigned long long full = __ballot(active && overflow) & seg_mask;
  const unsigned long long over = __ballot(active && pk > cap) & seg_mask;
  int ms = active ? (int)(t8 >> 8) : 0;
  for (int off = 1; off < lpc; off <<= 1) ms = max(ms, __shfl_xor(ms, off, 64));
  if (active) {
    unsigned fl = timed_flags[cand] & (kDeadlock | kIncomplete);
    if (full) fl |= kDeadlock | kIncomplete;
    const bool failed = fl != 0;
    if (!failed && over) fl = kOverCap;
    out_idle[cand * T.D + d] = failed ? -1ll : (long long)(ms - (int)(busy8 >> 8));
    out_peak[cand * T.D + d] = failed ? -1 : pk * T.unit_scale;
    if (d == 0) {
      out_makespan[cand] = failed ? 0x7fffffffffffffffll : (long long)ms;
      out_flags[cand] = (unsigned char)fl;
    }
  }
}

}  // namespace fpsched

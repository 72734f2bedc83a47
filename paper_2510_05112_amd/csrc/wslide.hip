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
//      between lanes until the final reduction.  A lane walks its row once.  One step per loop
//      iteration, the same code for all lanes: the oldest stashed item if it fits in front of the
//      item at the list cursor (or the list is over), else that item.  The new row leaves in
//      16-byte pieces collected in registers; memory is accounted along the new order.
// No global load sits on a step's critical path: op words and the low halves of their start times reach a
// lane through a 32-position LDS window that the whole wavefront tops up every eighth step, sixteen
// positions (32 bytes of each) at a time, the loads requested at one top-up landing at the next.  (With
// loads issued by each lane when it needs them the wavefront waited for memory in nearly every step:
// among 64 lanes at 64 different positions some lane always needs its next piece.)  The first kernel
// hands over sixteen bits per op: a start time is rebuilt from the device's free time in front of the op,
// start = free + ((low - free) mod 2^16), plus 2^16 times the entry of the row's escape list for the few
// ops that waited longer.  The stash is a ring of B words in LDS; only a stash deeper than the ring is
// read back from the device's own row, with the latency exposed.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

namespace fpsched {

namespace {

constexpr int kWin = 32;      // window: positions per lane (op words and the low halves of their start times)
constexpr int kPiece = 16;    // positions per load: 32 bytes of op words, 32 bytes of start times
constexpr int kRefillAt = 16; // a lane asks for its next piece when at most this many positions are unread
constexpr unsigned kTopUpMask = 7u;   // the window is topped up every eighth step
constexpr int kFifo = 16;     // stash ring: B words per lane
static_assert((2 * kWin + kFifo) * 64 * 2 == kSlideWaveLdsBytes, "LDS of one wavefront");

}  // namespace

__global__ __launch_bounds__(kSlideThreads) void wslide_place_kernel(
    SlotTables T, const uint16_t* __restrict__ ops, long long n_cand, int stride,
    const uint32_t* __restrict__ start_low, const uint32_t* __restrict__ escapes, int escape_cap,
    const int32_t* __restrict__ stop_pos,
    const unsigned char* __restrict__ timed_flags, uint16_t* __restrict__ ops_out, int stride_out,
    long long* __restrict__ out_makespan, long long* __restrict__ out_idle, int* __restrict__ out_peak,
    unsigned char* __restrict__ out_flags) {
  extern __shared__ int32_t lds[];
  const int lpc = T.lanes_per_cand;
  const int lpc_shift = __ffs(lpc) - 1;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // LDS: [the metadata rows, one int4 per (kind * 4 + chunk, device): x = dur << 8, w = units
  // allocated at the start (byte 0) | units freed at the end (byte 1)][per wavefront: op-word window
  // [position][lane], start-time window [position][lane], stash ring [entry][lane], all 16-bit]
  const int n_meta_ints = kNKinds * kMaxChunks * lpc * 4;
  for (int i = threadIdx.x; i < n_meta_ints; i += blockDim.x) lds[i] = T.ints[i];
  const int4* meta = reinterpret_cast<const int4*>(lds);
  uint16_t* word_win = reinterpret_cast<uint16_t*>(lds + n_meta_ints + wave * (kSlideWaveLdsBytes / 4)) + lane;   // entry i at + i * 64
  uint16_t* low_win = word_win + kWin * 64;
  uint16_t* fifo = low_win + kWin * 64;
  __syncthreads();

  const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const long long cand = t >> lpc_shift;
  const int d = (int)(t & (lpc - 1));
  const bool active = cand < n_cand && d < T.D;
  const size_t row_index = (size_t)(active ? cand : 0) * T.D + (active ? d : 0);
  const uint16_t* row = ops + row_index * (size_t)stride;
  // start times: [candidate][group of eight positions][lane of the candidate][8 x 16 bits], as dwords
  const uint32_t* start_row = start_low + (size_t)(active ? cand : 0) * ((size_t)stride >> 1) * (size_t)lpc + ((size_t)d << 2);
  const uint32_t* esc_row = escapes + row_index * (size_t)escape_cap;
  uint16_t* out_row = ops_out + row_index * (size_t)stride_out;
  int stop = active ? stop_pos[row_index] : 0;
  // a device that reached the end of its list runs what is still stashed back to back
  unsigned end_word = (active && stop < stride) ? row[stop] : 0u;
  // the first op that waited 2^16 time units or more (position << 8 | wait >> 16; all ones: none)
  unsigned esc = active ? esc_row[0] : 0xffffffffu;
  int esc_at = 1;
  // have them in registers before the loop: a wait for them inside the loop would also wait for
  // the window loads in flight
  asm volatile("" : "+v"(stop), "+v"(end_word), "+v"(esc));
  const bool at_end = active && (end_word >> 13) == (unsigned)kEnd;

  // window: positions [loaded - kWin, loaded) of the row are in the rings; the whole wavefront tops
  // them up every eighth step, the loads requested at one top-up landing at the next
  int loaded = 0;
  uint4 pend_w0 = make_uint4(0u, 0u, 0u, 0u), pend_w1 = pend_w0, pend_s0 = pend_w0, pend_s1 = pend_w0;
  bool has_pend = false;
  auto land8 = [&](int q, uint4 wv, uint4 sv) {
    word_win[(q + 0) * 64] = (uint16_t)wv.x; word_win[(q + 1) * 64] = (uint16_t)(wv.x >> 16);
    word_win[(q + 2) * 64] = (uint16_t)wv.y; word_win[(q + 3) * 64] = (uint16_t)(wv.y >> 16);
    word_win[(q + 4) * 64] = (uint16_t)wv.z; word_win[(q + 5) * 64] = (uint16_t)(wv.z >> 16);
    word_win[(q + 6) * 64] = (uint16_t)wv.w; word_win[(q + 7) * 64] = (uint16_t)(wv.w >> 16);
    low_win[(q + 0) * 64] = (uint16_t)sv.x; low_win[(q + 1) * 64] = (uint16_t)(sv.x >> 16);
    low_win[(q + 2) * 64] = (uint16_t)sv.y; low_win[(q + 3) * 64] = (uint16_t)(sv.y >> 16);
    low_win[(q + 4) * 64] = (uint16_t)sv.z; low_win[(q + 5) * 64] = (uint16_t)(sv.z >> 16);
    low_win[(q + 6) * 64] = (uint16_t)sv.w; low_win[(q + 7) * 64] = (uint16_t)(sv.w >> 16);
  };
  // a piece is sixteen positions, or eight at the end of a row whose stride is not a multiple of 16
  auto request = [&](int at) {
    pend_w0 = *reinterpret_cast<const uint4*>(row + at);
    pend_s0 = *reinterpret_cast<const uint4*>(start_row + ((size_t)(at >> 3) << (lpc_shift + 2)));
    if (at + 8 < stride) {
      pend_w1 = *reinterpret_cast<const uint4*>(row + at + 8);
      pend_s1 = *reinterpret_cast<const uint4*>(start_row + ((size_t)((at >> 3) + 1) << (lpc_shift + 2)));
    }
  };
  auto land = [&]() {
    const int q = loaded & (kWin - 1);
    land8(q, pend_w0, pend_s0);
    if (loaded + 8 < stride) land8(q + 8, pend_w1, pend_s1);
    loaded += (loaded + 8 < stride) ? kPiece : 8;
  };
  if (active)   // the head of the row is fetched before the first step
    for (int i = 0; i < 2 && loaded < stride; ++i) { request(loaded); land(); }

  int pos = 0, out_len = 0;
  unsigned t8 = 0u, busy8 = 0u;   // device free time and busy time, << 8
  unsigned u8 = 0u;               // the device's free time in the list without W items, << 8
  int mem = 0, pk = 0;
  bool overflow = false, done = !active;
  // stash ring: entries [q_head, q_tail) are B words whose W item is due, oldest first; `overflowed`:
  // B words from row position refill_pos on found no room and are still to be read back from the row
  int q_head = 0, q_tail = 0, refill_pos = 0;
  bool overflowed = false;
  unsigned q_word = 0u, q_dur8 = 0u;   // the oldest stashed item as a W word, its cost and what it frees
  int q_free = 0;
  // cost and freed units of the W item of each chunk of this device (rows kW * 4 + chunk of the metadata)
  unsigned w_dur8[kMaxChunks];
  int w_free[kMaxChunks];
#pragma unroll
  for (int c = 0; c < kMaxChunks; ++c) {
    const int4 Mw = meta[(kW * kMaxChunks + c) * lpc + d];
    w_dur8[c] = (unsigned)Mw.x;
    w_free[c] = (int)(((unsigned)Mw.w >> 8) & 0xffu);
  }
  // the new row leaves in 16-byte pieces: eight words shifted into four registers
  unsigned acc0 = 0u, acc1 = 0u, acc2 = 0u, acc3 = 0u;
  auto shift_in = [&](unsigned word) {
    acc0 = __builtin_amdgcn_alignbit(acc1, acc0, 16);
    acc1 = __builtin_amdgcn_alignbit(acc2, acc1, 16);
    acc2 = __builtin_amdgcn_alignbit(acc3, acc2, 16);
    acc3 = __builtin_amdgcn_alignbit(word, acc3, 16);
  };

  // One step per iteration and lane, the same straight-line code for all: look at the word at the list
  // cursor (in the window unless the lane has outrun it: then it waits for the next top-up); the oldest
  // stashed item runs if it ends by the start of that item (or the list is over); else the item issues, or
  // a W word of the input is passed over.
  for (unsigned step = 0;; ++step) {
    if ((step & kTopUpMask) == 0u) {
      if (has_pend) {
        land();
        has_pend = false;
      }
      if (!done && loaded - pos <= kRefillAt && loaded < stride) {
        request(loaded);
        has_pend = true;
      }
    }
    const unsigned slot0 = (unsigned)(pos & (kWin - 1)) * 64u, slot1 = (unsigned)((pos + 1) & (kWin - 1)) * 64u;
    const unsigned w0 = word_win[slot0], w1 = word_win[slot1];
    const unsigned l0 = low_win[slot0], l1 = low_win[slot1];
    // a W word of the input at the cursor is passed over at once when the word behind it is there as well
    // (it is never in the escape list: in the first pass it starts the moment its device is free)
    const bool hop = !done && pos + 1 < min(stop, loaded) && (w0 >> 13) == (unsigned)kW;
    pos += hop ? 1 : 0;
    const unsigned w = hop ? w1 : w0;
    const unsigned low8 = (hop ? l1 : l0) << 8;
    const bool have = pos < stop;
    const bool in_window = pos < loaded;
    // (any 16-bit value indexes a row of the table: the top five bits of the word)
    const int4 M = meta[((w >> 11) << lpc_shift) + d];
    // the start time from its low half and the free time in front of the op, plus what the escape
    // list says for an op that waited 2^16 time units or more
    const bool esc_here = (esc >> 8) == (unsigned)pos;
    const unsigned s8 = u8 + ((low8 - u8) & 0x00ffff00u) + (esc_here ? esc << 24 : 0u);
    const unsigned kind = w >> 13;
    const bool word_ok = !done && have && in_window;
    const bool item = word_ok && kind != (unsigned)kW;   // where the input put its W items is not used
    const bool skip = word_ok && kind == (unsigned)kW;
    const bool place = !done && q_head != q_tail && (have ? (item && t8 + q_dur8 <= s8) : at_end);
    const bool issue = item && !place;
    done = done || (!have && !place);
    if (place || issue) {
      const unsigned dur8 = place ? q_dur8 : (unsigned)M.x;
      const unsigned at8 = place ? t8 : s8;
      if (out_len < stride_out) {
        shift_in(place ? q_word : w);
        if ((out_len & 7) == 7) *reinterpret_cast<uint4*>(out_row + (out_len - 7)) = make_uint4(acc0, acc1, acc2, acc3);
        ++out_len;
      } else {
        overflow = true;   // the row keeps its first stride_out items; the candidate is reported as failed
      }
      mem += place ? 0 : (int)((unsigned)M.w & 0xffu);
      pk = max(pk, mem);
      mem -= place ? q_free : (int)(((unsigned)M.w >> 8) & 0xffu);
      t8 = at8 + dur8;
      busy8 += dur8;
      if (issue) u8 = t8;   // an item of the list ends when it would without any W item
    }
    bool new_head = false;
    if (place) {
      ++q_head;
      new_head = true;
      if (q_head == q_tail && overflowed) {
        // the ring ran empty while B words wait in the row: read them back, up to the list cursor
        int at = refill_pos;
        while (at < pos && q_tail - q_head < kFifo) {
          const unsigned b_word = row[at];
          if ((b_word >> 13) == (unsigned)kB) {
            fifo[(q_tail & (kFifo - 1)) * 64] = (uint16_t)b_word;
            ++q_tail;
          }
          ++at;
        }
        refill_pos = at;
        overflowed = at < pos;
      }
    }
    if (issue && kind == (unsigned)kB && !overflowed) {
      // an issued B item stashes its W item (once the ring has overflowed, later ones stay in the row)
      if (q_tail - q_head < kFifo) {
        fifo[(q_tail & (kFifo - 1)) * 64] = (uint16_t)w;
        new_head = q_tail == q_head;
        ++q_tail;
      } else {
        overflowed = true;
        refill_pos = pos;
      }
    }
    if (new_head && q_head != q_tail) {
      const unsigned b_word = fifo[(q_head & (kFifo - 1)) * 64];
      const unsigned c = (b_word >> 11) & 3u;
      q_word = (b_word & 0x1fffu) | ((unsigned)kW << 13);
      q_dur8 = c == 0u ? w_dur8[0] : (c == 1u ? w_dur8[1] : (c == 2u ? w_dur8[2] : w_dur8[3]));
      q_free = c == 0u ? w_free[0] : (c == 1u ? w_free[1] : (c == 2u ? w_free[2] : w_free[3]));
    }
    if (issue || skip) {
      if (esc_here) esc = esc_row[esc_at++];
      ++pos;
    }
    if (__ballot(!done) == 0ull) break;
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

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
// No global load sits on a step's critical path: op words and start times reach a lane through a
// 16-position LDS window that the whole wavefront tops up every fourth step, the loads requested
// at one top-up landing at the next.  (With loads issued by each lane when it needs them the
// wavefront waited for memory in nearly every step: among 64 lanes at 64 different positions some
// lane always needs its next piece.)  The stash is a ring of B words in LDS; only a stash deeper
// than the ring is read back from the device's own row, with the latency exposed.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

namespace fpsched {

namespace {

constexpr int kWin = 16;     // window: positions per lane (op words and their start times)
constexpr int kPiece = 4;    // positions per load: 8 bytes of op words, 16 bytes of start times
constexpr int kRefillAt = 9; // a lane asks for its next piece when at most this many positions are unread
constexpr int kFifo = 16;    // stash ring: B words per lane
static_assert((kWin * 64 + (kWin + kFifo) * 32) * 4 == kSlideWaveLdsBytes, "LDS of one wavefront");

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
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // LDS: [the metadata rows, one int4 per (kind * 4 + chunk, device): x = dur << 8, w = units
  // allocated at the start (byte 0) | units freed at the end (byte 1)][per wavefront: start-time
  // window [position][lane] (dwords), op-word window [position][lane], stash ring [entry][lane]]
  const int n_meta_ints = kNKinds * kMaxChunks * lpc * 4;
  for (int i = threadIdx.x; i < n_meta_ints; i += blockDim.x) lds[i] = T.ints[i];
  const int4* meta = reinterpret_cast<const int4*>(lds);
  uint32_t* start_win = reinterpret_cast<uint32_t*>(lds + n_meta_ints + wave * (kWin * 64 + (kWin + kFifo) * 32)) + lane;
  uint16_t* word_win = reinterpret_cast<uint16_t*>(start_win - lane + kWin * 64) + lane;   // entry i at + i * 64
  uint16_t* fifo = word_win + kWin * 64;
  __syncthreads();

  const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const long long cand = t >> lpc_shift;
  const int d = (int)(t & (lpc - 1));
  const bool active = cand < n_cand && d < T.D;
  const size_t row_index = (size_t)(active ? cand : 0) * T.D + (active ? d : 0);
  const uint16_t* row = ops + row_index * (size_t)stride;
  // start times: [candidate][group of four positions][lane of the candidate][4]
  const uint32_t* start_row = start8 + (size_t)(active ? cand : 0) * (size_t)stride * (size_t)lpc + ((size_t)d << 2);
  uint16_t* out_row = ops_out + row_index * (size_t)stride_out;
  int stop = active ? stop_pos[row_index] : 0;
  // a device that reached the end of its list runs what is still stashed back to back
  unsigned end_word = (active && stop < stride) ? row[stop] : 0u;
  // have both in registers before the loop: a wait for them inside the loop would also wait for
  // the window loads in flight
  asm volatile("" : "+v"(stop), "+v"(end_word));
  const bool at_end = active && (end_word >> 13) == (unsigned)kEnd;

  // window: positions [loaded - kWin, loaded) of the row are in the rings; the whole wavefront tops
  // them up every fourth step, the loads requested at one top-up landing at the next
  int loaded = 0;
  uint2 pend_words = make_uint2(0u, 0u);
  uint4 pend_starts = make_uint4(0u, 0u, 0u, 0u);
  bool has_pend = false;
  auto land = [&](uint2 wv, uint4 sv) {
    const int q = loaded & (kWin - 1);
    word_win[(q + 0) * 64] = (uint16_t)wv.x; word_win[(q + 1) * 64] = (uint16_t)(wv.x >> 16);
    word_win[(q + 2) * 64] = (uint16_t)wv.y; word_win[(q + 3) * 64] = (uint16_t)(wv.y >> 16);
    start_win[(q + 0) * 64] = sv.x; start_win[(q + 1) * 64] = sv.y;
    start_win[(q + 2) * 64] = sv.z; start_win[(q + 3) * 64] = sv.w;
    loaded += kPiece;
  };
  auto piece_words = [&](int at) { return *reinterpret_cast<const uint2*>(row + at); };
  auto piece_starts = [&](int at) { return *reinterpret_cast<const uint4*>(start_row + ((size_t)(at >> 2) << (lpc_shift + 2))); };
  if (active)   // the head of the row is fetched before the first step (strides are multiples of 8)
    for (int i = 0; i < 12 && i < stride; i += kPiece) land(piece_words(i), piece_starts(i));

  int pos = 0, out_len = 0;
  unsigned t8 = 0u, busy8 = 0u;   // device free time and busy time, << 8
  int mem = 0, pk = 0;
  bool overflow = false, done = !active;
  // the item at the list cursor: its word, metadata row and start time, read when the cursor moves
  unsigned w = 0u, s8 = 0u;
  int4 M = make_int4(0, 0, 0, 0);
  bool need_word = true;
  auto fetch = [&]() {   // (only called with pos < stop)
    if (pos < loaded) {
      w = word_win[(pos & (kWin - 1)) * 64];
      s8 = start_win[(pos & (kWin - 1)) * 64];
      M = meta[(w >> 11) * lpc + d];
      need_word = false;
    }
  };
  // stash ring: entries [q_head, q_tail) are B words whose W item is due, oldest first; `overflowed`:
  // B words from row position refill_pos on found no room and are still to be read back from the row
  int q_head = 0, q_tail = 0, refill_pos = 0;
  bool overflowed = false;
  unsigned q_word = 0u, q_dur8 = 0u;   // the oldest stashed item as a W word, its cost and what it frees
  int q_free = 0;
  auto stash_head = [&](unsigned b_word) {
    q_word = (b_word & 0x1fffu) | ((unsigned)kW << 13);
    const int4 Mq = meta[(q_word >> 11) * lpc + d];
    q_dur8 = (unsigned)Mq.x;
    q_free = (int)(((unsigned)Mq.w >> 8) & 0xffu);
  };
  auto stash_push = [&](unsigned b_word) -> bool {
    if (q_tail - q_head >= kFifo) return false;
    fifo[(q_tail & (kFifo - 1)) * 64] = (uint16_t)b_word;
    if (q_tail == q_head) stash_head(b_word);
    ++q_tail;
    return true;
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

  // One step per iteration and lane: the oldest stashed item runs if it ends by the start of the
  // item at the list cursor (or the list is over); else that item issues, or a W word of the input
  // is passed over.  A lane takes at most one position per step, so with these window sizes it
  // finds its word in the window (a lane that does not waits for the next top-up).
  for (unsigned step = 0;; ++step) {
    if ((step & 3u) == 0u) {
      if (has_pend) {
        land(pend_words, pend_starts);
        has_pend = false;
      }
      if (!done && loaded - pos <= kRefillAt && loaded < stride) {
        pend_words = piece_words(loaded);
        pend_starts = piece_starts(loaded);
        has_pend = true;
      }
    }
    if (!done) {
      const bool have = pos < stop;
      if (have && need_word) fetch();
      if (!(have && need_word)) {
        const unsigned kind = w >> 13;
        const bool item = have && kind != (unsigned)kW;   // where the input put its W items is not used
        const bool place = q_head < q_tail && (have ? (item && t8 + q_dur8 <= s8) : at_end);
        if (!have && !place) {
          done = true;
        } else {
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
            ++q_head;
            if (q_head == q_tail && overflowed) {
              // the ring ran empty while B words wait in the row: read them back, up to the list cursor
              int at = refill_pos;
              while (at < pos && q_tail - q_head < kFifo) {
                const unsigned b_word = row[at];
                if ((b_word >> 13) == (unsigned)kB) stash_push(b_word);
                ++at;
              }
              refill_pos = at;
              overflowed = at < pos;
            }
            if (q_head < q_tail) stash_head(fifo[(q_head & (kFifo - 1)) * 64]);
          } else {
            // the word at the list cursor is done with; an issued B item stashes its W item (once the
            // ring has overflowed, later ones stay in the row)
            if (kind == (unsigned)kB && !overflowed && !stash_push(w)) {
              overflowed = true;
              refill_pos = pos;
            }
            ++pos;
            need_word = true;
            if (pos < stop) fetch();
          }
        }
      }
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

// Weight-gradient sliding pass (paper Section 5.2, "Bubble optimizations": the weight-gradient part
// of a backward pass is stashed and run in a later bubble of the same actor, so that what other
// actors wait for runs first).  Input: candidate schedules of a problem with split backward; the W
// words of the input are dropped.  Every device walks its list under the evaluator's start rule; a
// B item that issues stashes its W item (first in, first out); in front of the next item of the
// list, which starts at t, the oldest stashed items run as long as they end by t; what is left
// when the list ends runs back to back.  Output: the new lists and their evaluation.
//
// Mapping and tables are those of the slot evaluation kernel (lane = device, 64 / pow2(D)
// candidates per wavefront, mail slots finish << 8 | producer stage per (direction, class,
// micro-batch), 4-bit activation states in lane-private LDS words, one 16-byte metadata row per
// (kind, chunk, device)); the control flow is plainer: candidates are assigned statically and a
// round is a loop body with branches in which a device does one thing (run its oldest stashed
// item, issue the item at its list cursor, or pass over a W word of the input).
//
// No global load sits on a round's critical path.  Op words reach a lane through a 16-word LDS
// window that the whole wavefront tops up every fourth round with 16-byte loads, the load
// requested at one top-up landing at the next (a lane that outruns its window waits for it).  The stash is a ring of B
// words in LDS; only a stash deeper than the ring is read back from the device's own row (the B
// words between the last one that found room and the list cursor), with the latency exposed.
// New rows leave in 16-byte pieces collected in registers (the kernel is bound by the latency of a
// round at the occupancy LDS allows: an LDS staging buffer for wider stores costs a wavefront per
// compute unit and more time than it saves).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

namespace fpsched {

namespace {

constexpr int kWin = 16;    // op window: words per lane
constexpr int kFifo = 16;   // stash ring: B words per lane

}  // namespace

template <int V, bool DEG2>
__global__ __launch_bounds__(kSlotMaxThreads) void wslide_kernel(
    SlotTables T, const uint16_t* __restrict__ ops, long long n_cand, int stride, uint16_t* __restrict__ ops_out,
    int stride_out, long long* __restrict__ out_makespan, long long* __restrict__ out_idle,
    int* __restrict__ out_peak, unsigned char* __restrict__ out_flags) {
  extern __shared__ int32_t lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n_waves = blockDim.x >> 6;
  const int m = T.m, cpw = T.cands_per_wave, lpc = T.lanes_per_cand;
  const int lpc_shift = __ffs(lpc) - 1;
  // LDS: [metadata rows][per wavefront: state words [word][lane], slots of its candidates,
  // op window [word][lane], stash ring [entry][lane]]
  for (int i = tid; i < T.n_shared_ints; i += blockDim.x) lds[i] = T.ints[i];
  const int wave_ints = T.state_words * 64 + cpw * T.slots_per_cand + (kWin + kFifo) * 32;
  uint32_t* stt = reinterpret_cast<uint32_t*>(lds + T.n_shared_ints + wave * wave_ints);
  uint32_t* slots = stt + T.state_words * 64;
  uint16_t* win = reinterpret_cast<uint16_t*>(slots + cpw * T.slots_per_cand) + lane;   // word i at + i * 64
  uint16_t* fifo = win + kWin * 64;                                                              // entry i at + i * 64
  const int4* meta = reinterpret_cast<const int4*>(lds);
  const int2* meta2 = reinterpret_cast<const int2*>(lds + T.off_meta2);
  __syncthreads();

  const int seg = lane >> lpc_shift, d = lane & (lpc - 1);
  const long long cand = ((long long)blockIdx.x * n_waves + wave) * cpw + seg;
  const bool in_seg = seg < cpw && cand < n_cand;
  const bool active = in_seg && d < T.D;
  const unsigned long long seg_mask = (lpc == 64 ? ~0ull : ((1ull << lpc) - 1ull)) << (seg * lpc);
  uint32_t* my_slots = slots + (seg < cpw ? seg : 0) * T.slots_per_cand;
  if (in_seg)
    for (int i = d; i < T.slots_per_cand; i += lpc) my_slots[i] = kEmptySlot;
  for (int i = 0; i < T.state_words; ++i) stt[i * 64 + lane] = 0u;

  const int dd = d < T.D ? d : 0;
  const int32_t* dev = T.ints + T.off_dev + dd * T.dev_ints;
  const int32_t* expect = T.ints + T.off_expect + dd * T.state_words;
  int cap = dev[1];
  asm volatile("" : "+v"(cap));
  int in_f[V], in_b[V], in_f2[V], in_b2[V];   // first slot of each chunk's inputs, per direction
#pragma unroll
  for (int c = 0; c < V; ++c) {
    in_f[c] = dev[2 + c];
    in_b[c] = dev[2 + V + c];
    in_f2[c] = DEG2 ? dev[2 + 2 * V + c] : 0;
    in_b2[c] = DEG2 ? dev[2 + 3 * V + c] : 0;
    // have the constants in registers before the loop: a wait for them inside the loop would
    // also wait for the op-window load in flight
    asm volatile("" : "+v"(in_f[c]), "+v"(in_b[c]), "+v"(in_f2[c]), "+v"(in_b2[c]));
  }
  const int words_per_chunk = (m + 7) >> 3;

  const size_t row_index = (size_t)(active ? cand : 0) * T.D + dd;
  const uint16_t* row = ops + row_index * (size_t)stride;
  uint16_t* out_row = ops_out + row_index * (size_t)stride_out;
  int cursor = 0, out_len = 0;
  unsigned free_at8 = 0, busy8 = 0;
  int mem = 0, pk = 0;
  bool done = !active, halted = false, overflow = false, seg_live = true;
  // op window: words [loaded - kWin, loaded) of the row are in the ring; the head of the row is
  // fetched before the first round
  int loaded = 0;
  uint4 pend = make_uint4(0u, 0u, 0u, 0u);
  bool has_pend = false;
  auto land = [&](uint4 v) {   // eight words: a 16-byte piece of the row (strides are multiples of 8)
    const int q = loaded & (kWin - 1);
    win[(q + 0) * 64] = (uint16_t)v.x; win[(q + 1) * 64] = (uint16_t)(v.x >> 16);
    win[(q + 2) * 64] = (uint16_t)v.y; win[(q + 3) * 64] = (uint16_t)(v.y >> 16);
    win[(q + 4) * 64] = (uint16_t)v.z; win[(q + 5) * 64] = (uint16_t)(v.z >> 16);
    win[(q + 6) * 64] = (uint16_t)v.w; win[(q + 7) * 64] = (uint16_t)(v.w >> 16);
    loaded += 8;
  };
  if (active) {
    land(*reinterpret_cast<const uint4*>(row));
    if (stride > 8) land(*reinterpret_cast<const uint4*>(row + 8));
  }
  // the new row leaves in 16-byte pieces: eight words shifted into four registers
  unsigned acc0 = 0u, acc1 = 0u, acc2 = 0u, acc3 = 0u;
  auto shift_in = [&](unsigned word) {
    acc0 = __builtin_amdgcn_alignbit(acc1, acc0, 16);
    acc1 = __builtin_amdgcn_alignbit(acc2, acc1, 16);
    acc2 = __builtin_amdgcn_alignbit(acc3, acc2, 16);
    acc3 = (acc3 >> 16) | (word << 16);
  };
  // stash ring: entries [q_head, q_tail); `overflowed`: B words from row position refill_pos on
  // found no room and are still to be read back from the row
  int q_head = 0, q_tail = 0, refill_pos = 0;
  bool overflowed = false;

  // The item at the list cursor, decoded when the cursor moves: its metadata rows and the LDS
  // indices of its state word and input slots stay in registers while the device waits for it.
  unsigned w = 0u;
  int4 M = make_int4(0, 0, 15, 0);
  int2 M2 = make_int2(0, 0);
  bool malformed = false;
  bool need_word = true;   // the word at the list cursor has not been decoded yet
  int x_state = lane, x_in = 0, x_in2 = 0;
  auto decode = [&](unsigned word) {
    w = word;
    need_word = false;
    const unsigned j = word & 0x7ffu, c5 = word >> 11, c = c5 & 3u, kind = word >> 13;
    M = meta[c5 * lpc + d];
    malformed = kind != (unsigned)kEnd && (j >= (unsigned)m || ((unsigned)M.z & 15u) == 15u);
    const unsigned jc = min(j, (unsigned)m - 1u), cc = min(c, (unsigned)(V - 1));   // (indices stay inside LDS)
    x_state = (int)((cc * words_per_chunk + (jc >> 3)) * 64u) + lane;
    const bool is_b = kind == (unsigned)kB, has_edges = is_b || kind == (unsigned)kF || kind == (unsigned)kFD;
    int base = 0, base2 = 0;
#pragma unroll
    for (int i = 0; i < V; ++i) {
      base = ((int)cc == i) ? (is_b ? in_b[i] : in_f[i]) : base;
      base2 = ((int)cc == i) ? (is_b ? in_b2[i] : in_f2[i]) : base2;
    }
    x_in = base + (int)jc;
    x_in2 = base2 + (int)jc;
    M2 = make_int2(0, 0);
    if (DEG2 && has_edges) M2 = meta2[((is_b ? 4u : 0u) + cc) * lpc + d];
  };
  // The oldest stashed item: the B word at the stash cursor as a W word, and its metadata row.
  unsigned q_word = 0u;
  int4 Mq = make_int4(0, 0, 15, 0);
  auto stash_head = [&](unsigned b_word) {
    q_word = (b_word & 0x1fffu) | ((unsigned)kW << 13);
    Mq = meta[(q_word >> 11) * lpc + d];
  };
  // a B word joins the stash (false: the ring is full)
  auto stash_push = [&](unsigned b_word) -> bool {
    if (q_tail - q_head >= kFifo) return false;
    fifo[(q_tail & (kFifo - 1)) * 64] = (uint16_t)b_word;
    if (q_tail == q_head) stash_head(b_word);
    ++q_tail;
    return true;
  };
  // the word at the list cursor, if it is in the window (or the row is over)
  auto fetch = [&]() {
    if (cursor >= stride) decode(0u);
    else if (cursor < loaded) decode(win[(cursor & (kWin - 1)) * 64]);
  };
  // The item issues at start8: the word joins the new row (false: the row is full), the device's
  // clock, memory and the activation state move on, the finish time goes to the output slots.
  auto issue = [&](unsigned word, const int4& Mo, const int2& M2o, unsigned start8) -> bool {
    if (out_len < stride_out) {
      shift_in(word);
      if ((out_len & 7) == 7) *reinterpret_cast<uint4*>(out_row + (out_len - 7)) = make_uint4(acc0, acc1, acc2, acc3);
      ++out_len;
    } else {
      overflow = true;   // the row keeps its first stride_out items; the candidate is reported as failed
    }
    const unsigned j = word & 0x7ffu, c = (word >> 11) & 3u;
    const unsigned fin8 = start8 + (unsigned)Mo.x;
    mem += (int)((unsigned)Mo.w & 0xffu);
    pk = max(pk, mem);
    mem -= (int)(((unsigned)Mo.w >> 8) & 0xffu);
    stt[(c * words_per_chunk + (j >> 3)) * 64 + lane] ^= (((unsigned)Mo.z >> 8) & 0xffu) << ((j & 7u) * 4u);
    const unsigned val = fin8 | (((unsigned)Mo.w >> 16) & 0xffu);
    my_slots[j + ((unsigned)Mo.z >> 18)] = val;   // an item without an output edge writes the dump region
    if (DEG2 && ((unsigned)M2o.y & kMetaHasProd)) my_slots[j + (((unsigned)M2o.y & 0xffffu) >> 2)] = val;
    free_at8 = fin8;
    busy8 += (unsigned)Mo.x;
    return true;
  };
  if (active) fetch();

  // the shortest W item of the device: idle time below it takes no stashed item, whichever is oldest
  unsigned min_w8 = 0xffffffffu;
  if (active)
    for (int c = 0; c < dev[0]; ++c) min_w8 = min(min_w8, (unsigned)meta[((int)kW * 4 + c) * lpc + d].x);

  // A round, per device: look at the item at the list cursor (can it start, and when); run the
  // oldest stashed item if the list is over or that item leaves room for it; issue the item of the
  // list in the same round unless another stashed item might still fit in front of it (then the
  // next round decides); pass over a W word of the input.  Every round but the last of a candidate
  // does one of these on some device, or some device waits for its window (fewer than eight
  // rounds per four words).
  const long long max_rounds = (long long)T.D * (3ll * stride + stride_out + 1) + 64;
  for (long long round = 0; round < max_rounds; ++round) {
    // wave-wide top-up of the op windows: what was requested four rounds ago lands now
    if ((round & 3) == 0) {
      if (has_pend) {
        land(pend);
        has_pend = false;
      }
      if (!done && !halted && seg_live && loaded - cursor <= 8 && loaded < stride) {
        pend = *reinterpret_cast<const uint4*>(row + loaded);
        has_pend = true;
      }
    }
    bool progressed = false;
    const bool running = !done && !halted && seg_live;
    if (running && need_word) {
      fetch();
      progressed = need_word;   // still waiting for its window: the device is not stuck
    }
    const bool live = running && !need_word;
    const unsigned kind = w >> 13;
    const bool at_end = kind == (unsigned)kEnd, at_w = kind == (unsigned)kW;
    // the item at the list cursor (indices are inside LDS whatever the word is)
    const unsigned sx = stt[x_state];
    const unsigned in1 = my_slots[x_in];
    const unsigned in2 = DEG2 ? my_slots[x_in2] : 0u;
    bool x_ok = live && !at_end && !at_w && !malformed && ((sx >> ((w & 7u) * 4u)) & 15u) == ((unsigned)M.z & 15u);
    unsigned ready8 = 0u;
    if ((unsigned)M.w >> 24) {
      const unsigned r = in1 + (unsigned)M.y;   // low byte zero iff the slot carries the upstream stage's tag
      x_ok = x_ok && (r & 0xffu) == 0u;
      ready8 = r;
    }
    if (DEG2 && ((unsigned)M2.y & kMetaHasCons)) {
      const unsigned r = in2 + (unsigned)M2.x;
      x_ok = x_ok && (r & 0xffu) == 0u;
      ready8 = max(ready8, r);
    }
    if (live && malformed) halted = true;
    // when the item of the list starts; at the end of the list stashed items run without a limit
    const unsigned start8 = at_end ? 0xffffffffu : max(free_at8, ready8);
    const bool run_w = live && !malformed && q_head < q_tail && (at_end || x_ok) && free_at8 + (unsigned)Mq.x <= start8;
    if (run_w) {
      if (!issue(q_word, Mq, make_int2(0, 0), free_at8)) {
        halted = true;
      } else {
        ++q_head;
        if (q_head == q_tail && overflowed) {
          // the ring ran empty while B words wait in the row: read them back, up to the list cursor
          int at = refill_pos;
          while (at < cursor && q_tail - q_head < kFifo) {
            const unsigned b_word = row[at];
            if ((b_word >> 13) == (unsigned)kB) stash_push(b_word);
            ++at;
          }
          refill_pos = at;
          overflowed = at < cursor;
        }
        if (q_head < q_tail) stash_head(fifo[(q_head & (kFifo - 1)) * 64]);
      }
      progressed = true;
    }
    // the item of the list issues now unless a stashed item may still fit in front of it
    const bool x_now = x_ok && !halted && (q_head == q_tail || !run_w || start8 - free_at8 < min_w8);
    bool consumed = live && at_w && !malformed;   // where the input put its W items is not used
    if (x_now) {
      if (issue(w, M, M2, start8)) consumed = true; else halted = true;
      progressed = true;
    }
    if (live && at_end && q_head == q_tail && !halted) {
      done = true;   // the list is over and nothing is stashed
      progressed = true;
    }
    if (consumed) {
      // an issued B item stashes its W item; once the ring has overflowed, later ones stay in the row
      if (kind == (unsigned)kB && !overflowed && !stash_push(w)) {
        overflowed = true;
        refill_pos = cursor;
      }
      ++cursor;
      need_word = true;
      fetch();
      progressed = true;
    }
    __builtin_amdgcn_wave_barrier();
    const unsigned long long moved = __ballot(progressed);
    if ((moved & seg_mask) == 0ull) seg_live = false;
    if (moved == 0ull) break;
  }

  // ---- the rest of the new row: END words up to the stride
  if (active) {
    int at = out_len;
    if (at & 7) {
      for (; at & 7; ++at) shift_in(0u);
      *reinterpret_cast<uint4*>(out_row + (at - 8)) = make_uint4(acc0, acc1, acc2, acc3);
    }
    for (; at < stride_out; at += 8) *reinterpret_cast<uint4*>(out_row + at) = make_uint4(0u, 0u, 0u, 0u);
  }
  // ---- the evaluation of the new lists
  bool incomplete = false;
  if (active)
    for (int i = 0; i < T.state_words; ++i) incomplete = incomplete || (stt[i * 64 + lane] != (unsigned)expect[i]);
  const unsigned long long stuck = __ballot(active && (!done || overflow)) & seg_mask;
  const unsigned long long stuck_bad = __ballot(active && (halted || overflow)) & seg_mask;
  const unsigned long long unfinished = __ballot(incomplete) & seg_mask;
  const unsigned long long over = __ballot(active && pk > cap) & seg_mask;
  int ms = active ? (int)(free_at8 >> 8) : 0;
  for (int off = 1; off < lpc; off <<= 1) ms = max(ms, __shfl_xor(ms, off, 64));
  unsigned fl = 0;
  if (stuck) fl = kDeadlock | (stuck_bad ? kIncomplete : 0);
  else if (unfinished) fl = kIncomplete;
  else if (over) fl = kOverCap;
  if (active) {
    const bool failed = (fl & (kDeadlock | kIncomplete)) != 0;
    out_idle[cand * T.D + d] = failed ? -1ll : (long long)(ms - (int)(busy8 >> 8));
    out_peak[cand * T.D + d] = failed ? -1 : pk * T.unit_scale;
    if (d == 0) {
      out_makespan[cand] = failed ? 0x7fffffffffffffffll : (long long)ms;
      out_flags[cand] = (unsigned char)fl;
    }
  }
}

#define FPSCHED_INSTANTIATE(V, G)                                                                              \
  template __global__ void wslide_kernel<V, G>(SlotTables, const uint16_t*, long long, int, uint16_t*, int,   \
                                               long long*, long long*, int*, unsigned char*);
FPSCHED_INSTANTIATE(1, false)
FPSCHED_INSTANTIATE(2, false)
FPSCHED_INSTANTIATE(4, false)
FPSCHED_INSTANTIATE(1, true)
FPSCHED_INSTANTIATE(2, true)
FPSCHED_INSTANTIATE(4, true)
#undef FPSCHED_INSTANTIATE

}  // namespace fpsched

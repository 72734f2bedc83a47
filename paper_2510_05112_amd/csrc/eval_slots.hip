// Slot evaluation kernel: the main path.  Any per-device op order, any stage DAG with
// at most two inputs and two outputs per stage, a few KB of LDS per candidate.
//
// Mapping: a wavefront carries `cands_per_wave` candidate segments, lane = device inside
// a segment; the wavefronts of a workgroup are independent and only share one LDS copy
// of the op-metadata table.  The grid is persistent: whenever a segment finishes a
// candidate it takes the next unevaluated one (from a global counter, through a small pool per
// wavefront so that short candidates do not pay one atomic each) and restarts while
// the other segments of the wavefront keep going, so fast and slow candidates (and
// unevenly loaded SIMDs) balance out.  Each lane walks its device's list
// with a cursor in registers; a lane whose next op cannot issue yet waits for a later
// round, and a round in which no lane of a segment moves ends that candidate (lists
// exhausted, or deadlock).
//
// Cross-stage finish times travel through per-micro-batch mail slots.  The edges of
// the stage DAG are split on the host into classes (chains of edges in which each edge
// starts at the stage the previous one ends in; a plain pipeline is one class).  For
// one micro-batch at most one edge of a class carries a live value at a time -- the
// value of F(a,j) on edge a->b is dead once F(b,j) has issued, and only then can the
// next edge of the class be produced -- so a class needs ONE slot per micro-batch and
// direction, tagged with the stage that produced it: slot[dir][class][j] =
// finish << 8 | producer stage.  A consumer finds its input iff the tag names its
// upstream stage.  No order of micro-batches is assumed and a producer never has to
// wait for room.
//
// Same-device ordering rules are the activation state machine of one (stage,
// micro-batch), 4 bits per entry, in lane-private LDS words.  Op words are staged
// through a lane-private 16-word LDS ring that the whole wavefront tops up with
// 8-byte global loads every fourth round; the load issued at one top-up is only
// written to LDS at the next, so its latency is off the critical path.  Between two
// top-ups run four unrolled rounds; only the last of them looks for finished segments.
//
// A round is straight-line code.  Everything that depends only on the op word -- the LDS
// addresses of its state word and input slot, its 16-byte metadata row (duration, latency,
// expected input tag, state transition, memory deltas, output slot; addressed by the top five
// bits of the word and the device) and the word behind it -- is worked out and fetched when the
// lane issues the previous op and kept in registers, so a blocked lane repeats no decoding; a
// round reads the state word and the input slot (one LDS round trip), decides with one byte
// compare, and on success updates the lane's registers, the state word and the output slot.
// Times are kept shifted left by eight bits, the way a slot holds them (finish << 8 | producer
// stage): adding the row's (latency << 8) - expected tag to a slot value yields the ready time
// with a low byte that is zero iff the slot carries the expected tag, so one addition serves
// the dependency test and the start rule.  Whether a candidate completed (every activation
// consumed) and whether a stuck device sits on a malformed word are decided once, when it ends.
//
// Start rule (paper Section 5.1 "Data dependency"; estimator sketch after Section 6):
// start = max(device free, finish of each cross-stage input + latency if the input ran
// on another device); finish = start + dur[kind][stage].
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

namespace fpsched {

namespace {

// LDS accesses by 32-bit LDS address (the per-lane addresses are kept as integers so that ring
// positions and table offsets can be OR-ed / multiplied into them)
#define FPSCHED_LDS __attribute__((address_space(3)))
template <class T>
__device__ __forceinline__ T lds_read(unsigned a) {
  return *reinterpret_cast<const FPSCHED_LDS T*>(a);
}
typedef int lds_int4 __attribute__((ext_vector_type(4)));
typedef int lds_int2 __attribute__((ext_vector_type(2)));
template <>
__device__ __forceinline__ int4 lds_read<int4>(unsigned a) {
  const lds_int4 v = *reinterpret_cast<const FPSCHED_LDS lds_int4*>(a);
  return make_int4(v.x, v.y, v.z, v.w);
}
template <>
__device__ __forceinline__ int2 lds_read<int2>(unsigned a) {
  const lds_int2 v = *reinterpret_cast<const FPSCHED_LDS lds_int2*>(a);
  return make_int2(v.x, v.y);
}
template <class T>
__device__ __forceinline__ void lds_write(unsigned a, T v) {
  *reinterpret_cast<FPSCHED_LDS T*>(a) = v;
}

// One value per chunk of a device, kept as ONE vector value: as an array of four ints the compiler turns the
// select chain below into a load with a variable index and puts the array into scratch memory.
template <int V>
struct PerChunk { typedef int type __attribute__((ext_vector_type(V))); };
template <int V>
__device__ __forceinline__ int pick(typename PerChunk<V>::type a, int c) {
  int r = a[0];
#pragma unroll
  for (int i = 1; i < V; ++i) r = (c == i) ? a[i] : r;
  return r;
}

// Op window: kRing words per lane, refilled kChunk words at a time every kSyncRounds rounds.
// A lane asks for its next chunk when at most kRefillAt words are left unread; with these
// values a lane that issues one op per round always finds the second word after its cursor in
// the ring (at least 6 unread words after every top-up, at most 13 <= kRing), and the word at
// its cursor is never overwritten.
constexpr int kRing = 16;
constexpr int kChunk = 4;
constexpr unsigned kSyncRounds = 4;
constexpr int kRefillAt = 9;
constexpr int kPrimeChunks = 3;

}  // namespace

__global__ void reset_counter_kernel(unsigned long long* counter, unsigned long long value) {
  if (threadIdx.x == 0) *counter = value;
}

// MODE kSlotTimes (TIMES below) is the first pass of the weight-gradient sliding (wslide.hip): the tables then
// describe the lists without their W items (a W word is a no-op that always issues at once), and
// instead of makespan, idle and peak the kernel writes, per op word, the low sixteen bits of the time
// the op started (eight positions of a device are 16 bytes, and the 16-byte pieces of a candidate's
// devices for the same eight positions lie side by side, [candidate][stride / 8][lanes per
// candidate][8]: the lanes of a candidate pass a position at about the same time, so a line fills up
// quickly) and, per device, the position at which its list stopped.  The second pass rebuilds a start
// time from the device's free time in front of the op, which it knows: start = free + ((low - free) mod
// 2^16).  That is exact while the op waits less than 2^16 time units for its inputs; an op that waits
// longer -- there are at most (largest possible finish time) / 2^16 of them in a row -- leaves an
// entry (position << 8 | wait >> 16) in the row's escape list, which ends with an all-ones word.
//
// MODE kSlotPerMicrobatch: the cost of an item depends on its micro-batch as well (micro-batches of
// unequal size).  The duration then comes from mb_rows [32 metadata rows][lanes per candidate][m]
// (cost << 8, zero for rows the device does not have) in device memory instead of the metadata row;
// it is requested when the word is decoded and first needed one round later.  That wait also
// covers the op-window load in flight, so the form is about twice as slow as the plain kernel.
// MODE kSlotPerMicrobatchLds: the same costs as values of one or two bytes in the shared part of LDS
// (T.off_mb), read like the metadata row; the host picks it when the table fits.
//
// MODE kSlotLinks: the link-occupancy variant of the cost model.  Every device a lane's device sends
// to has a word behind the lane's state words: the time until which that link is busy.  An op with an
// outgoing edge to another device writes into its output slot not its finish time but the time its
// value leaves, max(finish, link busy until), and keeps the link busy for the edge's latency from then;
// the consumer adds the latency as before.  The link word of the current op is read when the op is
// decoded (only the lane itself ever writes it, in program order before that read).
//
// MODE kSlotCopy: the copy-engine variant of the cost model (the paper names CPU offloading without saying how
// an offload is timed).  Offload and reload items run on a copy timeline of the device: the walk through the
// list hands such an item to the engine when it reaches it and goes on at once, unless T.copy_depth transfers
// are still unfinished (then it waits for the oldest of them); a transfer starts at max(hand-over, finish of the
// transfer before it).  A backward item waits for the reload of its activation: a reload sets bit 3 of the
// activation's state nibble (the decision looks at the low three bits only), and a backward item that finds the
// bit looks for its (chunk, micro-batch) among the last copy_depth transfers, which a lane keeps in a ring
// (older ones have finished before the walk got here).  Memory becomes a sum over events in time order: the
// transfers' events (a reload allocates at its start, an offload releases at its end) wait in a second ring
// and are applied as the walk passes their time, compute events first at equal times.  Transfers are no busy
// time; the makespan covers both timelines.
//
// MODE kSlotSync: stages whose items stand for groups of micro-batches (a synchronisation every n micro-batches,
// Section 4.2 / 7.2 of the paper) and dependency pairs between items of one direction.  An item of a stage with
// group n waits for the n values of its micro-batches, one slot per round: the lane keeps how many are still to
// come and the latest arrival so far, moves its input address on whenever the slot it looks at carries the
// expected tag, and may issue when the last one does; when it issues it writes its result into the n slots of
// its micro-batches.  Its state nibble is indexed by the item, its slots by the micro-batches.  (The host only
// selects this form when the neighbours of such a stage have one item per micro-batch.)  A pair (F, a) -> (F, b) or
// (B, a) -> (B, b) is an edge of its own slot class in one direction only.
//
// MODE kSlotSlide: the weight-gradient sliding pass (Section 5.2, bubble optimizations) when only the results of
// the new lists are wanted.  The tables are those of kSlotTimes (a W word of the input is a no-op), so every item
// starts when it would start without any W item; a B item that issues stashes its W item, and in front of every
// item the lane runs the oldest stashed items that end before the item starts (only the oldest is tried).  Of the
// stash a lane needs nothing but the chunks of its entries, oldest first: a queue of log2(V) bits per entry in one
// register (entries that find no room stay in the row and are read back from there, at the next top-up, when the
// queue has run empty).  What is still stashed when a list ends runs back to back behind it: a device's last finish time is
// its free time plus the cost of the W items it has not placed.
template <int V, bool DEG2, bool ONE_CLASS, int MODE>
__global__ __launch_bounds__(kSlotMaxThreads) void eval_slot_kernel(
    SlotTables T, const uint16_t* __restrict__ ops, long long n_cand, int stride,
    long long* __restrict__ out_makespan, long long* __restrict__ out_idle,
    int* __restrict__ out_peak, unsigned char* __restrict__ out_flags,
    unsigned long long* __restrict__ next_candidate, int draw_block,
    uint32_t* __restrict__ out_start8, int32_t* __restrict__ out_stop, const int32_t* __restrict__ mb_rows,
    uint32_t* __restrict__ out_escape, int escape_cap) {
  constexpr bool TIMES = MODE == kSlotTimes || MODE == kSlotTimesLinks;
  constexpr bool MBDUR = MODE == kSlotPerMicrobatch;
  constexpr bool MBLDS = MODE == kSlotPerMicrobatchLds || MODE == kSlotPerMicrobatchLdsLinks;
  constexpr bool LINKS = MODE == kSlotLinks || MODE == kSlotTimesLinks || MODE == kSlotPerMicrobatchLdsLinks || MODE == kSlotSlideLinks;
  constexpr bool COPY = MODE == kSlotCopy;
  constexpr bool SYNC = MODE == kSlotSync;
  constexpr bool SLIDE = MODE == kSlotSlide || MODE == kSlotSlideLinks;
  constexpr bool W_NOOP = TIMES || SLIDE;   // the tables describe the lists without their W items
  // SLIDE: bits per queue entry, entries the queue holds
  constexpr unsigned kQBits = V == 1 ? 0u : (V == 2 ? 1u : 2u);
  constexpr unsigned kQCap = V == 1 ? 0x7fffffffu : 32u / (kQBits ? kQBits : 1u);
  constexpr unsigned kRefillStall = 0x100u;   // value of `dead` while a lane waits for its queue to be read back
  extern __shared__ int32_t lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m = T.m;
  const int cpw = T.cands_per_wave;
  const int lpc = T.lanes_per_cand;
  const int lpc_shift = __ffs(lpc) - 1;

  // LDS: [metadata, padded to 2 KB][one 2 KB op window per wave][per wave: state words, slots].
  // A window is 2 KB-aligned so that a ring position can be OR-ed into its address.
  for (int i = tid; i < T.n_shared_ints; i += blockDim.x) lds[i] = T.ints[i];
  char* const L = reinterpret_cast<char*>(lds);
  const unsigned lds0 = (unsigned)(size_t)(FPSCHED_LDS char*)lds;   // LDS address of the array
  const unsigned shared_bytes = (unsigned)T.n_shared_ints * 4u;
  const unsigned rest_ints = (unsigned)T.wave_ints - (kRing / 2) * 64u;
  const unsigned rest_off = shared_bytes + (blockDim.x >> 6) * (kRing * 128u) + wave * rest_ints * 4u;
  // window: kRing sixteen-bit words per lane, laid out [word][lane]
  uint16_t* win = reinterpret_cast<uint16_t*>(L + shared_bytes + wave * (kRing * 128u));
  uint32_t* stt = reinterpret_cast<uint32_t*>(L + rest_off);              // [state word][lane]
  const int lane_words = T.state_words + (LINKS || COPY ? T.link_words : 0);   // state words, then link words / rings
  uint32_t* slots = stt + lane_words * 64;
  const int slots_per_cand = T.slots_per_cand;  // backward, forward, dump; a multiple of 8
  // TIMES, SLIDE: one dword behind the last wavefront's region stays zero; it is the state word of W words
  const unsigned zero_off = shared_bytes + (blockDim.x >> 6) * (kRing * 128u + rest_ints * 4u);
  if (W_NOOP && tid == 0) *reinterpret_cast<uint32_t*>(L + zero_off) = 0u;
  __syncthreads();

  const int seg = lane >> lpc_shift;
  const int d = lane & (lpc - 1);
  const bool lane_ok = (seg < cpw) && (d < T.D);
  uint32_t* my_slots = slots + (seg < cpw ? seg : 0) * slots_per_cand;
  long long cand = 0;

  // per-device constants: memory cap, byte offsets of the input slots of each chunk
  const int dd = d < T.D ? d : 0;
  const int32_t* dev = T.ints + T.off_dev + dd * T.dev_ints;
  const int32_t* expect = T.ints + T.off_expect + dd * T.state_words;
  int cap = dev[1];
  typename PerChunk<V>::type cons_f, cons_b, cons_f2, cons_b2;
#pragma unroll
  for (int c = 0; c < V; ++c) {
    int f = dev[2 + c] << 2, b = dev[2 + V + c] << 2;
    int f2 = DEG2 ? dev[2 + 2 * V + c] << 2 : 0, b2 = DEG2 ? dev[2 + 3 * V + c] << 2 : 0;
    // have the constants in registers before the loop: a wait for them inside the loop would
    // also wait for the op-window prefetch
    asm volatile("" : "+v"(f), "+v"(b), "+v"(f2), "+v"(b2));
    cons_f[c] = f; cons_b[c] = b; cons_f2[c] = f2; cons_b2[c] = b2;
  }
  asm volatile("" : "+v"(cap));
  // LINKS: per chunk the out-edges as latency << 16 | byte offset of the link word
  typename PerChunk<V>::type out_f, out_b, out_f2, out_b2;
#pragma unroll
  for (int c = 0; c < V; ++c) {
    int f = LINKS ? dev[2 + 4 * V + c] : 0, b = LINKS ? dev[2 + 5 * V + c] : 0;
    int f2 = LINKS && DEG2 ? dev[2 + 6 * V + c] : 0, b2 = LINKS && DEG2 ? dev[2 + 7 * V + c] : 0;
    if (LINKS) asm volatile("" : "+v"(f), "+v"(b), "+v"(f2), "+v"(b2));
    out_f[c] = f; out_b[c] = b; out_f2[c] = f2; out_b2[c] = b2;
  }
  // SYNC: per chunk the micro-batches per item (1: an ordinary stage) | items << 16
  typename PerChunk<V>::type grp;
#pragma unroll
  for (int c = 0; c < V; ++c) {
    int g = SYNC ? dev[2 + 4 * V + c] : 0;
    if (SYNC) asm volatile("" : "+v"(g));
    grp[c] = g;
  }
  const unsigned long long seg_mask =
      (lpc == 64 ? ~0ull : ((1ull << lpc) - 1ull)) << (seg * lpc);
  // LDS byte offsets of this lane's columns
  const unsigned row_bytes = (unsigned)lpc << 4;          // one metadata row: 16 bytes per device
  const unsigned meta_off = lds0 + ((unsigned)d << 4);
  const unsigned meta2_off = lds0 + (unsigned)T.off_meta2 * 4u + ((unsigned)d << 3);
  const unsigned words_per_chunk = (unsigned)(m + 7) >> 3;
  const unsigned win_off = lds0 + shared_bytes + wave * (kRing * 128u) + lane * 2u;   // word k at + k * 128
  const unsigned stt_off = lds0 + rest_off + lane * 4u;                               // word i at + i * 256
  // slots of this lane's candidate; the offset is a multiple of 32, so that the low five bits of
  // (slot_base + 4 j) are the position of micro-batch j's nibble in its state word
  const unsigned slot_base_ = lds0 + rest_off + (unsigned)lane_words * 256u +
                             (unsigned)(seg < cpw ? seg : 0) * (unsigned)slots_per_cand * 4u;
  const unsigned m4 = (unsigned)m << 2;
  const unsigned chunk_bytes = words_per_chunk << 8;   // state words of one chunk, all lanes
  unsigned slot_base = slot_base_;
  asm volatile("" : "+v"(slot_base));   // one register, not a sum to be re-associated every round
  // segment bookkeeping on the scalar unit: bit (seg * lpc) stands for segment seg
  unsigned long long base_bits = 0ull;
  for (int sgm = 0; sgm < cpw; ++sgm) base_bits |= 1ull << (sgm * lpc);
  int fold_shift[6];   // shifts 1, 2, 4, ... below the segment width, then 0 (no-ops)
#pragma unroll
  for (int i = 0; i < 6; ++i) fold_shift[i] = (1 << i) < lpc ? (1 << i) : 0;
  const unsigned long long high_bits = base_bits << (lpc - 1);
  unsigned long long run_bases = 0ull;   // base bits of the segments that are evaluating a candidate
  unsigned long long idle_fields = ~0ull;  // all lanes of the segments that are not
  bool any_special = true;               // wave-uniform: some segment starts, or has just started, a candidate

  // per-candidate registers
  const uint16_t* row = ops;
  int loaded = 0;  // words of this row already in the window ring
  uint2 pend = make_uint2(0, 0);
  bool has_pend = false;
  unsigned npos = 128u;              // (list position + 1) << 7 (the byte stride of the window ring)
  unsigned free_at8 = 0, busy8 = 0;  // device free time and busy time, << 8
  int mem = 0, pk = 0;               // in units of the problem's common unit divisor
  bool running = false;  // this lane's segment is evaluating a candidate
  unsigned dead = ~0u;   // 0 while this lane carries a device of a running candidate, else all ones
  bool fresh = true;     // (re)start the segment on `cand` at the top of the next round
  // TIMES: the low halves of the start times of the last eight ops, stored 16 bytes at a time at the
  // ops' positions; the row's escape list and its length
  unsigned st0 = 0u, st1 = 0u, st2 = 0u, st3 = 0u;
  uint32_t* start_row = out_start8;
  uint32_t* esc_row = out_escape;
  int n_esc = 0;

  // LDS addresses of everything a round reads for the current word.  They only change when the
  // lane issues, so they are worked out there, once per op, and a round starts with its reads.
  // The word's metadata row is fetched there as well and kept in registers, and so is the op
  // word behind it (a lane that issues the op at position k reads the word at k + 2).
  unsigned at_state = stt_off, at_slot = slot_base, at_in = slot_base, at_in2 = slot_base;
  int4 M = make_int4(0, 0, 15, 0);   // metadata row of the current word (an invalid row to begin with)
  // (SLIDE, SYNC, TIMES: the row as one 16-byte value from its load to the decision, so that it stays in the four
  // registers it was loaded into; as four separate values the register allocator copies some of them right behind
  // the load, which puts a wait for that load in front of the next round's reads.  The other modes measured the
  // same or slightly worse with it.)
  constexpr bool ROW16 = SLIDE || SYNC || TIMES;
  lds_int4 M_row = {0, 0, 15, 0};
  int2 M2 = make_int2(0, 0);         // its second-edge row
  unsigned w_next = 0u;              // the word behind the current one
  // SYNC: the item under the cursor: position of its state nibble, values of its group still to arrive (1: the
  // slot the round looks at is the last), the latest arrival so far, slots to write when it issues
  unsigned at_nib = 0u, gat_left = 1u, acc8 = 0u, n_out = 1u;
  // COPY: the copy timeline of this device.  Rings of eight dwords per lane behind its state words (entry i at
  // + i * 256): finish << 8 of the last transfers, their keys (low 13 bits of a reload's word, all ones for an
  // offload), time << 8 and units of the transfer events that the walk has not passed yet.
  const unsigned ring_fin = stt_off + (unsigned)T.state_words * 256u;
  const unsigned ring_key = ring_fin + 8u * 256u, ring_ev_time = ring_fin + 16u * 256u, ring_ev_units = ring_fin + 24u * 256u;
  const unsigned copy_depth = (unsigned)T.copy_depth;
  unsigned copy_free8 = 0u, n_copy = 0u, ev_head = 0u, ev_tail = 0u;
  unsigned next_ev8 = 0xffffffffu;   // time << 8 of the oldest pending event (all ones: none)
  unsigned cur_kind = 0u, cur_key = 0u;   // kind and (chunk, micro-batch) bits of the current word
  // apply the pending transfer events that come before a compute event at `limit8`
  auto pass_time = [&](unsigned limit8) {
    while (next_ev8 < limit8) {
      mem += (int)lds_read<uint32_t>(ring_ev_units + ((ev_head & 7u) << 8));
      pk = max(pk, mem);
      ++ev_head;
      next_ev8 = ev_head != ev_tail ? lds_read<uint32_t>(ring_ev_time + ((ev_head & 7u) << 8)) : 0xffffffffu;
    }
  };
  // SLIDE: the stash as a queue of chunk indices (oldest entry in the low bits), its length, the cost << 8 of the
  // W items placed so far; whether B items found no room, and from which row position on they are still in the row;
  // the chunk of the current word (what a B word stashes when it issues)
  unsigned q_bits = 0u, q_n = 0u, w_placed8 = 0u, cur_push = 0u;
  unsigned q_over = 0u;   // 1: B items found no room
  int q_refill_at = 0;
  typename PerChunk<V>::type w_dur8, w_free;
  unsigned w_total8 = 0u;
#pragma unroll
  for (int c = 0; c < V; ++c) {
    int wd = SLIDE ? T.ints[T.off_w + dd * (2 * kMaxChunks + 1) + c] : 0;
    int wf = SLIDE ? T.ints[T.off_w + dd * (2 * kMaxChunks + 1) + kMaxChunks + c] : 0;
    if (SLIDE) asm volatile("" : "+v"(wd), "+v"(wf));
    w_dur8[c] = wd; w_free[c] = wf;
  }
  if (SLIDE) {
    w_total8 = (unsigned)T.ints[T.off_w + dd * (2 * kMaxChunks + 1) + 2 * kMaxChunks];
    asm volatile("" : "+v"(w_total8));
  }
  // cost << 8 of the oldest stashed item (all ones: the queue is empty) and the units it frees
  unsigned q_head_dur8 = 0xffffffffu;
  int q_head_free = 0;
  auto new_head = [&]() {
    const unsigned head = V > 1 ? q_bits & (unsigned)(V - 1) : 0u;
    q_head_dur8 = q_n != 0u ? (unsigned)pick<V>(w_dur8, head) : 0xffffffffu;
    q_head_free = pick<V>(w_free, head);
  };
  int dur_mb8 = 0;                   // MBDUR: cost << 8 of the current word
  const unsigned mb_lane = (unsigned)d * (unsigned)m;   // this device's part of a row of mb_rows
  const unsigned mb_row_ints = (unsigned)lpc * (unsigned)m;
  // MBLDS: [block of the kind][chunk][device][micro-batch] costs of one or two bytes (kind 0 maps to block 0).
  // A device's row is an odd number of dwords long, so that the lanes of a candidate, which mostly ask
  // for the same micro-batch, fall into different banks.
  unsigned dur_mb16 = 0;
  const bool mb_wide = T.mb_value_bytes == 2;   // else one byte per value
  const unsigned mb_dev_bytes = slot_mb_row_dwords(m, T.mb_value_bytes) * 4u;
  const unsigned mb_chunk_bytes = (unsigned)lpc * mb_dev_bytes, mb_kind_bytes = mb_chunk_bytes * (unsigned)V;
  unsigned mb_lds_lane = lds0 + (unsigned)T.off_mb * 4u + (unsigned)d * mb_dev_bytes;
  const unsigned mb_kind_map = T.mb_kind_map;
  if (MBLDS) asm volatile("" : "+v"(mb_lds_lane));
  // LINKS: the current op's first out-edge (latency << 13 | link word offset), the address of its link
  // word and that word's value; the second out-edge is looked at when the op issues
  const unsigned link_base = stt_off + (unsigned)T.state_words * 256u;
  const unsigned link_dummy = LINKS ? (unsigned)(T.link_words - 1) * 256u : 0u;
  unsigned spare_at = link_base + link_dummy;
  if (LINKS) asm volatile("" : "+v"(spare_at));
  const unsigned dump_bytes = (unsigned)(2 * T.n_classes * m) * 4u;   // offset of the slots nobody reads
  unsigned out1 = link_dummy, out2 = link_dummy, at_link1 = link_base, lf1 = 0u;
  auto decode = [&](unsigned word) {
    if (COPY) {
      cur_kind = word >> 13;
      cur_key = word & 0x1fffu;
    }
    const unsigned j = word & 0x7ffu;
    const unsigned c5 = word >> 11;
    // (SYNC: the micro-batch field is the item; an item index beyond the stage's count is malformed)
    const unsigned group_items = SYNC ? (unsigned)pick<V>(grp, c5 & (unsigned)(V - 1)) : 0u;
    const unsigned jc = min(j, (SYNC ? max(group_items >> 16, 1u) : (unsigned)m) - 1u);
    // a micro-batch out of range reads row 0 (kind 0), which is invalid and never issues
    if (ROW16) M_row = *reinterpret_cast<const FPSCHED_LDS lds_int4*>(__umul24(j == jc ? c5 : 0u, row_bytes) + meta_off);
    else M = lds_read<int4>(__umul24(j == jc ? c5 : 0u, row_bytes) + meta_off);
    // (c5 < 32, d < lanes per candidate, jc < m: inside the table whatever the word holds)
    if (MBDUR) dur_mb8 = mb_rows[__umul24(c5, mb_row_ints) + mb_lane + jc];
    unsigned c = c5 & (unsigned)(V - 1);
    unsigned fwd = (word >> 13) & 1u;
    unsigned jw = jc >> 3;   // state word of the micro-batch inside its chunk
    // (opaque to the optimiser, which would otherwise turn the multiplications by these small
    // values into longer compare-and-select sequences)
    asm("" : "+v"(c), "+v"(fwd), "+v"(jw));
    unsigned chunk_at = __umul24(c, chunk_bytes) + stt_off;
    asm("" : "+v"(chunk_at));
    at_state = (jw << 8) + chunk_at;
    if (MBLDS) {
      const unsigned block = __builtin_amdgcn_ubfe(mb_kind_map, c5 & 0x1cu, 3);   // nibble `kind` of the map
      const unsigned at_row = __umul24(block, mb_kind_bytes) + mb_lds_lane + __umul24(c, mb_chunk_bytes);
      if (mb_wide) dur_mb16 = lds_read<uint16_t>(at_row + (jc << 1));
      else dur_mb16 = lds_read<uint8_t>(at_row + jc);
    }
    if (W_NOOP) at_state = (word >> 13) == (unsigned)kW ? lds0 + zero_off : at_state;
    if (SLIDE) cur_push = c;
    unsigned j_first = jc;
    if (SYNC) {
      const unsigned n = max(group_items & 0xffffu, 1u);
      at_nib = jc << 2;
      j_first = __umul24(jc, n);
      n_out = min((unsigned)m - j_first, n);
      gat_left = n_out;
      acc8 = 0u;
    }
    at_slot = (j_first << 2) + slot_base;   // slot j of the first class; low five bits = 4 (j & 7)
    const bool is_b = (word >> 13) == (unsigned)kB;
    // one class: backward inputs at slot j, forward inputs at slot m + j; bit 13 of the word is set
    // for F and FD and clear for B (other kinds have no input, whatever they read is ignored)
    at_in = ONE_CLASS ? __umul24(fwd, m4) + at_slot
                      : at_slot + (unsigned)(is_b ? pick<V>(cons_b, c) : pick<V>(cons_f, c));
    if (LINKS) {
      // by direction and chunk only: whether the op has an out-edge at all is known when its metadata
      // row is there, i.e. when it issues (an op without one must not touch a real link word)
      out1 = (unsigned)(is_b ? pick<V>(out_b, c) : pick<V>(out_f, c));
      at_link1 = link_base + (out1 & 0xffffu);
      lf1 = lds_read<uint32_t>(at_link1);
      if (DEG2) out2 = (unsigned)(is_b ? pick<V>(out_b2, c) : pick<V>(out_f2, c));
    }
    if (DEG2) {
      // second-edge rows are per direction, not per kind: only F, FD and B have cross-stage
      // edges, every other kind reads the all-zero ninth row
      const unsigned kind = word >> 13;
      const bool has_edges = is_b || kind == (unsigned)kF || kind == (unsigned)kFD;
      M2 = lds_read<int2>((((has_edges ? (is_b ? 4u : 0u) + c : 8u) << lpc_shift) << 3) + meta2_off);
      at_in2 = at_slot + (unsigned)(is_b ? pick<V>(cons_b2, c) : pick<V>(cons_f2, c));
    }
  };

  // Every candidate ends after at most D * stride + 2 rounds (each round but its last issues at
  // least one of its at most D * stride ops), so the bound below is never reached; it only makes
  // sure the wavefront leaves the loop whatever happens.
  // (SLIDE: a lane may wait a few rounds for its queue to be read back, once per kQCap items at most)
  const unsigned long long per_cand_rounds = (unsigned long long)T.D * (unsigned)stride * (SLIDE ? 2ull : 1ull) + 8ull;
  // (a segment cannot draw more than all candidates; fast segments draw more than their share)
  const unsigned long long my_cands = (unsigned long long)n_cand + 1ull;
  const unsigned long long bound = per_cand_rounds * my_cands;
  const unsigned max_rounds = bound > 0xfffffff0ull ? 0xfffffff0u : (unsigned)bound;
  // The first candidate of a segment is its global index; later ones are drawn from the counter
  // (which the host presets to the number of segments) at the moment they are needed, so that the
  // last candidates of a batch go to whichever segment is free.
  bool first_draw = true;
  // later candidates come from the wavefront's pool [pool_next, pool_end), refilled from the global
  // counter draw_block at a time: one atomic per refill, not one per candidate (a batch of short
  // candidates is otherwise bound by the rate of atomics on one address; long candidates are
  // drawn one by one, so that the last ones of a batch go to whichever segment is free)
  unsigned long long pool_next = 0ull, pool_end = 0ull;
  uint2 prime0 = make_uint2(0, 0), prime1 = make_uint2(0, 0), prime2 = make_uint2(0, 0);
  bool priming = false;      // the segment has requested the head of its rows and waits for the top-up
  const int prime_words = stride < kPrimeChunks * kChunk ? stride : kPrimeChunks * kChunk;
  for (unsigned round = 0; round < max_rounds; round += kSyncRounds) {
    if (SLIDE) {
      // ---- queues that ran empty while B items wait in the row are read back from there, up to the cursor
      const bool stalled = dead == kRefillStall;
      if (__ballot(stalled) != 0ull && stalled) {
        int at = q_refill_at;
        const int cursor = (int)(npos >> 7) - 1;
        while (at < cursor && q_n < kQCap) {
          const unsigned b_word = row[at];
          if ((b_word >> 13) == (unsigned)kB) {
            q_bits |= ((b_word >> 11) & (unsigned)(V - 1)) << (q_n * kQBits);
            ++q_n;
          }
          ++at;
        }
        q_refill_at = at;
        q_over = at < cursor ? 1u : 0u;
        new_head();
        dead = 0u;
      }
    }
    // ---- wave-wide top-up of the op windows.  Loads requested at the previous top-up are landed
    // now, four rounds later, so nobody waits for HBM.
    if (has_pend) {
      const int q = loaded & (kRing - 1);
      // [word][lane] with 16-bit elements: word k of lane l at k * 64 + l
      win[(q + 0) * 64 + lane] = (uint16_t)pend.x; win[(q + 1) * 64 + lane] = (uint16_t)(pend.x >> 16);
      win[(q + 2) * 64 + lane] = (uint16_t)pend.y; win[(q + 3) * 64 + lane] = (uint16_t)(pend.y >> 16);
      loaded += kChunk;
      has_pend = false;
      // a row that fills its stride has no END word: plant one behind it
      if (loaded >= stride) win[(stride & (kRing - 1)) * 64 + lane] = 0;
    }
    // (a lane that has reached its END word still tops up until its ring is full: harmless, the
    // words are inside its row)
    if (dead == 0u && loaded + 1 - (int)(npos >> 7) <= kRefillAt && loaded < stride) {
      pend = *reinterpret_cast<const uint2*>(row + loaded);
      has_pend = true;
    }
    // ---- the rare part, only when some segment starts or has just started a candidate
    if (any_special) {
      // segments restarted at the previous top-up: their row heads have arrived, they join in
      if (priming && lane_ok) {
        win[0 * 64 + lane] = (uint16_t)prime0.x; win[1 * 64 + lane] = (uint16_t)(prime0.x >> 16);
        win[2 * 64 + lane] = (uint16_t)prime0.y; win[3 * 64 + lane] = (uint16_t)(prime0.y >> 16);
        win[4 * 64 + lane] = (uint16_t)prime1.x; win[5 * 64 + lane] = (uint16_t)(prime1.x >> 16);
        win[6 * 64 + lane] = (uint16_t)prime1.y; win[7 * 64 + lane] = (uint16_t)(prime1.y >> 16);
        if (prime_words > 8) {
          win[8 * 64 + lane] = (uint16_t)prime2.x; win[9 * 64 + lane] = (uint16_t)(prime2.x >> 16);
          win[10 * 64 + lane] = (uint16_t)prime2.y; win[11 * 64 + lane] = (uint16_t)(prime2.y >> 16);
        }
        loaded = prime_words;
        if (loaded >= stride) win[(stride & (kRing - 1)) * 64 + lane] = 0;
        decode(prime0.x & 0xffffu);
        w_next = prime0.x >> 16;
        dead = 0u;
      }
      priming = false;
      // (re)start segments on their next candidate: reset their LDS, request the head of their
      // rows; they join in at the next top-up
      // hand the segments that ask for one (lane 0 of each speaks for it) their next candidate
      const unsigned long long want = __ballot(fresh && !first_draw && d == 0 && seg < cpw);
      unsigned long long from_pool = 0ull;
      if (want != 0ull) {
        const int n_want = __popcll(want);
        const int have = (int)(pool_end - pool_next);
        unsigned long long new_base = 0ull;
        int amount = 0;
        if (n_want > have) {
          amount = max(draw_block, n_want - have);
          if (lane == 0) new_base = atomicAdd(next_candidate, (unsigned long long)amount);
          new_base = __shfl(new_base, 0, 64);
        }
        const int rank = __popcll(want & ((1ull << lane) - 1ull));   // among the asking segments
        from_pool = rank < have ? pool_next + (unsigned)rank : new_base + (unsigned)(rank - have);
        if (n_want > have) {
          pool_next = new_base + (unsigned)(n_want - have);
          pool_end = new_base + (unsigned)amount;
        } else {
          pool_next += (unsigned)n_want;
        }
      }
      if (fresh) {
        fresh = false;
        unsigned long long drawn = ((unsigned long long)blockIdx.x * (blockDim.x >> 6) + wave) * cpw + seg;
        if (!first_draw) drawn = __shfl(from_pool, seg << lpc_shift, 64);
        first_draw = false;
        cand = (long long)drawn;
        running = (seg < cpw) && (cand < n_cand);
        priming = running;
        dead = ~0u;
        npos = 128u; free_at8 = 0; busy8 = 0; mem = 0; pk = 0;
        copy_free8 = 0u; n_copy = 0u; ev_head = 0u; ev_tail = 0u; next_ev8 = 0xffffffffu;
        q_bits = 0u; q_n = 0u; w_placed8 = 0u; cur_push = 0u; q_over = 0u; q_refill_at = 0; q_head_dur8 = 0xffffffffu;
        has_pend = false;
        loaded = 0;
        if (running) {
          for (int i = d; i < slots_per_cand; i += lpc) my_slots[i] = kEmptySlot;
        }
        if (running && lane_ok) {
          for (int i = 0; i < lane_words; ++i) stt[i * 64 + lane] = 0u;
          if (COPY)   // no transfer yet: keys that no word has
            for (unsigned i = 0; i < 8u; ++i) lds_write<uint32_t>(ring_key + (i << 8), 0xffffffffu);
          row = ops + ((size_t)cand * T.D + d) * (size_t)stride;
          // start times: [candidate][group of eight positions][lane of the candidate][8 x 16 bits]
          if (TIMES) {
            start_row = out_start8 + (size_t)cand * ((size_t)stride >> 1) * (size_t)lpc + ((size_t)d << 2);
            esc_row = out_escape + ((size_t)cand * T.D + d) * (size_t)escape_cap;
            n_esc = 0;
          }
          prime0 = *reinterpret_cast<const uint2*>(row);
          prime1 = *reinterpret_cast<const uint2*>(row + kChunk);
          if (prime_words > 8) prime2 = *reinterpret_cast<const uint2*>(row + 2 * kChunk);
        }
      }
      // segments that are priming do not count as running yet (nothing can move in them)
      const unsigned long long all_running = __ballot(running);
      const unsigned long long primers = __ballot(priming);
      const unsigned long long run_lanes = all_running & ~primers;
      run_bases = run_lanes & base_bits;
      idle_fields = ~run_lanes;
      any_special = primers != 0ull;
      if (all_running == 0ull) break;  // every segment of the wave is out of work
    }
    // kSyncRounds rounds between two top-ups; a segment that finishes in between idles until
    // the next top-up, where it is restarted
#pragma unroll
    for (unsigned sub = 0; sub < kSyncRounds; ++sub) {
    // ---- this round's reads
    unsigned sx = lds_read<uint32_t>(at_state);
    unsigned in1 = lds_read<uint32_t>(at_in);
    const unsigned bj = at_slot;
    unsigned in2 = 0u;
    if (DEG2) {
      in2 = lds_read<uint32_t>(at_in2);
      asm volatile("" : "+v"(in2), "+v"(M2.x), "+v"(M2.y));
    }
    // keep every load of the round in front of the decision (one LDS round trip per round)
    // (the metadata row was requested when the lane last issued; nothing may wait for it earlier)
    if (ROW16) {
      asm volatile("" : "+v"(sx), "+v"(in1), "+v"(M_row));
      M = make_int4(M_row.x, M_row.y, M_row.z, M_row.w);
    } else {
      asm volatile("" : "+v"(sx), "+v"(in1), "+v"(M.x), "+v"(M.y), "+v"(M.z), "+v"(M.w));
    }
    // ---- decide.  An exhausted lane sits on a word of kind 0, whose metadata row is invalid; invalid
    // rows require state 15, which no activation is ever in.  Lanes without a device (and idle
    // segments) never initialise their LDS words, so they are masked off explicitly.
    const unsigned dur8 = MBDUR ? (unsigned)dur_mb8 : (MBLDS ? dur_mb16 << 8 : (unsigned)M.x), lat_tag = (unsigned)M.y, mx_ = (unsigned)M.z, my_ = (unsigned)M.w;
    // Everything that can forbid the issue is OR-ed into the low byte of one word: wrong activation
    // state; input slot not tagged with the upstream stage (only if the op has an input: the top
    // byte of the last metadata dword is 0xff then, else 0).  A live lane has dead == 0, any other
    // lane all ones, which the word never equals.
    // (COPY: bit 3 of the nibble only says that the activation was reloaded)
    const unsigned state = __builtin_amdgcn_ubfe(sx, SYNC ? at_nib : bj, COPY ? 3 : 4);
    unsigned ready8 = (in1 + lat_tag) & (unsigned)((int)my_ >> 24);
    // (only the low byte counts: the state nibble is clean, byte 0 of the third metadata dword
    // holds nothing but the required state, and the ready time sits above its tag byte)
    unsigned veto = __builtin_amdgcn_bitop3_b32(state, mx_, ready8, 0xbe);   // (state ^ mx_) | ready8
    unsigned tag_bits = ready8;   // low byte zero iff every input slot carries its expected tag
    if (DEG2) {
      const unsigned ready2 = (in2 + (unsigned)M2.x) & (unsigned)(M2.y >> 31);
      veto |= ready2;
      if (SYNC) tag_bits |= ready2;
      ready8 = max(ready8, ready2);
    }
    unsigned long long gathered = 0ull;
    if (SYNC) {
      // an item that still waits for more values of its group takes the one in front of it, if it is there
      // (the tags say so), and looks at the next slot in the next round
      // (an item without an input has nothing to gather; nor has a malformed word, whose row says so too)
      const bool more = gat_left > 1u && (my_ >> 24) != 0u;
      const bool arrived = ((tag_bits & 0xffu) | dead) == 0u && more;
      gathered = __ballot(arrived);
      veto |= more ? 1u : 0u;
      if (arrived) {
        acc8 = max(acc8, ready8);
        at_in += 4u;
        if (DEG2) at_in2 += 4u;
        gat_left -= 1u;
      }
      ready8 = max(ready8, acc8);
    }
    // one compare of the low byte against `dead` yields the issue mask
    unsigned long long moved;
    asm volatile("v_cmp_eq_u32_sdwa %0, %1, %2 src0_sel:BYTE_0 src1_sel:DWORD"
                 : "=s"(moved) : "v"(veto), "v"(dead));
    const bool ok = __builtin_amdgcn_inverse_ballot_w64(moved);
    // ---- issue
    const bool transfer = COPY && (cur_kind - (unsigned)kO) < 2u;   // kO, kL
    if (COPY && ok && transfer) {
      // hand the transfer to the engine (waiting for room), time it on the copy timeline
      unsigned handover8 = free_at8;
      if (n_copy >= copy_depth) handover8 = max(handover8, lds_read<uint32_t>(ring_fin + (((n_copy - copy_depth) & 7u) << 8)));
      const unsigned begin8 = max(handover8, copy_free8);
      copy_free8 = begin8 + dur8;
      const bool reload = cur_kind == (unsigned)kL;
      lds_write<uint32_t>(ring_fin + ((n_copy & 7u) << 8), copy_free8);
      lds_write<uint32_t>(ring_key + ((n_copy & 7u) << 8), reload ? cur_key : 0xffffffffu);
      ++n_copy;
      free_at8 = handover8;
      pass_time(handover8);
      // its memory event: a reload allocates when it starts, an offload releases when it ends
      const unsigned ev8 = reload ? begin8 : copy_free8;
      lds_write<uint32_t>(ring_ev_time + ((ev_tail & 7u) << 8), ev8);
      lds_write<uint32_t>(ring_ev_units + ((ev_tail & 7u) << 8),
                          reload ? (my_ & 0xffu) : 0u - ((my_ >> 8) & 0xffu));
      next_ev8 = ev_head == ev_tail ? ev8 : next_ev8;
      ++ev_tail;
      unsigned flip;
      asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_1"
          : "=v"(flip) : "v"(bj), "v"(mx_));
      // (a reload marks the activation: bit 3 of its nibble)
      lds_write<uint32_t>(at_state, (sx ^ flip) | (reload ? 8u << (bj & 31u) : 0u));
      decode(w_next);
      npos += 128u;
      w_next = lds_read<uint16_t>((npos & ((kRing - 1) << 7)) | win_off);
    }
    // SLIDE: in front of the item, the oldest stashed W items that end before it starts (the item's start does not
    // move: it is the later of its inputs and the device's free time without any W item, and the W items end
    // before it).  A queue that runs empty while B items wait in the row is read back at the next top-up: the
    // device keeps the time it has reached and does nothing until then.
    // (the later of the device's free time and the inputs; placing W items in front does not change it)
    const unsigned first8 = max(free_at8, ready8);
    if (SLIDE && ok) {
      if (q_head_dur8 <= first8 - free_at8) {
        const unsigned before8 = free_at8;
        do {
          free_at8 += q_head_dur8;
          mem -= q_head_free;
          q_bits >>= kQBits;
          --q_n;
          new_head();
        } while (q_head_dur8 <= first8 - free_at8);
        w_placed8 += free_at8 - before8;
        if (q_over > q_n) dead = kRefillStall;   // empty, and B items wait in the row
      }
    }
    if (ok && !transfer && (!SLIDE || dead == 0u)) {
      unsigned start8 = first8;
      if (COPY && cur_kind == (unsigned)kB && ((sx >> (bj & 31u)) & 8u) != 0u) {
        // the activation was reloaded: if that transfer is among the last copy_depth ones it may still run
        // (all eight places of the ring are looked at, in one round trip: a transfer further back than
        // copy_depth has finished before the device got here, so a match there changes nothing)
        unsigned keys[8], fins[8];
#pragma unroll
        for (unsigned i = 0; i < 8u; ++i) {
          keys[i] = lds_read<uint32_t>(ring_key + (i << 8));
          fins[i] = lds_read<uint32_t>(ring_fin + (i << 8));
        }
#pragma unroll
        for (unsigned i = 0; i < 8u; ++i) start8 = max(start8, keys[i] == cur_key ? fins[i] : 0u);
      }
      const unsigned fin8 = start8 + dur8;
      if (TIMES) {
        // shift bits 8..23 of the start time (its low half in time units) into the 16 bytes
        st0 = __builtin_amdgcn_alignbit(st1, st0, 16);
        st1 = __builtin_amdgcn_alignbit(st2, st1, 16);
        st2 = __builtin_amdgcn_alignbit(st3, st2, 16);
        st3 = __builtin_amdgcn_perm(start8, st3, 0x06050302u);
        // npos = (position of this op + 1) << 7: the eighth op of a group completes it
        if ((npos & (7u << 7)) == 0u)
          *reinterpret_cast<uint4*>(start_row + ((size_t)((npos >> 10) - 1u) << (lpc_shift + 2))) = make_uint4(st0, st1, st2, st3);
        // an op that waited 2^16 time units or more for its inputs cannot be rebuilt from the low half
        const unsigned wait8 = start8 - free_at8;
        if ((wait8 >> 24) != 0u && n_esc < escape_cap - 1)
          esc_row[n_esc++] = (((npos >> 7) - 1u) << 8) | (wait8 >> 24);
      }
      if (COPY) pass_time(start8);
      mem += (int)(my_ & 0xffu);
      pk = max(pk, mem);
      if (COPY) pass_time(fin8);
      mem -= (int)((my_ >> 8) & 0xffu);
      // state ^= (need ^ next) << nibble position; the shift takes the low five bits of bj
      unsigned flip;
      const unsigned nib_at = SYNC ? at_nib : bj;
      asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_1"
          : "=v"(flip) : "v"(nib_at), "v"(mx_));
      lds_write<uint32_t>(at_state, sx ^ flip);
      // LINKS: the value leaves when the link to its consumer's device is free, and keeps it busy for
      // the edge's latency (an op that sends nothing off the device uses the lane's spare link word,
      // which never holds more than an earlier finish time)
      unsigned leave8 = fin8;
      if (LINKS) {
        // (an op without an out-edge writes the dump region and the lane's last link word: never read back
        // by an op whose value counts)
        leave8 = max(fin8, lf1);
        const bool has_out = (mx_ >> 16) != dump_bytes;
        lds_write<uint32_t>(has_out ? at_link1 : spare_at, leave8 + ((out1 >> 16) << 8));
      }
      // finish << 8 | own stage (byte 2 of the last metadata dword; the low byte of fin8 is zero)
      const unsigned val = __builtin_amdgcn_perm(leave8, my_, 0x07060502u);
      // byte offset of the output slot in the high half; ops without an output edge write the
      // candidate's dump region, which nobody reads (LINKS: the lane's last link word instead; that
      // form's tables have no dump region, its offset only marks such ops)
      if (LINKS) lds_write<uint32_t>((mx_ >> 16) != dump_bytes ? bj + (mx_ >> 16) : spare_at, val);
      else lds_write<uint32_t>(bj + (mx_ >> 16), val);
      if (SYNC) {
        // an item of a group is the value of each of its micro-batches
        for (unsigned k = 1; k < n_out; ++k) lds_write<uint32_t>(bj + (mx_ >> 16) + (k << 2), val);
        if (DEG2 && ((unsigned)M2.y & kMetaHasProd))
          for (unsigned k = 1; k < n_out; ++k) lds_write<uint32_t>(bj + ((unsigned)M2.y & 0xffffu) + (k << 2), val);
      }
      if (DEG2) {
        if ((unsigned)M2.y & kMetaHasProd) {
          unsigned val2 = val;
          if (LINKS) {
            // (read after the write above: both edges may use the same link)
            const unsigned at_link2 = link_base + (out2 & 0xffffu);
            const unsigned leave2 = max(fin8, lds_read<uint32_t>(at_link2));
            lds_write<uint32_t>(at_link2, leave2 + ((out2 >> 16) << 8));
            val2 = __builtin_amdgcn_perm(leave2, my_, 0x07060502u);
          }
          lds_write<uint32_t>(bj + ((unsigned)M2.y & 0xffffu), val2);
        }
      }
      free_at8 = fin8;
      busy8 += dur8;
      // (B is the only kind that takes an activation from resident to backward-done)
      if (SLIDE && ((mx_ >> 8) & 0xffu) == (unsigned)(kRes ^ kBDone)) {
        // a B item stashes its W item (once the queue has overflowed, later ones stay in the row)
        if (q_n + (q_over << 6) < kQCap) {
          q_bits |= cur_push << (q_n * kQBits);
          ++q_n;
          new_head();
        } else if (q_over == 0u) {
          q_over = 1u;
          q_refill_at = (int)(npos >> 7) - 1;
        }
      }
      decode(w_next);
      npos += 128u;
      w_next = lds_read<uint16_t>((npos & ((kRing - 1) << 7)) | win_off);
    }
    // A segment none of whose lanes issued is finished, and stays so: nothing it reads changes any
    // more.  It could only be restarted at the next top-up anyway, so only the last round before
    // the top-up looks.  Cheap scalar pre-test: does the issue mask, with the fields of idle
    // segments filled, contain an all-zero field of lpc bits?  (x - lows) & ~x & highs is non-zero
    // iff some field of x is zero.
    // (SLIDE: a device that waits for its queue to be read back is not finished)
    if (SLIDE && sub == kSyncRounds - 1) gathered = __ballot(dead == kRefillStall);
    const unsigned long long x = moved | gathered | idle_fields;
    if (sub == kSyncRounds - 1 && (((x - base_bits) & ~x) & high_bits) != 0ull) {
      // fold the issue mask onto the segments' base bits to find which segments ended
      unsigned long long any_moved = moved | gathered;
#pragma unroll
      for (int i = 0; i < 6; ++i) any_moved |= any_moved >> fold_shift[i];
      const unsigned long long ended = ~any_moved & run_bases;
      const bool seg_ended = ((ended >> (seg << lpc_shift)) & 1ull) != 0ull;
      // ---- the candidate is over: lists exhausted or nothing can move any more
      bool bad_head = false, incomplete = false;
      // the word the lane stopped at is still in its ring (kind 0 if its list is exhausted)
      const unsigned w = lds_read<uint16_t>(((npos - 128u) & ((kRing - 1) << 7)) | win_off);
      if (seg_ended && lane_ok) {
        // a stuck device sits on a malformed word?
        const int4 Mh = lds_read<int4>(__umul24(w >> 11, row_bytes) + meta_off);
        const int n_items = SYNC ? pick<V>(grp, (int)((w >> 11) & (unsigned)(V - 1))) >> 16 : m;
        bad_head = (w >> 13) != 0u && (((unsigned)Mh.z & 15u) == 15u || (int)(w & 0x7ff) >= n_items);
        // every activation of this device consumed?
        for (int i = 0; i < T.state_words; ++i)
          incomplete = incomplete || ((stt[i * 64 + lane] & (COPY ? 0x77777777u : ~0u)) != (unsigned)expect[i]);
        if (COPY) pass_time(0xffffffffu);   // what the copy engine still had to do when the list ended
      }
      // (kind 0 ends a list whatever its low bits are)
      const unsigned long long stuck = __ballot(lane_ok && (w >> 13) != 0u) & seg_mask;
      const unsigned long long stuck_bad = __ballot(bad_head) & seg_mask;
      const unsigned long long unfinished = __ballot(incomplete) & seg_mask;
      const unsigned long long over = __ballot(lane_ok && pk > cap) & seg_mask;
      // (SLIDE: what is still stashed runs back to back behind the list)
      int ms = lane_ok ? (int)((COPY ? max(free_at8, copy_free8) : SLIDE ? free_at8 + (w_total8 - w_placed8) : free_at8) >> 8) : 0;
      for (int off = 1; off < lpc; off <<= 1) ms = max(ms, __shfl_xor(ms, off, 64));
      if (seg_ended) {
        unsigned flg = 0;
        if (stuck) flg = kDeadlock | (stuck_bad ? kIncomplete : 0);
        else if (unfinished) flg = kIncomplete;
        else if (over) flg = kOverCap;
        if (TIMES) {
          if (lane_ok) {
            // the start times of an unfinished group of eight, the end of the escape list, and where
            // the list stopped
            const unsigned stop = (npos >> 7) - 1u;
            if (stop & 7u) {
              for (unsigned i = stop & 7u; i < 8u; ++i) {
                st0 = __builtin_amdgcn_alignbit(st1, st0, 16);
                st1 = __builtin_amdgcn_alignbit(st2, st1, 16);
                st2 = __builtin_amdgcn_alignbit(st3, st2, 16);
                st3 >>= 16;
              }
              *reinterpret_cast<uint4*>(start_row + ((size_t)(stop >> 3) << (lpc_shift + 2))) = make_uint4(st0, st1, st2, st3);
            }
            esc_row[n_esc] = 0xffffffffu;
            out_stop[cand * T.D + d] = (int)stop;
            if (d == 0) out_flags[cand] = (unsigned char)(flg & (kDeadlock | kIncomplete));
          }
        } else if (lane_ok) {
          const bool failed = (flg & (kDeadlock | kIncomplete)) != 0;
          out_idle[cand * T.D + d] = failed ? -1ll : (long long)(ms - (int)((busy8 + (SLIDE ? w_total8 : 0u)) >> 8));
          out_peak[cand * T.D + d] = failed ? -1 : pk * T.unit_scale;
          if (d == 0) {
            out_makespan[cand] = failed ? 0x7fffffffffffffffll : (long long)ms;
            out_flags[cand] = (unsigned char)flg;
          }
        }
        running = false;
        dead = ~0u;
        fresh = true;
      }
      // the finished segments stop counting as running at once
      const unsigned long long run_lanes = __ballot(running && !priming);
      run_bases = run_lanes & base_bits;
      idle_fields = ~run_lanes;
      any_special = true;
    }
    }  // sub-rounds
  }
}

#define FPSCHED_INSTANTIATE_MODE(V, G, O, MODE)                                                           \
  template __global__ void eval_slot_kernel<V, G, O, MODE>(                                               \
      SlotTables, const uint16_t*, long long, int, long long*, long long*, int*, unsigned char*,          \
      unsigned long long*, int, uint32_t*, int32_t*, const int32_t*, uint32_t*, int);
#define FPSCHED_INSTANTIATE(V, G, O)               \
  FPSCHED_INSTANTIATE_MODE(V, G, O, kSlotPlain)    \
  FPSCHED_INSTANTIATE_MODE(V, G, O, kSlotTimes)    \
  FPSCHED_INSTANTIATE_MODE(V, G, O, kSlotPerMicrobatch) \
  FPSCHED_INSTANTIATE_MODE(V, G, O, kSlotPerMicrobatchLds) \
  FPSCHED_INSTANTIATE_MODE(V, G, O, kSlotLinks)            \
  FPSCHED_INSTANTIATE_MODE(V, G, O, kSlotTimesLinks)       \
  FPSCHED_INSTANTIATE_MODE(V, G, O, kSlotPerMicrobatchLdsLinks) \
  FPSCHED_INSTANTIATE_MODE(V, G, O, kSlotCopy) \
  FPSCHED_INSTANTIATE_MODE(V, G, O, kSlotSync) \
  FPSCHED_INSTANTIATE_MODE(V, G, O, kSlotSlide) \
  FPSCHED_INSTANTIATE_MODE(V, G, O, kSlotSlideLinks)
FPSCHED_INSTANTIATE(1, false, true)
FPSCHED_INSTANTIATE(2, false, true)
FPSCHED_INSTANTIATE(4, false, true)
FPSCHED_INSTANTIATE(1, false, false)
FPSCHED_INSTANTIATE(2, false, false)
FPSCHED_INSTANTIATE(4, false, false)
FPSCHED_INSTANTIATE(1, true, false)
FPSCHED_INSTANTIATE(2, true, false)
FPSCHED_INSTANTIATE(4, true, false)
#undef FPSCHED_INSTANTIATE
#undef FPSCHED_INSTANTIATE_MODE

}  // namespace fpsched

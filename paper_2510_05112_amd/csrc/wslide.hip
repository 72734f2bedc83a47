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
// (kind, chunk, device)); the control flow is plain: candidates are assigned statically, a round is
// a loop body with branches, op words come from global memory in 8-byte pieces fetched one piece
// ahead, and the new rows are collected 16 words at a time in LDS and stored 32 bytes at a time.
//
// The stash needs no storage: it is the B words of the device's own list between a second cursor
// and the first one (every B word before the second cursor has had its W item issued).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

namespace fpsched {

namespace {

// 4 op words in one 64-bit register, refilled from an 8-byte aligned row one piece ahead
struct WordReader {
  const uint16_t* row;
  int stride;
  unsigned long long cur, next;
  __device__ __forceinline__ unsigned long long piece(int at) const {
    return at < stride ? *reinterpret_cast<const unsigned long long*>(row + at) : 0ull;
  }
  __device__ __forceinline__ void start(const uint16_t* r, int s) {
    row = r; stride = s;
    cur = piece(0);
    next = piece(4);
  }
  // word at position i (i only ever moves forward by one, starting at 0)
  __device__ __forceinline__ unsigned at(int i) const { return (unsigned)(cur >> ((i & 3) * 16)) & 0xffffu; }
  // call after moving on to position i
  __device__ __forceinline__ void moved_to(int i) {
    if ((i & 3) == 0) {
      cur = next;
      next = piece(i + 4);
    }
  }
};

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
  // 8 staging dwords [dword][lane]]
  for (int i = tid; i < T.n_shared_ints; i += blockDim.x) lds[i] = T.ints[i];
  const int wave_ints = T.state_words * 64 + cpw * T.slots_per_cand + 8 * 64;
  uint32_t* stt = reinterpret_cast<uint32_t*>(lds + T.n_shared_ints + wave * wave_ints);
  uint32_t* slots = stt + T.state_words * 64;
  uint32_t* staging = slots + cpw * T.slots_per_cand + lane;   // dword i at + i * 64
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
  const int cap = dev[1];
  int in_f[V], in_b[V], in_f2[V], in_b2[V];   // first slot of each chunk's inputs, per direction
#pragma unroll
  for (int c = 0; c < V; ++c) {
    in_f[c] = dev[2 + c];
    in_b[c] = dev[2 + V + c];
    in_f2[c] = DEG2 ? dev[2 + 2 * V + c] : 0;
    in_b2[c] = DEG2 ? dev[2 + 3 * V + c] : 0;
  }
  const int words_per_chunk = (m + 7) >> 3;

  const size_t row_index = (size_t)(active ? cand : 0) * T.D + dd;
  WordReader list, scan;   // the list cursor and the stash cursor read the same row
  list.start(ops + row_index * (size_t)stride, active ? stride : 0);
  scan = list;
  uint16_t* out_row = ops_out + row_index * (size_t)stride_out;
  int cursor = 0, wcur = 0, out_len = 0;
  unsigned free_at8 = 0, busy8 = 0;
  int mem = 0, pk = 0;
  bool done = !active, halted = false, seg_live = true;

  // Is the item of `word` (kind in its top three bits) allowed to issue, and when are its inputs
  // there?  0 = yes (ready8 set), 1 = not yet, 2 = never (malformed word).
  auto check = [&](unsigned word, int4& M, int2& M2, unsigned& ready8) -> int {
    const unsigned j = word & 0x7ffu, c5 = word >> 11, c = c5 & 3u, kind = word >> 13;
    M = meta[c5 * lpc + d];
    if (j >= (unsigned)m || ((unsigned)M.z & 15u) == 15u) return 2;
    const unsigned sx = stt[(c * words_per_chunk + (j >> 3)) * 64 + lane];
    if (((sx >> ((j & 7u) * 4u)) & 15u) != ((unsigned)M.z & 15u)) return 1;
    const bool is_b = kind == (unsigned)kB, has_edges = is_b || kind == (unsigned)kF || kind == (unsigned)kFD;
    ready8 = 0u;
    if ((unsigned)M.w >> 24) {
      int base = in_f[0];
#pragma unroll
      for (int i = 0; i < V; ++i) base = ((int)c == i) ? (is_b ? in_b[i] : in_f[i]) : base;
      const unsigned r = my_slots[base + j] + (unsigned)M.y;
      if (r & 0xffu) return 1;   // the slot does not carry the upstream stage's tag yet
      ready8 = r;
    }
    M2 = make_int2(0, 0);
    if (DEG2 && has_edges) {
      M2 = meta2[((is_b ? 4u : 0u) + c) * lpc + d];
      if ((unsigned)M2.y & kMetaHasCons) {
        int base = in_f2[0];
#pragma unroll
        for (int i = 0; i < V; ++i) base = ((int)c == i) ? (is_b ? in_b2[i] : in_f2[i]) : base;
        const unsigned r = my_slots[base + j] + (unsigned)M2.x;
        if (r & 0xffu) return 1;
        ready8 = max(ready8, r);
      }
    }
    return 0;
  };
  // The item issues at start8: the word joins the new row (false: the row is full), the device's
  // clock, memory and the activation state move on, the finish time goes to the output slots.
  auto issue = [&](unsigned word, const int4& M, const int2& M2, unsigned start8) -> bool {
    if (out_len >= stride_out) return false;
    reinterpret_cast<uint16_t*>(staging + ((out_len >> 1) & 7) * 64)[out_len & 1] = (uint16_t)word;
    if ((out_len & 15) == 15) {
      uint4* dst = reinterpret_cast<uint4*>(out_row + (out_len - 15));
      dst[0] = make_uint4(staging[0], staging[64], staging[128], staging[192]);
      dst[1] = make_uint4(staging[256], staging[320], staging[384], staging[448]);
    }
    ++out_len;
    const unsigned j = word & 0x7ffu, c = (word >> 11) & 3u;
    const unsigned fin8 = start8 + (unsigned)M.x;
    mem += (int)((unsigned)M.w & 0xffu);
    pk = max(pk, mem);
    mem -= (int)(((unsigned)M.w >> 8) & 0xffu);
    stt[(c * words_per_chunk + (j >> 3)) * 64 + lane] ^= (((unsigned)M.z >> 8) & 0xffu) << ((j & 7u) * 4u);
    const unsigned val = fin8 | (((unsigned)M.w >> 16) & 0xffu);
    my_slots[j + ((unsigned)M.z >> 18)] = val;   // an item without an output edge writes the dump region
    if (DEG2 && ((unsigned)M2.y & kMetaHasProd)) my_slots[j + (((unsigned)M2.y & 0xffffu) >> 2)] = val;
    free_at8 = fin8;
    busy8 += (unsigned)M.x;
    return true;
  };
  // The oldest stashed item: the B word at the stash cursor, as a W word.  It issues at the time the
  // device is free if it ends by limit8 (false: it does not fit, or the row is full -> halted).
  auto run_stashed = [&](unsigned limit8) -> bool {
    const unsigned w_word = (scan.at(wcur) & 0x1fffu) | ((unsigned)kW << 13);
    int4 M;
    int2 M2;
    unsigned unused;
    if (check(w_word, M, M2, unused) != 0) { halted = true; return false; }   // cannot happen: its B has issued
    if (free_at8 + (unsigned)M.x > limit8) return false;
    if (!issue(w_word, M, M2, free_at8)) { halted = true; return false; }
    // on to the next B word in front of the list cursor
    do {
      ++wcur;
      scan.moved_to(wcur);
    } while (wcur < cursor && (scan.at(wcur) >> 13) != (unsigned)kB);
    return true;
  };

  // every round but the last of a candidate consumes a word of the list or issues an item
  // (or is the one in which a device finds the end of its list)
  const long long max_rounds = (long long)T.D * ((long long)stride + stride_out + 1) + 8;
  for (long long round = 0; round < max_rounds; ++round) {
    bool progressed = false;
    if (!done && !halted && seg_live) {
      const unsigned w = cursor < stride ? list.at(cursor) : 0u;
      const unsigned kind = w >> 13;
      if (kind == (unsigned)kEnd) {
        while (wcur < cursor && run_stashed(0xffffffffu)) {}
        done = !halted;
        progressed = true;
      } else {
        int4 M;
        int2 M2;
        unsigned ready8 = 0u;
        const int verdict = check(w, M, M2, ready8);
        bool consumed = false;
        if (verdict == 2) {
          halted = true;
        } else if (kind == (unsigned)kW) {
          consumed = true;   // where the input put its W items is not used
        } else if (verdict == 0) {
          const unsigned start8 = max(free_at8, ready8);
          while (wcur < cursor && run_stashed(start8)) {}
          if (!halted) {
            if (issue(w, M, M2, start8)) consumed = true; else halted = true;
          }
          progressed = true;
        }
        if (consumed) {
          // the stash cursor follows the list cursor unless it rests on a B word whose W item is due
          if (wcur == cursor && kind != (unsigned)kB) {
            ++wcur;
            scan.moved_to(wcur);
          }
          ++cursor;
          list.moved_to(cursor);
          progressed = true;
        }
      }
    }
    __builtin_amdgcn_wave_barrier();
    const unsigned long long moved = __ballot(progressed);
    if ((moved & seg_mask) == 0ull) seg_live = false;
    if (moved == 0ull) break;
  }

  // ---- the rest of the new row: staged words, then END words up to the stride
  if (active) {
    int at = out_len & ~15;
    if (out_len & 15) {
      for (int i = out_len & 15; i < 16; ++i) reinterpret_cast<uint16_t*>(staging + (i >> 1) * 64)[i & 1] = 0;
      if (at < stride_out)
        *reinterpret_cast<uint4*>(out_row + at) = make_uint4(staging[0], staging[64], staging[128], staging[192]);
      if (at + 8 < stride_out)
        *reinterpret_cast<uint4*>(out_row + at + 8) = make_uint4(staging[256], staging[320], staging[384], staging[448]);
      at += 16;
    }
    for (; at < stride_out; at += 8) *reinterpret_cast<uint4*>(out_row + at) = make_uint4(0u, 0u, 0u, 0u);
  }
  // ---- the evaluation of the new lists
  bool incomplete = false;
  if (active)
    for (int i = 0; i < T.state_words; ++i) incomplete = incomplete || (stt[i * 64 + lane] != (unsigned)expect[i]);
  const unsigned long long stuck = __ballot(active && !done) & seg_mask;
  const unsigned long long stuck_bad = __ballot(active && halted) & seg_mask;
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

// General evaluation kernel: any per-device op order, any stage DAG.
//
// One wavefront owns `cands_per_wave` candidates; inside a candidate, lane = device
// (lanes_per_cand is the device count rounded up to a power of two).  Each lane
// walks its device's op list with a cursor held in registers.  The finish times
// of forward and backward ops, indexed by (stage, micro-batch), and the
// activation state of every (stage, micro-batch) live in LDS; a lane whose next
// op cannot issue yet (input not evaluated, wrong activation state) simply waits
// for a later round.  A round in which no lane of a candidate moves ends that
// candidate: either every list is exhausted or the rest is deadlocked.
//
// Start rule (paper Section 5.1 "Data dependency"; estimator sketch after Section
// 6): start = max(device free, finish of each cross-stage input + latency if the
// input ran on another device); finish = start + dur[kind][stage].
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

namespace fpsched {

__global__ __launch_bounds__(64) void eval_general_kernel(
    DevTables T, const uint16_t* __restrict__ ops, long long n_cand, int stride,
    long long* __restrict__ out_makespan, long long* __restrict__ out_idle,
    int* __restrict__ out_peak, unsigned char* __restrict__ out_flags, const int32_t* __restrict__ dur_mb) {
  extern __shared__ int32_t lds[];
  const int lane = threadIdx.x;
  const int S = T.S, m = T.m, SM = S * m;
  const int per_cand_ints = 2 * SM + ((SM + 3) >> 2);
  const int cpw = T.cands_per_wave;
  const int lpc = T.lanes_per_cand;
  const int lpc_shift = __ffs(lpc) - 1;

  // stage the shared tables, clear the per-candidate tables
  for (int i = lane; i < T.n_table_ints; i += 64) lds[i] = T.ints[i];
  int32_t* cand_base = lds + T.n_table_ints;
  for (int c = 0; c < cpw; ++c) {
    int32_t* p = cand_base + c * per_cand_ints;
    for (int i = lane; i < 2 * SM; i += 64) p[i] = -1;
    for (int i = 2 * SM + lane; i < per_cand_ints; i += 64) p[i] = 0;
  }
  __syncthreads();

  const int32_t* tab = lds;
  const int seg = lane >> lpc_shift;
  const int d = lane & (lpc - 1);
  const long long cand = (long long)blockIdx.x * cpw + seg;
  const bool active = (seg < cpw) && (d < T.D) && (cand < n_cand);
  int32_t* fin_fwd = cand_base + (seg < cpw ? seg : 0) * per_cand_ints;
  int32_t* fin_bwd = fin_fwd + SM;
  unsigned char* state = reinterpret_cast<unsigned char*>(fin_fwd + 2 * SM);

  const int dd = active ? d : 0;
  const int nch = tab[T.off_n_chunks + dd];
  const int cap = tab[T.off_mem_cap + dd];
  const uint16_t* row = ops + ((size_t)(active ? cand : 0) * T.D + dd) * (size_t)stride;
  const unsigned long long seg_mask =
      (lpc == 64 ? ~0ull : ((1ull << lpc) - 1ull)) << (seg * lpc);
  const unsigned free_mask = (1u << kFD) | (1u << kO) | (T.has_w ? (1u << kW) : (1u << kB));
  const int terminal_kind = T.has_w ? kW : kB;

  int cursor = 0, free_at = 0, busy = 0, mem = 0, pk = 0, n_term = 0;
  bool done = !active, bad = false, seg_live = true;
  unsigned w = (active && stride > 0) ? row[0] : 0u;

  for (;;) {
    bool progressed = false;
    if (!done && seg_live) {
      const int kind = w >> 13;
      if (kind == kEnd) {
        done = true;
        progressed = true;
      } else {
        const int c = (w >> 11) & 3, j = w & 0x7ff;
        if (c >= nch || j >= m || (kind == kW && !T.has_w)) {
          bad = true;
        } else {
          const int s = tab[T.off_local_stage + d * kMaxChunks + c];
          const int idx = s * m + j;
          const int st = state[idx];
          const int need = (0x03124100u >> (4 * kind)) & 0xf;
          if (st == need) {
            int ready = 0;
            bool blocked = false;
            if (kind == kF || kind == kFD) {
              const int e1 = tab[T.off_pred_off + s + 1];
              for (int e = tab[T.off_pred_off + s]; e < e1; ++e) {
                const int t = fin_fwd[tab[T.off_pred_stage + e] * m + j];
                if (t < 0) blocked = true;
                ready = max(ready, t + tab[T.off_pred_comm + e]);
              }
            } else if (kind == kB) {
              const int e1 = tab[T.off_succ_off + s + 1];
              for (int e = tab[T.off_succ_off + s]; e < e1; ++e) {
                const int t = fin_bwd[tab[T.off_succ_stage + e] * m + j];
                if (t < 0) blocked = true;
                ready = max(ready, t + tab[T.off_succ_comm + e]);
              }
            }
            if (!blocked) {
              const int dt = dur_mb ? dur_mb[(kind * S + s) * m + j] : tab[T.off_dur + kind * S + s];
              const int u = tab[T.off_mem_units + s];
              const int fin = max(free_at, ready) + dt;
              if ((0xD2u >> kind) & 1u) {  // F, R, L, FD allocate at their start
                mem += u;
                pk = max(pk, mem);
              }
              if ((free_mask >> kind) & 1u) mem -= u;
              state[idx] = (unsigned char)((0x21315410u >> (4 * kind)) & 0xf);
              if (kind == kF || kind == kFD) fin_fwd[idx] = fin;
              else if (kind == kB) fin_bwd[idx] = fin;
              n_term += (kind == terminal_kind);
              free_at = fin;
              busy += dt;
              ++cursor;
              w = (cursor < stride) ? row[cursor] : 0u;
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

  // per-candidate reductions over the candidate's lanes
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

}  // namespace fpsched

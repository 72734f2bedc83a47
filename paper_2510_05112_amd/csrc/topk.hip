// Top-k under the memory cap: the k feasible candidates (flags == 0) with the
// smallest (makespan, index), ascending (paper Section 7.1: the tuner keeps the
// schedules whose bubble ratio is lowest; with fixed total work that is the
// least makespan).
//
// Tile sort + tree merge, all in LDS: every workgroup loads one tile of
// kTile (makespan, index) keys (infeasible candidates become +inf keys), sorts it
// with a bitonic network and writes its k smallest keys; the next level treats
// those survivors as its input, until one tile is left.  The result is a pure
// function of the keys, so it does not depend on workgroup scheduling, and ties
// on makespan are broken by the candidate index because the index is part of
// the key.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

namespace fpsched {

constexpr long long kInf = 0x7fffffffffffffffll;

__device__ __forceinline__ bool key_less(const Key& a, const Key& b) {
  return a.makespan < b.makespan || (a.makespan == b.makespan && a.idx < b.idx);
}

// level 0 reads (makespan, flags); later levels read Key arrays.
// Output: per tile, k keys (ascending).  When `final_out` is set (single tile),
// the keys are unpacked into idx / makespan / count instead.
__global__ __launch_bounds__(kTopkThreads) void topk_tile_kernel(
    const long long* __restrict__ in_makespan, const unsigned char* __restrict__ in_flags,
    const Key* __restrict__ in_keys, long long n, int k, Key* __restrict__ out_keys,
    long long* __restrict__ final_idx, long long* __restrict__ final_makespan,
    int* __restrict__ final_count) {
  __shared__ Key tile[kTile];
  const long long base = (long long)blockIdx.x * kTile;
  for (int i = threadIdx.x; i < kTile; i += kTopkThreads) {
    const long long g = base + i;
    Key key{kInf, kInf};
    if (g < n) {
      if (in_keys) {
        key = in_keys[g];
      } else if (in_flags[g] == 0) {
        key.makespan = in_makespan[g];
        key.idx = g;
      }
    }
    tile[i] = key;
  }
  __syncthreads();
  for (int size = 2; size <= kTile; size <<= 1) {
    for (int strd = size >> 1; strd > 0; strd >>= 1) {
      for (int t = threadIdx.x; t < kTile / 2; t += kTopkThreads) {
        const int lo = ((t / strd) * (strd << 1)) + (t % strd);
        const int hi = lo + strd;
        const bool ascending = ((lo & size) == 0);
        const Key a = tile[lo], b = tile[hi];
        if (key_less(b, a) == ascending) {
          tile[lo] = b;
          tile[hi] = a;
        }
      }
      __syncthreads();
    }
  }
  if (final_idx) {
    for (int i = threadIdx.x; i < k; i += kTopkThreads) {
      const Key key = tile[i];
      const bool real = key.idx != kInf;
      final_idx[i] = real ? key.idx : -1ll;
      final_makespan[i] = real ? key.makespan : kInf;
    }
    if (threadIdx.x == 0) {
      // keys are sorted, the real ones come first: binary search the boundary within [0, k]
      int lo = 0, hi = k;
      while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (tile[mid].idx != kInf) lo = mid + 1; else hi = mid;
      }
      *final_count = lo;
    }
  } else {
    Key* dst = out_keys + (long long)blockIdx.x * k;
    for (int i = threadIdx.x; i < k; i += kTopkThreads) dst[i] = tile[i];
  }
}

// Ranking keys of evaluated candidates (one thread per candidate): the quantities the tuner can
// rank by besides the makespan -- the largest peak memory over the devices and the summed bubble
// time (Section 7.1: bubble ratio; Section 2: memory footprint as the second axis of a schedule).
// Two-part keys are packed primary << 32 | secondary (both below 2^31), so that the top-k kernel,
// which orders by (key, index), orders lexicographically.
__global__ void rank_keys_kernel(const long long* makespan, const long long* idle, const int* peak,
                                 const unsigned char* flags, long long n, int D, int mode, int include_over_cap,
                                 long long* key_out, unsigned char* excluded_out) {
  const long long c = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= n) return;
  const unsigned fl = flags[c];
  const bool out = (fl & (kDeadlock | kIncomplete)) != 0 || (!include_over_cap && (fl & kOverCap) != 0);
  long long key = 0;
  if (!out) {
    int max_peak = 0;
    long long sum_idle = 0;
    for (int d = 0; d < D; ++d) {
      max_peak = max(max_peak, peak[c * D + d]);
      sum_idle += idle[c * D + d];
    }
    const long long ms = makespan[c];
    key = mode == 0 ? ms : (mode == 1 ? ((ms << 32) | (long long)max_peak)
                                      : (mode == 2 ? (((long long)max_peak << 32) | ms) : sum_idle));
  }
  key_out[c] = key;
  excluded_out[c] = out ? 1 : 0;
}

}  // namespace fpsched

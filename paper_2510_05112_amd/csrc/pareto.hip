// Pareto front of (makespan, largest peak[d]) over the candidates that completed, and the
// OVER_CAP flag recomputed for other caps.  A schedule has two properties in the paper, its bubble
// ratio (Section 7.1) and its memory footprint (Section 2); the front is every trade-off between
// the two that no other candidate beats, instead of one cut at a fixed cap.
//
// Two kernels.  pareto_tile_kernel: one workgroup per tile of kTile candidates sorts the tile by
// (makespan, peak, index) in LDS, takes the running minimum of the peaks along the sorted order
// and keeps the entries whose peak is below every peak before them: the tile's own front, by
// ascending makespan and strictly descending peak, written compacted.  pareto_merge_kernel: one
// workgroup walks all tile fronts at once, a cursor per tile.  The next point of the global front
// is the smallest (makespan, peak, index) among the entries whose peak is below the peak of the
// point found before; since peaks descend along a tile front, the entries a cursor skips can
// never qualify again, so every cursor only moves forward.  Both steps are pure functions of the
// values, independent of workgroup scheduling.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

namespace fpsched {

namespace {

constexpr long long kInf = 0x7fffffffffffffffll;
constexpr int kNoPeak = 0x7fffffff;

struct FrontKey {
  long long makespan;
  int peak;
  int local;   // index within the tile; kTile marks a slot without a candidate
};

__device__ __forceinline__ bool front_less(const FrontKey& a, const FrontKey& b) {
  if (a.makespan != b.makespan) return a.makespan < b.makespan;
  if (a.peak != b.peak) return a.peak < b.peak;
  return a.local < b.local;
}

// Exclusive scan over the kTopkThreads per-thread values in `buf` (min or sum); returns this
// thread's prefix, *total = the reduction over all threads.
template <bool MIN>
__device__ __forceinline__ int block_exclusive_scan(int* buf, int mine, int identity, int* total) {
  const int t = threadIdx.x;
  buf[t] = mine;
  __syncthreads();
  for (int step = 1; step < kTopkThreads; step <<= 1) {
    const int other = t >= step ? buf[t - step] : identity;
    __syncthreads();
    buf[t] = MIN ? min(buf[t], other) : buf[t] + other;
    __syncthreads();
  }
  const int prefix = t > 0 ? buf[t - 1] : identity;
  *total = buf[kTopkThreads - 1];
  __syncthreads();
  return prefix;
}

}  // namespace

__global__ __launch_bounds__(kTopkThreads) void pareto_tile_kernel(
    const long long* __restrict__ makespan, const int* __restrict__ peak, const unsigned char* __restrict__ flags,
    long long n, int D, Key* __restrict__ front_keys, int* __restrict__ front_peak, int* __restrict__ tile_count) {
  __shared__ FrontKey tile[kTile];
  __shared__ int scan_buf[kTopkThreads];
  const long long base = (long long)blockIdx.x * kTile;
  for (int i = threadIdx.x; i < kTile; i += kTopkThreads) {
    const long long g = base + i;
    FrontKey key{kInf, kNoPeak, kTile};
    if (g < n && (flags[g] & (kDeadlock | kIncomplete)) == 0) {
      int mp = 0;
      for (int d = 0; d < D; ++d) mp = max(mp, peak[g * D + d]);
      key = FrontKey{makespan[g], mp, i};
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
        const FrontKey a = tile[lo], b = tile[hi];
        if (front_less(b, a) == ascending) {
          tile[lo] = b;
          tile[hi] = a;
        }
      }
      __syncthreads();
    }
  }
  // every thread owns kTile / kTopkThreads consecutive entries of the sorted tile
  constexpr int kPer = kTile / kTopkThreads;
  const int first = threadIdx.x * kPer;
  int my_min = kNoPeak;
  for (int i = 0; i < kPer; ++i) my_min = min(my_min, tile[first + i].peak);   // empty slots hold kNoPeak
  int unused;
  int running = block_exclusive_scan<true>(scan_buf, my_min, kNoPeak, &unused);
  unsigned keep = 0;
  for (int i = 0; i < kPer; ++i) {
    const FrontKey e = tile[first + i];
    // the first entry of a tile that holds any candidate is always on its front
    if (e.local < kTile && (e.peak < running || first + i == 0)) {
      keep |= 1u << i;
      running = e.peak;
    }
  }
  int total;
  int at = block_exclusive_scan<false>(scan_buf, __popc(keep), 0, &total);
  for (int i = 0; i < kPer; ++i) {
    if (keep >> i & 1) {
      const FrontKey e = tile[first + i];
      front_keys[base + at] = Key{e.makespan, base + e.local};
      front_peak[base + at] = e.peak;
      ++at;
    }
  }
  if (threadIdx.x == 0) tile_count[blockIdx.x] = total;
}

__global__ __launch_bounds__(kParetoMergeThreads) void pareto_merge_kernel(
    const Key* __restrict__ front_keys, const int* __restrict__ front_peak, const int* __restrict__ tile_count,
    int tiles, int kmax, long long* __restrict__ out_idx, long long* __restrict__ out_makespan,
    int* __restrict__ out_peak, int* __restrict__ out_count) {
  __shared__ int cursor[kParetoMaxTiles];
  constexpr int kWaves = kParetoMergeThreads / 64;
  __shared__ long long wave_ms[2][kWaves];
  __shared__ long long wave_idx[2][kWaves];
  __shared__ int wave_peak[2][kWaves];
  for (int t = threadIdx.x; t < tiles; t += kParetoMergeThreads) cursor[t] = 0;   // read back by the same thread only
  long long below = kInf;   // the next point needs a peak smaller than this
  int written = 0;
  while (written < kmax) {
    long long b_ms = kInf, b_idx = kInf;
    int b_peak = kNoPeak;
    for (int t = threadIdx.x; t < tiles; t += kParetoMergeThreads) {   // each tile has one owner thread
      const long long base = (long long)t * kTile;
      int cur = cursor[t];
      const int cnt = tile_count[t];
      while (cur < cnt && front_peak[base + cur] >= below) ++cur;
      cursor[t] = cur;
      if (cur < cnt) {
        const Key k = front_keys[base + cur];
        const int pk = front_peak[base + cur];
        if (k.makespan < b_ms || (k.makespan == b_ms && (pk < b_peak || (pk == b_peak && k.idx < b_idx)))) {
          b_ms = k.makespan; b_peak = pk; b_idx = k.idx;
        }
      }
    }
    for (int off = 32; off > 0; off >>= 1) {
      const long long o_ms = __shfl_xor(b_ms, off), o_idx = __shfl_xor(b_idx, off);
      const int o_peak = __shfl_xor(b_peak, off);
      if (o_ms < b_ms || (o_ms == b_ms && (o_peak < b_peak || (o_peak == b_peak && o_idx < b_idx)))) {
        b_ms = o_ms; b_peak = o_peak; b_idx = o_idx;
      }
    }
    const int buf = written & 1;
    if ((threadIdx.x & 63) == 0) {
      wave_ms[buf][threadIdx.x >> 6] = b_ms;
      wave_idx[buf][threadIdx.x >> 6] = b_idx;
      wave_peak[buf][threadIdx.x >> 6] = b_peak;
    }
    __syncthreads();
    for (int w = 0; w < kWaves; ++w) {
      const long long o_ms = wave_ms[buf][w], o_idx = wave_idx[buf][w];
      const int o_peak = wave_peak[buf][w];
      if (o_ms < b_ms || (o_ms == b_ms && (o_peak < b_peak || (o_peak == b_peak && o_idx < b_idx)))) {
        b_ms = o_ms; b_peak = o_peak; b_idx = o_idx;
      }
    }
    if (b_idx == kInf) break;   // the same value in every thread: no entry is left
    if (threadIdx.x == 0) {
      out_idx[written] = b_idx;
      out_makespan[written] = b_ms;
      out_peak[written] = b_peak;
    }
    below = b_peak;
    ++written;
  }
  for (int i = written + threadIdx.x; i < kmax; i += kParetoMergeThreads) {
    out_idx[i] = -1;
    out_makespan[i] = kInf;
    out_peak[i] = -1;
  }
  if (threadIdx.x == 0) *out_count = written;
}

__global__ void apply_caps_kernel(const int* __restrict__ peak, const int* __restrict__ caps, int per_candidate,
                                  long long n, int D, unsigned char* __restrict__ flags) {
  const long long c = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= n) return;
  const unsigned fl = flags[c];
  bool over = false;
  for (int d = 0; d < D; ++d) over |= peak[c * D + d] > caps[per_candidate ? c * D + d : d];
  over &= (fl & (kDeadlock | kIncomplete)) == 0;
  flags[c] = (unsigned char)((fl & ~(unsigned)kOverCap) | (over ? kOverCap : 0));
}

}  // namespace fpsched

// Kernel declarations shared by the translation units of libfpsched.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "device_tables.h"

namespace fpsched {

struct Key {
  long long makespan;
  long long idx;
};
constexpr int kTile = 2048;
constexpr int kTopkThreads = 1024;

// dur_mb: nullptr, or costs per micro-batch [kinds][S][m] in device memory that replace the table's.
__global__ void eval_general_kernel(DevTables T, const uint16_t* ops, long long n_cand, int stride,
                                    long long* out_makespan, long long* out_idle, int* out_peak,
                                    unsigned char* out_flags, const int32_t* dur_mb);

// Synchronisation stages and dependency pairs (eval_sync.hip): the table form of the evaluator with one
// dependency list per (kind, stage) and items that stand for groups of micro-batches.
// COPY: offload and reload items run on a copy engine beside the computation (T.copy_depth transfers at
// most in the engine); needs 1536 more dwords of LDS per workgroup and one more table per candidate.
template <bool COPY>
__global__ void eval_sync_kernel(SyncTables T, const uint16_t* ops, long long n_cand, int stride,
                                 long long* out_makespan, long long* out_idle, int* out_peak,
                                 unsigned char* out_flags);

constexpr int kSlotMaxWaves = 16;
constexpr int kSlotMaxThreads = 64 * kSlotMaxWaves;

// V = compile-time bound on the stages (chunks) per device: 1, 2 or 4.  DEG2 = some stage
// has two inputs or two outputs in the stage DAG.  ONE_CLASS = the DAG is a single chain.
// next_candidate: a counter in device memory, preset to the number of segments in the grid, from
// which wavefronts draw their work, draw_block candidates per atomic (1 <= draw_block <= 64).
// MODE kSlotTimes: first pass of the weight-gradient sliding; writes out_start8 [n_cand][stride / 8][lanes per
// candidate][8 x 16 bits] (low half of the start time of the op at each position), out_escape [n_cand][D][escape_cap]
// (position << 8 | wait >> 16 of the ops that waited 2^16 time units or more, ended by an all-ones word), out_stop
// [n_cand][D] (words issued per device) and out_flags (DEADLOCK / INCOMPLETE only) instead of makespan, idle and peak;
// needs 16 bytes of LDS more.
// MODE kSlotPerMicrobatch: durations from mb_rows [32][lanes per candidate][m] (cost << 8 per metadata
// row, device and micro-batch) instead of the metadata rows.  MODE kSlotPerMicrobatchLds: from the
// sixteen-bit table at T.off_mb, which travels to LDS with the metadata.
// MODE kSlotLinks: every ordered pair of devices is a link that carries one value at a time; a
// producer holds its value back until its link is free (T.link_words, the longer dev rows).
// MODE kSlotTimesLinks: the timing pass of the sliding under the link model (both of the above).
// MODE kSlotPerMicrobatchLdsLinks: costs per micro-batch from LDS and link occupancy together.
// MODE kSlotCopy: offload and reload items run on a copy engine beside the computation (T.copy_depth transfers
// at most in the engine; T.link_words = 32 dwords per lane behind its state words: the finish times and keys of
// the last eight transfers, and a ring of eight pending memory events).
// MODE kSlotSync: synchronisation stages (one item per group of micro-batches) and dependency pairs of the
// forms the mail slots can carry (forward to forward, backward to backward); the dev rows then have V more ints:
// per chunk the micro-batches per item | items << 16.
// MODE kSlotSlide: the weight-gradient sliding pass without its lists: the results of the lists the two-pass form
// would write, in one kernel (tables as for kSlotTimes plus the W items' costs at T.off_w; 16 bytes of LDS more).
constexpr int kSlotPlain = 0, kSlotTimes = 1, kSlotPerMicrobatch = 2, kSlotPerMicrobatchLds = 3, kSlotLinks = 4,
              kSlotTimesLinks = 5, kSlotPerMicrobatchLdsLinks = 6, kSlotCopy = 7, kSlotSync = 8, kSlotSlide = 9,
              kSlotSlideLinks = 10;   // kSlotSlide under the link model
constexpr int kSlotCopyWords = 32;
template <int V, bool DEG2, bool ONE_CLASS, int MODE>
__global__ void eval_slot_kernel(SlotTables T, const uint16_t* ops, long long n_cand, int stride,
                                 long long* out_makespan, long long* out_idle, int* out_peak,
                                 unsigned char* out_flags, unsigned long long* next_candidate, int draw_block,
                                 uint32_t* out_start8, int32_t* out_stop, const int32_t* mb_rows,
                                 uint32_t* out_escape, int escape_cap);

__global__ void reset_counter_kernel(unsigned long long* counter, unsigned long long value);

// V as above; DEG = bound on the in- and out-degree of a stage (1, 2, or 0 = any).  One wavefront per
// workgroup, 64 / lanes_per_cand parameter sets per wavefront at a time; next_set: a counter in
// device memory, preset to the number of segments in the grid, from which segments draw their sets.
// select: null, or which of the n_src parameter sets each output row takes (outside 0 .. n_src - 1: none).
// TIMED (DEG 1 or 2 only): the schedules are timed as they are generated and only the results R are
// written (ops and select unused); workgroups of up to kGenTimedThreads threads.
struct GenResults {
  long long* makespan;
  long long* idle;
  int32_t* peak;
  unsigned char* flags;
};
constexpr int kGenTimedThreads = 512;
// FORM: kGenPlain writes the lists; kGenTimed times them instead (above); kGenSlide times them after the
// weight-gradient sliding pass (T.gen_spill_words dwords of LDS more per lane)
constexpr int kGenPlain = 0, kGenTimed = 1, kGenSlide = 2;
template <int V, int DEG, int FORM>
__global__ void generate_kernel(DevTables T, const int32_t* policy, const int32_t* inflight, const long long* select,
                                long long n_src, long long n_sets, int stride, uint16_t* ops, int32_t* out_steps,
                                unsigned char* out_status, unsigned long long* next_set, GenResults R);

__global__ void topk_tile_kernel(const long long* in_makespan, const unsigned char* in_flags,
                                 const Key* in_keys, long long n, int k, Key* out_keys,
                                 long long* final_idx, long long* final_makespan, int* final_count);

__global__ void rank_keys_kernel(const long long* makespan, const long long* idle, const int* peak,
                                 const unsigned char* flags, long long n, int D, int mode, int include_over_cap,
                                 long long* key_out, unsigned char* excluded_out);

// Second kernel of the weight-gradient sliding: one lane per (candidate, device) row places the W
// items into the idle time in front of the ops timed by eval_slot_kernel<..., kSlotTimes>.
constexpr int kSlideThreads = 384;
// dynamic LDS of a workgroup: the metadata rows, then 10 KB per wavefront (windows and stash ring)
constexpr int kSlideWaveLdsBytes = 10240;
__global__ void wslide_place_kernel(SlotTables T, const uint16_t* ops, long long n_cand, int stride,
                                    const uint32_t* start_low, const uint32_t* escapes, int escape_cap,
                                    const int32_t* stop_pos,
                                    const unsigned char* timed_flags, uint16_t* ops_out, int stride_out,
                                    long long* out_makespan, long long* out_idle, int* out_peak,
                                    unsigned char* out_flags);

// Pareto front: at most kParetoMaxTiles tiles of kTile candidates (one cursor per tile in LDS).
constexpr int kParetoMergeThreads = 1024;
constexpr int kParetoMaxTiles = 8192;

__global__ void pareto_tile_kernel(const long long* makespan, const int* peak, const unsigned char* flags,
                                   long long n, int D, Key* front_keys, int* front_peak, int* tile_count);

__global__ void pareto_merge_kernel(const Key* front_keys, const int* front_peak, const int* tile_count, int tiles,
                                    int kmax, long long* out_idx, long long* out_makespan, int* out_peak,
                                    int* out_count);

__global__ void apply_caps_kernel(const int* peak, const int* caps, int per_candidate, long long n, int D,
                                  unsigned char* flags);

}  // namespace fpsched

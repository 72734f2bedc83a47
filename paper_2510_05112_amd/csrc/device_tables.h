// Device-side view of one problem: small integer tables that every candidate of a
// batch shares.  Built on the host by fpsched_problem_create and passed to the
// kernels by value (the pointers are DEVICE pointers into one upload).
#pragma once
#include <stdint.h>

namespace fpsched {

constexpr int kMaxDevices = 64;
constexpr int kMaxChunks = 4;
constexpr int kNKinds = 8;

enum Kind : int { kEnd = 0, kF = 1, kB = 2, kW = 3, kR = 4, kO = 5, kL = 6, kFD = 7 };

// Activation state of one (stage, micro-batch); all transitions happen on the
// stage's own device.
enum ActState : int { kAbsent = 0, kRes = 1, kDisc = 2, kOff = 3, kBDone = 4, kDone = 5 };

enum Flag : int { kDeadlock = 1, kIncomplete = 2, kOverCap = 4 };

struct DevTables {
  int32_t D, S, m, has_w;
  int32_t lanes_per_cand;   // power of two >= D
  int32_t cands_per_wave;   // <= 64 / lanes_per_cand, limited by LDS
  int32_t n_table_ints;     // length of `ints`
  // offsets (in int32 units) into `ints`
  int32_t off_dur;          // [kNKinds][S]
  int32_t off_mem_units;    // [S]
  int32_t off_pred_off;     // [S+1]
  int32_t off_pred_stage;   // [E]
  int32_t off_pred_comm;    // [E]  latency, already 0 for same-device edges
  int32_t off_succ_off;     // [S+1]
  int32_t off_succ_stage;   // [E]
  int32_t off_succ_comm;    // [E]
  int32_t off_local_stage;  // [D][kMaxChunks], -1 = none
  int32_t off_n_chunks;     // [D]
  int32_t off_mem_cap;      // [D]
  // Timed form of the generator (generate.hip): one row of eight ints per (instruction type F / B / W,
  // chunk < gen_row_chunks, device), -1 if the DAG has a stage with more than two inputs or outputs:
  //   0 duration   1 units allocated at the start   2 units freed at the end
  //   3 byte offset of the first input slot   4 latency of the first input, or -2^30 if there is none
  //   5, 6 the same for the second input   7 first output slot | second output slot << 16 (degree one:
  //   the first output slot alone)
  // Slots of one parameter set: one word per (direction, class, micro-batch) as in the slot kernel
  // (backward class k at k m, forward class k at (classes + k) m) holding a plain finish time, then m
  // words that take what items without an out-edge write (and that items without an input read).
  int32_t off_gen_rows;
  int32_t gen_row_chunks;   // 1, 2 or 4
  int32_t gen_slot_words;   // (2 * classes + 1) * m
  int32_t gen_spill_words;  // sliding form of the timed generator: queue words per lane in LDS (a power of two), set per launch
  const int32_t* ints;      // DEVICE
};

// Slot kernel tables.  `ints` = [meta][meta2][pad to 512 ints][costs per micro-batch, if any][dev][expect]:
//   meta  [kNKinds * 4][lanes_per_cand] x 4 ints, one 16-byte row per (top five bits of the op
//     word = kind * 4 + chunk, device):
//     x = dur << 8
//     y = (latency of the first input edge << 8) - tag expected on the first input
//     z = required state (low nibble of byte 0) | state transition need ^ next (byte 1)
//         | byte offset of the first output slot, or of the dump region (16) << 16
//     w = units allocated at the op's start (byte 0) | units freed at its end (byte 1)
//         | own stage (byte 2) | 0xff if the op has a first input edge, else 0 (byte 3)
//     Rows of words that may not appear on the device (no such chunk, kind 0, W without split
//     backward) require state 15, which no activation is ever in.
//   meta2 [2 * 4 + 1][lanes_per_cand] x 2 ints, second input/output edge per (direction, chunk,
//     device); the last row is all zero (read by kinds without cross-stage edges):
//     x = (latency of the second input edge << 8) - its tag
//     y = byte offset of the second output slot (16) | kMetaHasProd | kMetaHasCons
//   dev   [lanes_per_cand] x (2 + 4V) ints: chunks on the device, memory cap / unit_scale, then per
//     chunk the slot offsets of the first forward / first backward / second forward / second
//     backward input
//   expect [lanes_per_cand][state_words]: the device's state words when every activation is done
// A slot is one dword, finish << 8 | producer stage; offsets count from the candidate's slot
// base: class * m slots for backward values, (classes + class) * m for forward values; the dump
// region (m slots written by ops without an output edge, never read) starts at 2 * classes * m.
// Memory units are divided by their greatest common divisor (unit_scale) and must then fit a byte.
constexpr unsigned kMetaHasProd = 1u << 30;
constexpr unsigned kMetaHasCons = 1u << 31;
constexpr unsigned kEmptySlot = 0x000000ffu;  // finish 0, tag 0xff = no stage

// dwords of one device's row of costs per micro-batch (one or two bytes each): enough for m values, and odd
constexpr unsigned slot_mb_row_dwords(int m, int value_bytes) { return (((unsigned)m * (unsigned)value_bytes + 3u) >> 2) | 1u; }

struct SlotTables {
  int32_t D, m;
  int32_t lanes_per_cand;   // power of two >= D
  int32_t cands_per_wave;
  int32_t n_classes;        // slot classes (1 for a chain)
  int32_t slots_per_cand;   // (2 * classes + 1) * m, rounded up to a multiple of 8
  int32_t unit_scale;       // common divisor of the memory units
  int32_t state_words;      // dwords of 4-bit activation states per lane
  int32_t wave_ints;        // LDS dwords owned by one wavefront (512 of them its op window)
  int32_t n_shared_ints;    // meta + meta2 + pad to a multiple of 512, copied to LDS once per workgroup
  int32_t off_meta2;        // in ints
  int32_t off_dev;          // in ints
  int32_t dev_ints;         // 2 + 4V
  int32_t off_expect;       // in ints
  int32_t off_mb;           // in ints; costs per micro-batch inside the shared part (0 = none): values of
                            // mb_value_bytes (1 or 2) bytes, [block][chunk < V][lanes_per_cand][row of
                            // slot_mb_row_dwords(m, bytes) dwords], padded to a multiple of 512 ints
  int32_t mb_value_bytes;
  int32_t link_words;       // link mode: dwords per lane behind its state words, one per device this device
                            // sends to, one for values that stay on the device and, last, one that takes
                            // what ops without an out-edge write (0 = plain model);
                            // the dev rows then have 4V more ints: per chunk the first forward / first backward /
                            // second forward / second backward out-edge as latency << 16 | byte offset of its
                            // link word (link index * 256)
  int32_t copy_depth;       // copy-engine form: transfers the engine holds at most (1..7), else 0; link_words is
                            // then the number of ring dwords per lane behind its state words
  int32_t off_w;            // in ints; sliding form: per device [lanes_per_cand][2 * kMaxChunks + 1]: cost << 8 of the
                            // W item of each chunk, the units it frees, then (cost << 8 of all W items of the device)
  uint32_t mb_kind_map;     // four bits per kind: which block of the table at off_mb holds the kind's costs
                            // (kinds with the same costs share a block)
  const int32_t* ints;      // DEVICE
};

// Tables of the evaluation with synchronisation stages and dependency pairs (eval_sync.hip).  Every
// dependency of an item -- the edges of the stage DAG and the user's pairs alike -- is one entry of a list
// per (kind, stage): which finish-time table it looks into (0 forward, 1 backward, 2 weight gradient), the
// producing stage, and the latency (already 0 when both stages sit on one device).
struct SyncTables {
  int32_t D, S, m, has_w;
  int32_t lanes_per_cand;   // power of two >= D
  int32_t cands_per_wave;   // limited by LDS
  int32_t n_fin_tables;     // 2, or 3 if some pair waits for a weight-gradient item
  int32_t copy_depth;       // copy-engine form: transfers the engine holds at most (1..7), else 0
  int32_t n_table_ints;     // length of `ints`
  // offsets (in int32 units) into `ints`
  int32_t off_dur;          // [kNKinds][S]
  int32_t off_mem_units;    // [S]
  int32_t off_group;        // [S] micro-batches per item of the stage
  int32_t off_items;        // [S] items per kind: ceil(m / group)
  int32_t off_dep_off;      // [kNKinds * S + 1] first entry of (kind, stage) in the dependency list
  int32_t off_dep;          // [entries][3]: table, producing stage, latency
  int32_t off_local_stage;  // [D][kMaxChunks], -1 = none
  int32_t off_n_chunks;     // [D]
  int32_t off_mem_cap;      // [D]
  const int32_t* ints;      // DEVICE
};

}  // namespace fpsched

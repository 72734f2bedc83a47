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
  int32_t off_pred_cls;     // [E]  slot class of the edge (pred CSR order)
  int32_t off_succ_cls;     // [E]  slot class of the edge (succ CSR order)
  // slot kernel geometry
  int32_t n_classes;        // slot classes (1 for a chain)
  int32_t state_words;      // dwords of 4-bit activation states per lane
  int32_t slot_cands_per_wave;
  int32_t wave_ints;        // LDS dwords owned by one wavefront in the slot kernel
  int32_t table_ints_padded;
  const int32_t* ints;      // DEVICE
};

}  // namespace fpsched

// C ABI of libfpsched: problem handles, host-side helpers and kernel launches.
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <new>
#include <numeric>
#include <vector>

#include "../../include/fpsched.h"
#include "kernels.h"

using namespace fpsched;

struct fpsched_problem {
  int32_t D = 0, S = 0, m = 0, has_w = 0;
  int device_id = -1;
  int32_t max_stride = 0;
  std::vector<int32_t> stage_device, stage_chunk, local_stage, n_chunks;
  std::vector<int32_t> host_ints;  // the table image uploaded to the GPU
  DevTables tables{};
  int32_t* d_ints = nullptr;
  int32_t lds_bytes = 0;           // dynamic LDS of the general kernel (one wave per group)
  int32_t max_lds = 0;
  int32_t max_degree = 0;          // largest in- or out-degree of a stage in the DAG
  int32_t n_cu = 0;                // compute units of the device
  void* d_static_scratch = nullptr; // this device's copy of the library's static scratch array
  bool general_ok = false, slots_ok = false;  // which kernels fit this problem in LDS
  bool use_slots = false;          // selected kernel: slot kernel (default when it fits) or general
  int32_t slot_v = 0;              // template bound on chunks per device
  bool slot_deg2 = false;          // some stage has two inputs or two outputs
  int32_t slot_lds_bytes = 0;      // dynamic LDS of one slot-kernel workgroup
  int32_t slot_waves = 0;          // wavefronts per slot-kernel workgroup
  int32_t slot_grid = 0;           // resident workgroups: the persistent grid
  bool slide_ok = false;           // the sliding pass is available (split backward, slot tables)
  SlotTables stab_times{};         // the slot tables of the lists without their W items
  int32_t* d_times_ints = nullptr;
  bool slide_eval_ok = false;      // the one-kernel form of the sliding pass (results only) is available
  SlotTables stab_slide{};         // stab_times plus the costs of the W items
  int32_t* d_slide_ints = nullptr;
  std::vector<int32_t> slide_w_table;   // host copy of those costs (layout: SlotTables::off_w)
  bool links_slide_eval_ok = false;     // ... and its form under the link model
  SlotTables stab_slide_links{};
  int32_t* d_slide_links_image = nullptr;
  SlotTables stab{};
  std::vector<int32_t> slot_ints;
  int32_t* d_slot_ints = nullptr;
  // costs per micro-batch (fpsched_problem_set_microbatch_costs)
  int64_t max_comm = 0;
  bool mb_set = false;
  bool mb_slots_ok = false;        // the table's values fit the slot kernel's 24-bit times
  int32_t* d_mb_raw = nullptr;     // [kinds][S][m]
  int32_t* d_mb_rows = nullptr;    // [32 metadata rows][lanes per candidate][m], << 8
  // link occupancy (fpsched_problem_set_link_occupancy): a table image with longer dev rows
  int64_t max_dur = 0;
  bool links_on = false;
  SlotTables stab_links{};
  int32_t* d_links_image = nullptr;
  // both variants together: the cost-table image with the link form's device rows
  std::vector<int32_t> mb_image_host;   // host copy of the image behind stab_mb
  std::vector<int32_t> link_rows;       // [lanes per candidate][4V] out-edge entries of the link form
  int32_t link_words = 0;
  int64_t mb_max_dur = 0;               // largest value of the cost table that is set
  bool combo_ok = false;
  SlotTables stab_combo{};
  int32_t* d_combo_image = nullptr;
  size_t combo_image_ints = 0;
  int32_t combo_waves = 0, combo_grid = 0, combo_lds_bytes = 0;
  std::vector<int32_t> times_ints;      // host copy of the timing pass's table image
  bool links_slide_ok = false;          // the sliding pass has a link form (its LDS fits)
  SlotTables stab_times_links{};
  int32_t* d_times_links_image = nullptr;
  int32_t links_waves = 0, links_grid = 0, links_lds_bytes = 0;
  // synchronisation stages and dependency pairs (fpsched_problem_set_sync)
  bool sync_on = false;
  int32_t copy_depth = 0;               // copy-engine form (fpsched_problem_set_copy_engine), 0 = off
  bool sync_slots_ok = false;           // the synchronisation model has a slot-kernel form for this setting
  SlotTables stab_sync{};
  bool sync_deg2 = false;
  int32_t* d_sync_slot_image = nullptr;
  size_t sync_slot_image_ints = 0;
  int32_t sync_slot_waves = 0, sync_slot_grid = 0, sync_slot_lds_bytes = 0;
  bool copy_slots_ok = false;           // ... which the slot kernel can run (its rings fit LDS)
  SlotTables stab_copy{};
  int32_t copy_waves = 0, copy_grid = 0, copy_lds_bytes = 0;
  std::vector<int32_t> sync_items;      // [S] items per kind of each stage (m while the model is off)
  SyncTables sync_tab{};
  int32_t* d_sync_ints = nullptr;
  size_t sync_ints_capacity = 0;
  int32_t sync_lds_bytes = 0;
  // ... or, when the values fit sixteen bits and the table fits LDS, inside a second table image
  bool mb_in_lds = false;
  SlotTables stab_mb{};
  int32_t* d_mb_image = nullptr;
  size_t mb_image_ints = 0;
  int32_t mb_waves = 0, mb_grid = 0, mb_lds_bytes = 0;
};

namespace {

int check_hip(hipError_t e) { return e == hipSuccess ? FPSCHED_OK : FPSCHED_EHIP; }

// Device memory of fpsched_evaluate_topk_static, the entry point for callers that cannot allocate: the
// work counter and the top-k key buffers that the other entry points take from the caller's workspace.
// Every GPU the library runs on holds its own copy of the array until the process ends.  In host code the
// array's name is only a stand-in: the address on a device comes from hipGetSymbolAddress, asked once per
// device with that device current, and only that pointer is ever handed to a kernel.
constexpr size_t kStaticScratchBytes = FPSCHED_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxGpus = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxGpus] = {nullptr};

// The device must be current.  FPSCHED_EHIP if the runtime does not give the address.
int static_scratch_of(int device_id, void** out) {
  *out = nullptr;
  if (device_id < 0 || device_id >= kMaxGpus) return FPSCHED_EINVAL;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device_id]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
      (void)hipGetLastError();
      return FPSCHED_EHIP;
    }
    g_scratch_ptr[device_id] = ptr;
  }
  *out = g_scratch_ptr[device_id];
  return FPSCHED_OK;
}

struct DeviceGuard {
  int prev = -1;
  bool ok = false;
  explicit DeviceGuard(int dev) {
    if (hipGetDevice(&prev) != hipSuccess) return;
    ok = (prev == dev) || hipSetDevice(dev) == hipSuccess;
    if (prev == dev) prev = -1;
  }
  ~DeviceGuard() {
    if (prev >= 0) (void)hipSetDevice(prev);
  }
};

using SlotKernel = void (*)(SlotTables, const uint16_t*, long long, int, long long*, long long*, int*,
                            unsigned char*, unsigned long long*, int, uint32_t*, int32_t*, const int32_t*, uint32_t*, int);
template <int MODE>   // kSlotPlain, kSlotTimes, ...
SlotKernel slot_kernel_of(int v, bool deg2, bool one_class) {
  if (deg2)
    return v == 1 ? &eval_slot_kernel<1, true, false, MODE>
                  : (v == 2 ? &eval_slot_kernel<2, true, false, MODE> : &eval_slot_kernel<4, true, false, MODE>);
  if (one_class)
    return v == 1 ? &eval_slot_kernel<1, false, true, MODE>
                  : (v == 2 ? &eval_slot_kernel<2, false, true, MODE> : &eval_slot_kernel<4, false, true, MODE>);
  return v == 1 ? &eval_slot_kernel<1, false, false, MODE>
                : (v == 2 ? &eval_slot_kernel<2, false, false, MODE> : &eval_slot_kernel<4, false, false, MODE>);
}
SlotKernel slot_kernel_ptr(int v, bool deg2, bool one_class) { return slot_kernel_of<kSlotPlain>(v, deg2, one_class); }

// Launch shape of the slot kernel for a batch: `waves` wavefronts per workgroup and `grid` workgroups fill the
// chip; a batch too small for that is spread over as many compute units as it has wavefronts' worth of
// candidates (a wavefront that has a SIMD to itself runs its rounds faster than three that share one), with
// fewer wavefronts per workgroup and the LDS that goes with them.
struct SlotLaunch { int waves; int64_t blocks; size_t lds_bytes; };
static SlotLaunch slot_launch(const SlotTables& tab, int waves, int grid, size_t lds_bytes, int64_t n_cand) {
  const int64_t cpw = tab.cands_per_wave;
  const int64_t spread = (n_cand + cpw * grid - 1) / (cpw * grid);   // wavefronts per workgroup that cover the batch
  const int w = (int)std::clamp<int64_t>(spread, 1, waves);
  SlotLaunch L;
  L.waves = w;
  L.blocks = std::min<int64_t>((n_cand + cpw * w - 1) / (cpw * w), grid);
  L.lds_bytes = lds_bytes - (size_t)(waves - w) * (size_t)tab.wave_ints * 4u;
  return L;
}

// Workgroup shape of the slot kernel for a shared LDS part of n_shared_ints dwords: candidates per
// wavefront, then the split of a compute unit's LDS into workgroups that keeps the most wavefronts
// resident (LDS is the only limiter: ~50 VGPRs).  Returns wavefronts per workgroup (0 = does not fit).
struct SlotGeometry { int cands_per_wave, wave_ints, waves, groups; };
SlotGeometry slot_geometry(int64_t n_shared_ints, int lanes_per_cand, int state_words, int slots_per_cand, int max_lds,
                           int max_cands_per_wave = 64) {
  int scpw = std::min(64 / lanes_per_cand, max_cands_per_wave);
  const int64_t fixed = 64ll * (8 + state_words);  // 16 op words + state words per lane
  const int64_t lds_ints = max_lds / 4;
  while (scpw > 1 && n_shared_ints + fixed + (int64_t)scpw * slots_per_cand > lds_ints) scpw >>= 1;
  const int64_t wave_ints = fixed + (int64_t)scpw * slots_per_cand;
  int best_waves = 0, best_groups = 0, best_total = 0;
  for (int groups = 1; groups <= 8; ++groups) {
    const int64_t per_group = lds_ints / groups - n_shared_ints - 64;  // allocation slack
    int wv = per_group > 0 ? (int)std::min<int64_t>(per_group / wave_ints, kSlotMaxWaves) : 0;
    wv = std::min(wv, 32 / groups);  // 8 wavefronts per SIMD, 4 SIMDs per compute unit
    if (wv * groups > best_total) { best_total = wv * groups; best_waves = wv; best_groups = groups; }
  }
  // tuning knob: FPSCHED_SLOT_WAVES=n caps the wavefronts per workgroup (one workgroup per CU)
  if (const char* env = getenv("FPSCHED_SLOT_WAVES")) {
    const int cap_waves = atoi(env);
    if (cap_waves >= 1 && cap_waves < best_waves * best_groups) { best_waves = std::min(cap_waves, best_waves); best_groups = 1; }
  }
  return SlotGeometry{scpw, (int)wave_ints, best_waves, std::max(best_groups, 1)};
}

int next_pow2(int x) {
  int p = 1;
  while (p < x) p <<= 1;
  return p;
}

}  // namespace

extern "C" {

int fpsched_version(void) { return FPSCHED_VERSION; }

const char* fpsched_strerror(int code) {
  switch (code) {
    case FPSCHED_OK: return "ok";
    case FPSCHED_EINVAL: return "invalid argument";
    case FPSCHED_ENOMEM: return "out of memory or workspace too small";
    case FPSCHED_EHIP: return "HIP runtime call failed";
    case FPSCHED_EOVERFLOW: return "time bound does not fit int32";
    case FPSCHED_ENODEV: return "host-only problem handle";
    case FPSCHED_EUNSUPPORTED: return "problem too large for the on-chip tables";
    case FPSCHED_ESCRATCH: return "batch too large for the library's static scratch memory";
    default: return "unknown error";
  }
}

int fpsched_problem_create(const fpsched_problem_desc* desc, int device_id, int32_t max_stride_words,
                           fpsched_problem** out) {
  if (!desc || !out) return FPSCHED_EINVAL;
  *out = nullptr;
  const int D = desc->n_devices, S = desc->n_stages, m = desc->n_microbatches, E = desc->n_edges;
  if (D < 1 || D > FPSCHED_MAX_DEVICES || S < 1 || S > D * FPSCHED_MAX_CHUNKS || m < 1 ||
      m > FPSCHED_MAX_MICROBATCHES || E < 0 || max_stride_words < 8 || (max_stride_words & 7))
    return FPSCHED_EINVAL;
  if (!desc->stage_device || !desc->dur || !desc->mem_units || !desc->mem_cap) return FPSCHED_EINVAL;
  if (E > 0 && (!desc->edge_src || !desc->edge_dst || !desc->edge_comm)) return FPSCHED_EINVAL;

  fpsched_problem* p = new (std::nothrow) fpsched_problem;
  if (!p) return FPSCHED_ENOMEM;
  p->D = D; p->S = S; p->m = m; p->has_w = desc->has_w ? 1 : 0;
  p->device_id = device_id < 0 ? -1 : device_id;
  p->max_stride = max_stride_words;
  p->stage_device.assign(desc->stage_device, desc->stage_device + S);
  p->stage_chunk.assign(S, 0);
  p->local_stage.assign((size_t)D * kMaxChunks, -1);
  p->n_chunks.assign(D, 0);
  p->sync_items.assign(S, m);
  int rc = FPSCHED_OK;
  for (int s = 0; s < S && rc == FPSCHED_OK; ++s) {
    const int d = p->stage_device[s];
    if (d < 0 || d >= D || p->n_chunks[d] >= kMaxChunks) { rc = FPSCHED_EINVAL; break; }
    p->stage_chunk[s] = p->n_chunks[d];
    p->local_stage[(size_t)d * kMaxChunks + p->n_chunks[d]++] = s;
  }
  // edges: range, non-negative latency, acyclic (Kahn over stages)
  int64_t max_dur = 0, max_comm = 0, units_total = 0;
  if (rc == FPSCHED_OK) {
    std::vector<int> indeg(S, 0);
    for (int e = 0; e < E; ++e) {
      const int a = desc->edge_src[e], b = desc->edge_dst[e];
      if (a < 0 || a >= S || b < 0 || b >= S || a == b || desc->edge_comm[e] < 0) { rc = FPSCHED_EINVAL; break; }
      indeg[b]++;
      max_comm = std::max<int64_t>(max_comm, desc->edge_comm[e]);
    }
    if (rc == FPSCHED_OK) {
      std::vector<int> order;
      for (int s = 0; s < S; ++s) if (!indeg[s]) order.push_back(s);
      for (size_t i = 0; i < order.size(); ++i)
        for (int e = 0; e < E; ++e)
          if (desc->edge_src[e] == order[i] && --indeg[desc->edge_dst[e]] == 0) order.push_back(desc->edge_dst[e]);
      if ((int)order.size() != S) rc = FPSCHED_EINVAL;
    }
  }
  if (rc == FPSCHED_OK) {
    for (int i = 0; i < kNKinds * S; ++i) {
      if (desc->dur[i] < 0) { rc = FPSCHED_EINVAL; break; }
      max_dur = std::max<int64_t>(max_dur, desc->dur[i]);
    }
    for (int s = 0; s < S && rc == FPSCHED_OK; ++s) {
      if (desc->mem_units[s] < 0) rc = FPSCHED_EINVAL;
      units_total += (int64_t)desc->mem_units[s] * m;
    }
    // (a negative cap would round towards zero when divided by the units' common divisor)
    for (int d = 0; d < D && rc == FPSCHED_OK; ++d)
      if (desc->mem_cap[d] < 0) rc = FPSCHED_EINVAL;
  }
  // every finish time is at most (number of listed ops) * (largest duration + largest
  // latency); resident memory is at most the sum of all activations
  if (rc == FPSCHED_OK) {
    const int64_t bound = (int64_t)D * max_stride_words * (max_dur + max_comm);
    if (bound >= (int64_t)1 << 31 || units_total >= (int64_t)1 << 31) rc = FPSCHED_EOVERFLOW;
  }
  if (rc != FPSCHED_OK) { delete p; return rc; }
  p->max_comm = max_comm;
  p->max_dur = max_dur;

  // table image
  std::vector<int32_t>& I = p->host_ints;
  DevTables& T = p->tables;
  T.D = D; T.S = S; T.m = m; T.has_w = p->has_w;
  auto append = [&](const int32_t* src, size_t n) { int32_t off = (int32_t)I.size(); I.insert(I.end(), src, src + n); return off; };
  T.off_dur = append(desc->dur, (size_t)kNKinds * S);
  T.off_mem_units = append(desc->mem_units, S);
  std::vector<int32_t> poff(S + 1, 0), soff(S + 1, 0), pst(E), pcm(E), sst(E), scm(E);
  for (int e = 0; e < E; ++e) { poff[desc->edge_dst[e] + 1]++; soff[desc->edge_src[e] + 1]++; }
  for (int s = 0; s < S; ++s) { poff[s + 1] += poff[s]; soff[s + 1] += soff[s]; }
  {
    std::vector<int32_t> pf(S, 0), sf(S, 0);
    for (int e = 0; e < E; ++e) {
      const int a = desc->edge_src[e], b = desc->edge_dst[e];
      const int32_t lat = p->stage_device[a] != p->stage_device[b] ? desc->edge_comm[e] : 0;
      pst[poff[b] + pf[b]] = a; pcm[poff[b] + pf[b]++] = lat;
      sst[soff[a] + sf[a]] = b; scm[soff[a] + sf[a]++] = lat;
    }
  }
  T.off_pred_off = append(poff.data(), S + 1);
  T.off_pred_stage = append(pst.data(), E);
  T.off_pred_comm = append(pcm.data(), E);
  T.off_succ_off = append(soff.data(), S + 1);
  T.off_succ_stage = append(sst.data(), E);
  T.off_succ_comm = append(scm.data(), E);
  for (int s = 0; s < S; ++s)
    p->max_degree = std::max({p->max_degree, poff[s + 1] - poff[s], soff[s + 1] - soff[s]});
  T.off_local_stage = append(p->local_stage.data(), (size_t)D * kMaxChunks);
  T.off_n_chunks = append(p->n_chunks.data(), D);
  T.off_mem_cap = append(desc->mem_cap, D);
  // Slot classes: chains of edges such that each edge starts at the stage the previous
  // one ends in.  Stages are visited in topological order; an out-edge continues the
  // class of a not yet continued in-edge of its stage, else it opens a new class.
  std::vector<int32_t> edge_cls(E, -1);
  int n_classes = 0;
  {
    std::vector<int> indeg(S, 0), order;
    for (int e = 0; e < E; ++e) indeg[desc->edge_dst[e]]++;
    for (int s = 0; s < S; ++s) if (!indeg[s]) order.push_back(s);
    for (size_t i = 0; i < order.size(); ++i) {
      const int s = order[i];
      std::vector<int32_t> arriving;
      for (int e = 0; e < E; ++e) if (desc->edge_dst[e] == s) arriving.push_back(edge_cls[e]);
      size_t used = 0;
      for (int e = 0; e < E; ++e) {
        if (desc->edge_src[e] != s) continue;
        edge_cls[e] = used < arriving.size() ? arriving[used++] : n_classes++;
        if (--indeg[desc->edge_dst[e]] == 0) order.push_back(desc->edge_dst[e]);
      }
    }
    if (n_classes == 0) n_classes = 1;
  }
  T.n_table_ints = (int32_t)I.size();   // what the table-walking kernels copy to LDS ends here
  // Rows of the timed generator: what an item of (type, chunk) on a device costs, where its inputs'
  // finish times lie and where its own goes (layout: device_tables.h).
  T.off_gen_rows = -1;
  T.gen_row_chunks = 1;
  T.gen_slot_words = (2 * n_classes + 1) * m;
  if (p->max_degree <= 2 && 4ll * (2 * n_classes + 1) * m <= 0xffff) {
    int max_chunks = 1;
    for (int d = 0; d < D; ++d) max_chunks = std::max(max_chunks, p->n_chunks[d]);
    const int V = max_chunks <= 1 ? 1 : (max_chunks <= 2 ? 2 : 4);
    T.gen_row_chunks = V;
    std::vector<int32_t> pcl(E), scl(E), pf(S, 0), sf(S, 0);
    for (int e = 0; e < E; ++e) {
      const int a = desc->edge_src[e], b = desc->edge_dst[e];
      pcl[poff[b] + pf[b]++] = edge_cls[e];
      scl[soff[a] + sf[a]++] = edge_cls[e];
    }
    const int32_t dump = 4 * 2 * n_classes * m, none = -(1 << 30);   // slot offsets in bytes
    std::vector<int32_t> rows((size_t)3 * V * D * 8, 0);
    for (int t = 0; t < 3; ++t)
      for (int c = 0; c < V; ++c)
        for (int d = 0; d < D; ++d) {
          int32_t* r = &rows[(((size_t)t * V + c) * D + d) * 8];
          // (a DAG of degree one has no second output: word 7 is then the first output's offset alone)
          r[3] = dump; r[4] = none; r[5] = dump; r[6] = none; r[7] = p->max_degree <= 1 ? dump : dump | (dump << 16);
          if (c >= p->n_chunks[d]) continue;
          const int s = p->local_stage[(size_t)d * kMaxChunks + c];
          const int kind = t == 0 ? kF : (t == 1 ? kB : kW);
          r[0] = desc->dur[kind * S + s];
          r[1] = t == 0 ? desc->mem_units[s] : 0;
          r[2] = (t == 2 || (t == 1 && !p->has_w)) ? desc->mem_units[s] : 0;
          if (t == 2) continue;
          // forward items read the values of their in-edges and write those of their out-edges; backward
          // items the other way round
          const std::vector<int32_t>& ioff = t == 0 ? poff : soff;
          const std::vector<int32_t>& icl = t == 0 ? pcl : scl;
          const std::vector<int32_t>& ilat = t == 0 ? pcm : scm;
          const std::vector<int32_t>& ooff = t == 0 ? soff : poff;
          const std::vector<int32_t>& ocl = t == 0 ? scl : pcl;
          const int32_t dir_base = t == 0 ? n_classes : 0;
          for (int k = 0; k < ioff[s + 1] - ioff[s]; ++k) {
            r[3 + 2 * k] = 4 * (dir_base + icl[ioff[s] + k]) * m;
            r[4 + 2 * k] = ilat[ioff[s] + k];
          }
          int32_t out[2] = {dump, dump};
          for (int k = 0; k < ooff[s + 1] - ooff[s]; ++k) out[k] = 4 * (dir_base + ocl[ooff[s] + k]) * m;
          r[7] = p->max_degree <= 1 ? out[0] : out[0] | (out[1] << 16);
        }
    T.off_gen_rows = append(rows.data(), rows.size());
  }
  T.lanes_per_cand = next_pow2(D);
  T.cands_per_wave = 64 / T.lanes_per_cand;

  if (p->device_id >= 0) {
    DeviceGuard g(p->device_id);
    if (!g.ok) { delete p; return FPSCHED_EHIP; }
    int max_lds = 0;
    if (hipDeviceGetAttribute(&max_lds, hipDeviceAttributeMaxSharedMemoryPerBlock, p->device_id) != hipSuccess) {
      delete p; return FPSCHED_EHIP;
    }
    p->max_lds = max_lds;
    if (static_scratch_of(p->device_id, &p->d_static_scratch) != FPSCHED_OK) { delete p; return FPSCHED_EHIP; }
    // (The dynamic-LDS limit of a kernel is one value per process, not per handle: it is always raised
    // to the device's maximum, so that handles with different needs never undo each other's setting.)
    // general kernel geometry: finish-time tables and state bytes of whole candidates in LDS
    const int64_t SM = (int64_t)S * m;
    const int64_t per_cand = 4 * (2 * SM + ((SM + 3) >> 2));
    const int64_t table_bytes = 4ll * T.n_table_ints;
    int cpw = T.cands_per_wave;
    while (cpw > 1 && table_bytes + cpw * per_cand > max_lds) cpw >>= 1;
    p->general_ok = table_bytes + cpw * per_cand <= max_lds;
    T.cands_per_wave = cpw;
    p->lds_bytes = (int32_t)(table_bytes + cpw * per_cand);
    // ---- slot kernel: metadata per (kind, chunk, device), geometry, fit ----
    {
      SlotTables& ST = p->stab;
      int max_chunks = 1;
      for (int d = 0; d < D; ++d) max_chunks = std::max(max_chunks, p->n_chunks[d]);
      const int V = p->slot_v = max_chunks <= 1 ? 1 : (max_chunks <= 2 ? 2 : 4);
      const int lpc = T.lanes_per_cand;
      // memory units are carried in bytes: divide them (and the caps) by their common divisor
      int64_t unit_scale = 0;
      for (int s = 0; s < S; ++s) unit_scale = std::gcd<int64_t, int64_t>(unit_scale, desc->mem_units[s]);
      if (unit_scale < 1) unit_scale = 1;
      const int slot_stride = ((2 * n_classes + 1) * m + 7) & ~7;   // slots of one candidate
      // slot byte offsets are 16-bit, tags 8-bit (0xff = empty), finish times 24-bit
      bool fits = 4ll * slot_stride <= 0xffff && S <= 255 && max_comm < (1ll << 16) &&
                  (int64_t)D * max_stride_words * (max_dur + max_comm) < (1ll << 24);
      bool deg2 = false;
      for (int s = 0; s < S; ++s) {
        const int nin = poff[s + 1] - poff[s], nout = soff[s + 1] - soff[s];
        if (nin > 2 || nout > 2) fits = false;
        if (nin > 1 || nout > 1) deg2 = true;
        if (desc->mem_units[s] / unit_scale > 0xff) fits = false;
      }
      p->slot_deg2 = deg2;
      // classes of the edges in pred-CSR and succ-CSR order
      std::vector<int32_t> pcl(E), scl(E);
      {
        std::vector<int32_t> pf(S, 0), sf(S, 0);
        for (int e = 0; e < E; ++e) {
          const int a = desc->edge_src[e], b = desc->edge_dst[e];
          pcl[poff[b] + pf[b]++] = edge_cls[e];
          scl[soff[a] + sf[a]++] = edge_cls[e];
        }
      }
      const int n_meta = kNKinds * kMaxChunks * lpc * 4;
      const int n_meta2 = deg2 ? (2 * kMaxChunks + 1) * lpc * 2 : 0;   // + one all-zero row
      const int n_shared = (n_meta + n_meta2 + 511) & ~511;   // the op windows behind it are 2 KB-aligned
      const unsigned dump_bytes = (unsigned)(2 * n_classes * m) * 4u;
      const int dev_ints = 2 + 4 * V;
      const int words_per_chunk = (m + 7) / 8;
      const int state_words = V * words_per_chunk;
      std::vector<int32_t>& J = p->slot_ints;
      J.assign((size_t)n_shared + (size_t)lpc * dev_ints + (size_t)lpc * state_words, 0);
      static const int need_of[kNKinds] = {15, kAbsent, kRes, kBDone, kDisc, kRes, kOff, kAbsent};
      static const int next_of[kNKinds] = {0, kRes, kBDone, kDone, kRes, kOff, kRes, kDisc};
      for (int kind = 0; kind < kNKinds; ++kind)
        for (int c = 0; c < kMaxChunks; ++c)
          for (int d = 0; d < lpc; ++d) {
            int32_t* e = &J[(((size_t)kind * kMaxChunks + c) * lpc + d) * 4];
            e[2] = (int32_t)(15u | (dump_bytes << 16));
            if (d >= D || c >= p->n_chunks[d] || kind == kEnd || (kind == kW && !p->has_w)) continue;
            const int s = p->local_stage[(size_t)d * kMaxChunks + c];
            const unsigned units = (unsigned)(desc->mem_units[s] / unit_scale);
            const bool allocs = kind == kF || kind == kFD || kind == kR || kind == kL;
            const bool frees = kind == kFD || kind == kO || kind == (p->has_w ? kW : kB);
            unsigned has_in = 0, tag = 0, prod = dump_bytes;
            unsigned comm = 0;
            if (kind == kF || kind == kFD) {
              if (poff[s + 1] > poff[s]) { has_in = 0xffu; tag = (unsigned)pst[poff[s]]; comm = (unsigned)pcm[poff[s]]; }
              if (soff[s + 1] > soff[s]) prod = (unsigned)((n_classes + scl[soff[s]]) * m) * 4u;
            } else if (kind == kB) {
              if (soff[s + 1] > soff[s]) { has_in = 0xffu; tag = (unsigned)sst[soff[s]]; comm = (unsigned)scm[soff[s]]; }
              if (poff[s + 1] > poff[s]) prod = (unsigned)(pcl[poff[s]] * m) * 4u;
            }
            e[0] = (int32_t)((unsigned)desc->dur[kind * S + s] << 8);
            e[1] = (int32_t)((comm << 8) - tag);
            e[2] = (int32_t)((unsigned)need_of[kind] | ((unsigned)(need_of[kind] ^ next_of[kind]) << 8) | (prod << 16));
            e[3] = (int32_t)((allocs ? units : 0u) | ((frees ? units : 0u) << 8) | ((unsigned)s << 16) | (has_in << 24));
          }
      for (int dir = 0; dir < 2 && deg2; ++dir)
        for (int c = 0; c < kMaxChunks; ++c)
          for (int d = 0; d < D; ++d) {
            if (c >= p->n_chunks[d]) continue;
            const int s = p->local_stage[(size_t)d * kMaxChunks + c];
            int32_t* e = &J[(size_t)n_meta + (((size_t)dir * kMaxChunks + c) * lpc + d) * 2];
            unsigned y = 0;
            if (dir == 0) {
              if (poff[s + 1] - poff[s] > 1) { y |= kMetaHasCons; e[0] = (int32_t)(((unsigned)pcm[poff[s] + 1] << 8) - (unsigned)pst[poff[s] + 1]); }
              if (soff[s + 1] - soff[s] > 1) y |= kMetaHasProd | ((unsigned)((n_classes + scl[soff[s] + 1]) * m) * 4u);
            } else {
              if (soff[s + 1] - soff[s] > 1) { y |= kMetaHasCons; e[0] = (int32_t)(((unsigned)scm[soff[s] + 1] << 8) - (unsigned)sst[soff[s] + 1]); }
              if (poff[s + 1] - poff[s] > 1) y |= kMetaHasProd | ((unsigned)(pcl[poff[s] + 1] * m) * 4u);
            }
            e[1] = (int32_t)y;
          }
      for (int d = 0; d < D; ++d) {
        // state words of device d once every activation placed on it is consumed
        int32_t* x = &J[(size_t)n_shared + (size_t)lpc * dev_ints + (size_t)d * state_words];
        const unsigned terminal = p->has_w ? kDone : kBDone;
        for (int c = 0; c < p->n_chunks[d]; ++c)
          for (int j = 0; j < m; ++j)
            x[c * words_per_chunk + (j >> 3)] |= (int32_t)(terminal << ((j & 7) * 4));
      }
      for (int d = 0; d < D; ++d) {
        int32_t* e = &J[(size_t)n_shared + (size_t)d * dev_ints];
        e[0] = p->n_chunks[d];
        e[1] = (int32_t)(desc->mem_cap[d] / unit_scale);   // peak > cap  <=>  peak / scale > floor(cap / scale)
        for (int c = 0; c < p->n_chunks[d]; ++c) {
          const int s = p->local_stage[(size_t)d * kMaxChunks + c];
          const int nin = poff[s + 1] - poff[s], nout = soff[s + 1] - soff[s];
          e[2 + c] = nin > 0 ? (n_classes + pcl[poff[s]]) * m : 0;
          e[2 + V + c] = nout > 0 ? scl[soff[s]] * m : 0;
          e[2 + 2 * V + c] = nin > 1 ? (n_classes + pcl[poff[s] + 1]) * m : 0;
          e[2 + 3 * V + c] = nout > 1 ? scl[soff[s] + 1] * m : 0;
        }
      }
      ST.D = D; ST.m = m; ST.lanes_per_cand = lpc; ST.n_classes = n_classes;
      ST.slots_per_cand = slot_stride;
      ST.unit_scale = (int32_t)unit_scale;
      ST.state_words = state_words;
      ST.off_expect = n_shared + lpc * dev_ints;
      ST.n_shared_ints = n_shared;
      ST.off_meta2 = n_meta;
      ST.off_dev = n_shared;
      ST.dev_ints = dev_ints;
      ST.off_mb = 0;
      ST.link_words = 0;
      ST.mb_kind_map = 0;
      ST.mb_value_bytes = 2;
      const SlotGeometry geo = slot_geometry(ST.n_shared_ints, lpc, ST.state_words, ST.slots_per_cand, max_lds);
      const int scpw = geo.cands_per_wave, best_waves = geo.waves, best_groups = geo.groups;
      const int64_t wave_ints = geo.wave_ints;
      p->slots_ok = fits && best_waves >= 1;
      ST.cands_per_wave = scpw;
      ST.wave_ints = (int32_t)wave_ints;
      p->slot_waves = best_waves;
      p->slot_lds_bytes = (int32_t)(4ll * (ST.n_shared_ints + (int64_t)best_waves * wave_ints));
      int n_cu = 0;
      if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, p->device_id) != hipSuccess || n_cu < 1) {
        delete p; return FPSCHED_EHIP;
      }
      p->slot_grid = n_cu * std::max(best_groups, 1);
      p->n_cu = n_cu;
    }
    if (!p->general_ok && !p->slots_ok) { delete p; return FPSCHED_EUNSUPPORTED; }
    p->use_slots = p->slots_ok;
    if (hipMalloc(&p->d_ints, I.size() * sizeof(int32_t)) != hipSuccess) { delete p; return FPSCHED_ENOMEM; }
    bool ok = hipMemcpy(p->d_ints, I.data(), I.size() * sizeof(int32_t), hipMemcpyHostToDevice) == hipSuccess;
    if (ok && p->general_ok)
      ok = hipFuncSetAttribute(reinterpret_cast<const void*>(&eval_general_kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, p->max_lds) == hipSuccess;
    if (ok && p->slots_ok) {
      ok = hipMalloc(&p->d_slot_ints, p->slot_ints.size() * sizeof(int32_t)) == hipSuccess &&
           hipMemcpy(p->d_slot_ints, p->slot_ints.data(), p->slot_ints.size() * sizeof(int32_t),
                     hipMemcpyHostToDevice) == hipSuccess &&
           hipFuncSetAttribute(reinterpret_cast<const void*>(slot_kernel_ptr(p->slot_v, p->slot_deg2, p->stab.n_classes == 1)),
                               hipFuncAttributeMaxDynamicSharedMemorySize, p->max_lds) == hipSuccess;
      p->stab.ints = p->d_slot_ints;
      // The sliding pass times the lists without their W items with the evaluation kernel's TIMES
      // form: the same tables, except that a W word is a no-op (any state, no cost, no memory) and a
      // (stage, micro-batch) is finished once its B item ran.
      if (ok && p->has_w) {
        std::vector<int32_t> J = p->slot_ints;
        const int lpc = p->stab.lanes_per_cand;
        for (int c = 0; c < kMaxChunks; ++c)
          for (int d = 0; d < D; ++d) {
            if (c >= p->n_chunks[d]) continue;
            int32_t* e = &J[(((size_t)kW * kMaxChunks + c) * lpc + d) * 4];
            e[0] = 0;
            e[1] = 0;
            e[2] = (int32_t)((unsigned)e[2] & 0xffff0000u);   // required state 0, no transition, same output slot
            e[3] = (int32_t)((unsigned)e[3] & 0x00ff0000u);   // own stage only
          }
        const int words_per_chunk = (m + 7) / 8;
        for (int d = 0; d < D; ++d) {
          int32_t* x = &J[(size_t)p->stab.off_expect + (size_t)d * p->stab.state_words];
          for (int i = 0; i < p->stab.state_words; ++i) x[i] = 0;
          for (int c = 0; c < p->n_chunks[d]; ++c)
            for (int j = 0; j < m; ++j) x[c * words_per_chunk + (j >> 3)] |= (int32_t)((unsigned)kBDone << ((j & 7) * 4));
        }
        p->stab_times = p->stab;
        p->times_ints = J;
        const bool up = hipMalloc(&p->d_times_ints, J.size() * sizeof(int32_t)) == hipSuccess &&
                        hipMemcpy(p->d_times_ints, J.data(), J.size() * sizeof(int32_t), hipMemcpyHostToDevice) == hipSuccess &&
                        hipFuncSetAttribute(reinterpret_cast<const void*>(slot_kernel_of<kSlotTimes>(p->slot_v, p->slot_deg2, p->stab.n_classes == 1)),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, p->max_lds) == hipSuccess &&
                        hipFuncSetAttribute(reinterpret_cast<const void*>(&wslide_place_kernel),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, p->max_lds) == hipSuccess;
        if (up) {
          p->stab_times.ints = p->d_times_ints;
          p->slide_ok = true;
          // the one-kernel form: the same image, and behind it per device the cost << 8 of the W item of each
          // chunk, the units it frees, and the cost << 8 of all W items of the device
          std::vector<int32_t> JS = J;
          const int32_t off_w = (int32_t)JS.size();
          JS.resize(JS.size() + (size_t)lpc * (2 * kMaxChunks + 1), 0);
          for (int d = 0; d < D; ++d) {
            int32_t* w = &JS[(size_t)off_w + (size_t)d * (2 * kMaxChunks + 1)];
            int64_t total = 0;
            for (int c = 0; c < p->n_chunks[d]; ++c) {
              const int s = p->local_stage[(size_t)d * kMaxChunks + c];
              w[c] = (int32_t)((unsigned)desc->dur[kW * S + s] << 8);
              w[kMaxChunks + c] = (int32_t)(desc->mem_units[s] / p->stab.unit_scale);
              total += (int64_t)m * desc->dur[kW * S + s];
            }
            w[2 * kMaxChunks] = (int32_t)((uint32_t)total << 8);   // (below 2^24: the slot form's bound on all times)
          }
          p->slide_w_table.assign(JS.begin() + off_w, JS.end());
          if (hipMalloc(&p->d_slide_ints, JS.size() * sizeof(int32_t)) == hipSuccess &&
              hipMemcpy(p->d_slide_ints, JS.data(), JS.size() * sizeof(int32_t), hipMemcpyHostToDevice) == hipSuccess &&
              hipFuncSetAttribute(reinterpret_cast<const void*>(slot_kernel_of<kSlotSlide>(p->slot_v, p->slot_deg2, p->stab.n_classes == 1)),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, p->max_lds) == hipSuccess) {
            p->stab_slide = p->stab_times;
            p->stab_slide.ints = p->d_slide_ints;
            p->stab_slide.off_w = off_w;
            p->slide_eval_ok = true;
          } else {
            (void)hipGetLastError();
            if (p->d_slide_ints) { (void)hipFree(p->d_slide_ints); p->d_slide_ints = nullptr; }
          }
        } else {
          (void)hipGetLastError();
          if (p->d_times_ints) { (void)hipFree(p->d_times_ints); p->d_times_ints = nullptr; }
        }
      }
    }
    if (!ok) {
      (void)hipFree(p->d_ints);
      if (p->d_slot_ints) (void)hipFree(p->d_slot_ints);
    if (p->d_sync_slot_image) (void)hipFree(p->d_sync_slot_image);
      if (p->d_times_ints) (void)hipFree(p->d_times_ints);
    if (p->d_slide_ints) (void)hipFree(p->d_slide_ints);
      if (p->d_slide_ints) (void)hipFree(p->d_slide_ints);
      delete p;
      return FPSCHED_EHIP;
    }
    T.ints = p->d_ints;
  }
  *out = p;
  return FPSCHED_OK;
}

void fpsched_problem_destroy(fpsched_problem* p) {
  if (!p) return;
  if (p->d_ints || p->d_slot_ints || p->d_sync_ints) {
    DeviceGuard g(p->device_id);
    if (p->d_ints) (void)hipFree(p->d_ints);
    if (p->d_slot_ints) (void)hipFree(p->d_slot_ints);
    if (p->d_sync_slot_image) (void)hipFree(p->d_sync_slot_image);
    if (p->d_times_ints) (void)hipFree(p->d_times_ints);
    if (p->d_mb_raw) (void)hipFree(p->d_mb_raw);
    if (p->d_mb_rows) (void)hipFree(p->d_mb_rows);
    if (p->d_mb_image) (void)hipFree(p->d_mb_image);
    if (p->d_links_image) (void)hipFree(p->d_links_image);
    if (p->d_times_links_image) (void)hipFree(p->d_times_links_image);
    if (p->d_slide_links_image) (void)hipFree(p->d_slide_links_image);
    if (p->d_combo_image) (void)hipFree(p->d_combo_image);
    if (p->d_sync_ints) (void)hipFree(p->d_sync_ints);
  }
  delete p;
}

int fpsched_problem_info(const fpsched_problem* p, int32_t* lanes_per_candidate,
                         int32_t* candidates_per_wave, int32_t* lds_bytes_per_wave) {
  if (!p) return FPSCHED_EINVAL;
  const bool slots = p->use_slots;
  if (lanes_per_candidate) *lanes_per_candidate = p->tables.lanes_per_cand;
  if (candidates_per_wave) *candidates_per_wave = slots ? p->stab.cands_per_wave : p->tables.cands_per_wave;
  if (lds_bytes_per_wave) *lds_bytes_per_wave = slots ? p->slot_lds_bytes / std::max(p->slot_waves, 1) : p->lds_bytes;
  return FPSCHED_OK;
}

int fpsched_problem_select_kernel(fpsched_problem* p, int which) {
  if (!p) return FPSCHED_EINVAL;
  if (p->device_id < 0) return FPSCHED_ENODEV;
  if (which == FPSCHED_KERNEL_AUTO) p->use_slots = p->slots_ok;
  else if (which == FPSCHED_KERNEL_GENERAL) { if (!p->general_ok) return FPSCHED_EUNSUPPORTED; p->use_slots = false; }
  else if (which == FPSCHED_KERNEL_SLOTS) { if (!p->slots_ok) return FPSCHED_EUNSUPPORTED; p->use_slots = true; }
  else return FPSCHED_EINVAL;
  return FPSCHED_OK;
}

int fpsched_problem_active_kernel(const fpsched_problem* p) {
  if (!p) return FPSCHED_EINVAL;
  if (p->device_id < 0) return FPSCHED_ENODEV;
  if (p->sync_on) return p->use_slots && p->sync_slots_ok ? FPSCHED_KERNEL_SLOTS : FPSCHED_KERNEL_GENERAL;
  if (p->copy_depth > 0) return p->use_slots && p->copy_slots_ok ? FPSCHED_KERNEL_SLOTS : FPSCHED_KERNEL_GENERAL;
  return p->use_slots && (!p->mb_set || p->mb_slots_ok) ? FPSCHED_KERNEL_SLOTS : FPSCHED_KERNEL_GENERAL;
}

static int64_t topk_level_sizes(int64_t n, int32_t k, int64_t* first, int64_t* second) {
  // survivors after level 0 and after level 1 (the two ping-pong buffers)
  const int64_t t0 = std::max<int64_t>(1, (n + kTile - 1) / kTile);
  const int64_t n1 = t0 * k;
  const int64_t t1 = std::max<int64_t>(1, (n1 + kTile - 1) / kTile);
  *first = n1;
  *second = t1 * k;
  return n1 + *second;
}

size_t fpsched_workspace_bytes(const fpsched_problem* p, int64_t n_cand, int32_t k) {
  if (!p || n_cand < 0) return 0;
  int64_t a = 0, b = 0;
  const int64_t keys = k > 0 ? topk_level_sizes(n_cand, std::min(k, 1024), &a, &b) : 0;
  return (size_t)(256 + keys * (int64_t)sizeof(Key));
}

int fpsched_evaluate(const fpsched_problem* p, const uint16_t* d_ops, int64_t n_cand,
                     int32_t stride_words, fpsched_results out, void* d_workspace,
                     size_t workspace_bytes, void* hip_stream) {
  if (!p || n_cand < 0) return FPSCHED_EINVAL;
  if (p->device_id < 0) return FPSCHED_ENODEV;
  if (n_cand == 0) return FPSCHED_OK;
  if (!d_ops || !out.makespan || !out.idle || !out.peak || !out.flags) return FPSCHED_EINVAL;
  if (stride_words < 8 || (stride_words & 7) || stride_words > p->max_stride) return FPSCHED_EINVAL;
  if (reinterpret_cast<uintptr_t>(d_ops) & 15) return FPSCHED_EINVAL;
  DeviceGuard g(p->device_id);
  if (!g.ok) return FPSCHED_EHIP;
  const bool copy_on_slots = p->copy_depth > 0 && p->use_slots && p->copy_slots_ok;
  const bool sync_on_slots = p->sync_on && p->use_slots && p->sync_slots_ok;
  if ((p->sync_on || p->copy_depth > 0) && !copy_on_slots && !sync_on_slots) {
    const int cpw = p->sync_tab.cands_per_wave;
    const int64_t blocks = (n_cand + cpw - 1) / cpw;
    if (blocks > 0x7fffffffll) return FPSCHED_EINVAL;
    hipLaunchKernelGGL(p->copy_depth > 0 ? eval_sync_kernel<true> : eval_sync_kernel<false>, dim3((unsigned)blocks), dim3(64), (size_t)p->sync_lds_bytes,
                       static_cast<hipStream_t>(hip_stream), p->sync_tab, d_ops, (long long)n_cand,
                       (int)stride_words, reinterpret_cast<long long*>(out.makespan),
                       reinterpret_cast<long long*>(out.idle), out.peak, out.flags);
    return check_hip(hipGetLastError());
  }
  if (p->links_on && !p->use_slots) return FPSCHED_EUNSUPPORTED;   // the general kernel has no link form
  if (copy_on_slots || sync_on_slots || (p->use_slots && (!p->mb_set || p->mb_slots_ok))) {
    // the first 8 bytes of the workspace hold the counter the segments draw candidates from
    if (!d_workspace || (reinterpret_cast<uintptr_t>(d_workspace) & 15)) return FPSCHED_EINVAL;
    if (workspace_bytes < 256) return FPSCHED_ENOMEM;
    unsigned long long* counter = static_cast<unsigned long long*>(d_workspace);
    // costs per micro-batch: their own table image and workgroup shape when the table sits in LDS
    const bool mb_lds = p->mb_set && p->mb_in_lds;
    const bool combo = p->links_on && p->mb_set;   // both variants: the setters made sure the tables exist
    if (combo && !p->combo_ok) return FPSCHED_EUNSUPPORTED;
    const bool links = p->links_on && !combo;
    const SlotTables& tab = sync_on_slots ? p->stab_sync : copy_on_slots ? p->stab_copy : combo ? p->stab_combo : links ? p->stab_links : (mb_lds ? p->stab_mb : p->stab);
    const int waves = sync_on_slots ? p->sync_slot_waves : copy_on_slots ? p->copy_waves : combo ? p->combo_waves : links ? p->links_waves : (mb_lds ? p->mb_waves : p->slot_waves);
    const int grid = sync_on_slots ? p->sync_slot_grid : copy_on_slots ? p->copy_grid : combo ? p->combo_grid : links ? p->links_grid : (mb_lds ? p->mb_grid : p->slot_grid);
    const size_t lds_bytes = (size_t)(sync_on_slots ? p->sync_slot_lds_bytes : copy_on_slots ? p->copy_lds_bytes : combo ? p->combo_lds_bytes : links ? p->links_lds_bytes
                                      : (mb_lds ? p->mb_lds_bytes : p->slot_lds_bytes));
    const SlotLaunch L = slot_launch(tab, waves, grid, lds_bytes, n_cand);
    const int per_block = tab.cands_per_wave * L.waves;
    const int64_t blocks = L.blocks;
    // Candidates per atomic draw.  Atomics on one address complete at some 8e7 per second; a batch of
    // long candidates stays far below that and is drawn one by one (best balance at the end of the
    // batch), short rows are drawn several at a time: about one draw per 12 K op words.
    const int64_t row_words = (int64_t)p->D * stride_words;
    const int draw_block = (int)std::clamp<int64_t>((12288 + row_words - 1) / row_words, 1, tab.cands_per_wave);
    // segment g starts on candidate g; the counter hands out the candidates after those
    hipLaunchKernelGGL(reset_counter_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(hip_stream), counter,
                       (unsigned long long)(blocks * per_block));
    const bool one_class = tab.n_classes == 1;
    const SlotKernel kernel = sync_on_slots ? slot_kernel_of<kSlotSync>(p->slot_v, p->sync_deg2, one_class)
                              : copy_on_slots ? slot_kernel_of<kSlotCopy>(p->slot_v, p->slot_deg2, one_class)
                              : combo ? slot_kernel_of<kSlotPerMicrobatchLdsLinks>(p->slot_v, p->slot_deg2, one_class)
                              : links ? slot_kernel_of<kSlotLinks>(p->slot_v, p->slot_deg2, one_class)
                              : !p->mb_set ? slot_kernel_ptr(p->slot_v, p->slot_deg2, one_class)
                              : (mb_lds ? slot_kernel_of<kSlotPerMicrobatchLds>(p->slot_v, p->slot_deg2, one_class)
                                        : slot_kernel_of<kSlotPerMicrobatch>(p->slot_v, p->slot_deg2, one_class));
    hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(64 * L.waves), L.lds_bytes,
                       static_cast<hipStream_t>(hip_stream), tab, d_ops,
                       (long long)n_cand, (int)stride_words, reinterpret_cast<long long*>(out.makespan),
                       reinterpret_cast<long long*>(out.idle), out.peak, out.flags, counter, draw_block,
                       (uint32_t*)nullptr, (int32_t*)nullptr,
                       (const int32_t*)(p->mb_set && !mb_lds && !combo ? p->d_mb_rows : nullptr), (uint32_t*)nullptr, 0);
    return check_hip(hipGetLastError());
  }
  const int cpw = p->tables.cands_per_wave;
  const int64_t blocks = (n_cand + cpw - 1) / cpw;
  if (blocks > 0x7fffffffll) return FPSCHED_EINVAL;
  hipLaunchKernelGGL(eval_general_kernel, dim3((unsigned)blocks), dim3(64), (size_t)p->lds_bytes,
                     static_cast<hipStream_t>(hip_stream), p->tables, d_ops, (long long)n_cand,
                     (int)stride_words, reinterpret_cast<long long*>(out.makespan),
                     reinterpret_cast<long long*>(out.idle), out.peak, out.flags,
                     (const int32_t*)(p->mb_set ? p->d_mb_raw : nullptr));
  return check_hip(hipGetLastError());
}

// Costs per micro-batch and link occupancy together: the image behind stab_mb with the link form's longer
// device rows.  Needs both built (the cost table in LDS).  FPSCHED_EUNSUPPORTED if it does not fit.
static int build_combined_tables(fpsched_problem* p) {
  p->combo_ok = false;
  if (!p->mb_in_lds || p->mb_image_host.empty() || p->link_rows.empty()) return FPSCHED_EUNSUPPORTED;
  const SlotTables& MT = p->stab_mb;
  const int V = p->slot_v, lpc = MT.lanes_per_cand;
  const int dev_ints = MT.dev_ints + 4 * V;
  const int slots_per_cand = (2 * MT.n_classes * p->m + 7) & ~7;   // no dump region in the link form
  SlotGeometry geo = slot_geometry(MT.n_shared_ints, lpc, MT.state_words + p->link_words, slots_per_cand, p->max_lds,
                                   MT.cands_per_wave);
  if (geo.waves * geo.groups < 4 || geo.cands_per_wave != MT.cands_per_wave) return FPSCHED_EUNSUPPORTED;
  const std::vector<int32_t>& B = p->mb_image_host;
  std::vector<int32_t> J((size_t)MT.n_shared_ints + (size_t)lpc * dev_ints + (size_t)lpc * MT.state_words, 0);
  std::copy(B.begin(), B.begin() + MT.n_shared_ints, J.begin());
  for (int d = 0; d < lpc; ++d) {
    int32_t* row = &J[(size_t)MT.n_shared_ints + (size_t)d * dev_ints];
    std::copy(B.begin() + MT.off_dev + (size_t)d * MT.dev_ints, B.begin() + MT.off_dev + (size_t)(d + 1) * MT.dev_ints, row);
    std::copy(p->link_rows.begin() + (size_t)d * 4 * V, p->link_rows.begin() + (size_t)(d + 1) * 4 * V, row + MT.dev_ints);
  }
  std::copy(B.begin() + MT.off_expect, B.end(), J.begin() + MT.n_shared_ints + (size_t)lpc * dev_ints);
  DeviceGuard g(p->device_id);
  if (!g.ok) return FPSCHED_EHIP;
  if (hipDeviceSynchronize() != hipSuccess) return FPSCHED_EHIP;   // an earlier image may be in use
  if (J.size() > p->combo_image_ints) {
    if (p->d_combo_image) (void)hipFree(p->d_combo_image);
    p->d_combo_image = nullptr;
    p->combo_image_ints = 0;
    if (hipMalloc(&p->d_combo_image, J.size() * sizeof(int32_t)) != hipSuccess) { p->d_combo_image = nullptr; return FPSCHED_ENOMEM; }
    p->combo_image_ints = J.size();
  }
  const int32_t lds_bytes = (int32_t)(4ll * (MT.n_shared_ints + (int64_t)geo.waves * geo.wave_ints));
  if (hipMemcpy(p->d_combo_image, J.data(), J.size() * sizeof(int32_t), hipMemcpyHostToDevice) != hipSuccess ||
      hipFuncSetAttribute(reinterpret_cast<const void*>(slot_kernel_of<kSlotPerMicrobatchLdsLinks>(p->slot_v, p->slot_deg2, MT.n_classes == 1)),
                          hipFuncAttributeMaxDynamicSharedMemorySize, p->max_lds) != hipSuccess)
    return FPSCHED_EHIP;
  p->stab_combo = MT;
  p->stab_combo.ints = p->d_combo_image;
  p->stab_combo.link_words = p->link_words;
  p->stab_combo.slots_per_cand = slots_per_cand;
  p->stab_combo.dev_ints = dev_ints;
  p->stab_combo.off_expect = MT.n_shared_ints + lpc * dev_ints;
  p->stab_combo.cands_per_wave = geo.cands_per_wave;
  p->stab_combo.wave_ints = geo.wave_ints;
  p->combo_waves = geo.waves;
  p->combo_grid = p->n_cu * geo.groups;
  p->combo_lds_bytes = lds_bytes;
  p->combo_ok = true;
  if (getenv("FPSCHED_VERBOSE"))
    fprintf(stderr, "[fpsched] costs per micro-batch + link occupancy: %d x %d wavefronts per compute unit\n", geo.groups, geo.waves);
  return FPSCHED_OK;
}

int fpsched_problem_set_microbatch_costs(fpsched_problem* p, const int32_t* dur_mb) {
  if (!p) return FPSCHED_EINVAL;
  if (!dur_mb) {
    p->mb_set = false;   // the tables stay allocated for the next call
    return FPSCHED_OK;
  }
  if (p->sync_on || p->copy_depth > 0) return FPSCHED_EUNSUPPORTED;   // those models know one cost per (type, stage)
  const int D = p->D, S = p->S, m = p->m;
  const size_t n_raw = (size_t)kNKinds * S * m;
  int64_t max_dur = 0;
  for (size_t i = 0; i < n_raw; ++i) {
    if (dur_mb[i] < 0) return FPSCHED_EINVAL;
    max_dur = std::max<int64_t>(max_dur, dur_mb[i]);
  }
  // (with links every item may add two transfers to the longest chain)
  const int64_t bound = (int64_t)D * p->max_stride * (max_dur + (p->links_on ? 2 : 1) * p->max_comm);
  if (bound >= (int64_t)1 << 31) return FPSCHED_EOVERFLOW;
  const bool fits_slots = bound < (1ll << 24);
  if (p->device_id < 0) {
    p->mb_set = true;
    p->mb_slots_ok = fits_slots;
    p->mb_max_dur = max_dur;
    return FPSCHED_OK;
  }
  if (p->links_on && !(p->slots_ok && fits_slots)) return FPSCHED_EUNSUPPORTED;   // the link form is the slot kernel's
  if (!(p->slots_ok && fits_slots) && !p->general_ok) return FPSCHED_EUNSUPPORTED;
  const int lpc = p->tables.lanes_per_cand;
  const size_t n_rows = (size_t)kNKinds * kMaxChunks * lpc * m;
  std::vector<int32_t> rows(n_rows, 0);
  for (int kind = 1; kind < kNKinds; ++kind)
    for (int c = 0; c < kMaxChunks; ++c)
      for (int d = 0; d < D; ++d) {
        if (c >= p->n_chunks[d]) continue;
        const int s = p->local_stage[(size_t)d * kMaxChunks + c];
        for (int j = 0; j < m; ++j)
          rows[(((size_t)kind * kMaxChunks + c) * lpc + d) * m + j] =
              fits_slots ? (int32_t)((unsigned)dur_mb[((size_t)kind * S + s) * m + j] << 8) : 0;
      }
  DeviceGuard g(p->device_id);
  if (!g.ok) return FPSCHED_EHIP;
  // work that reads the previous table must be over before it is overwritten
  if (hipDeviceSynchronize() != hipSuccess) return FPSCHED_EHIP;
  p->mb_set = false;   // a failure from here on leaves the handle on the costs of its description
  if (!p->d_mb_raw && hipMalloc(&p->d_mb_raw, n_raw * sizeof(int32_t)) != hipSuccess) { p->d_mb_raw = nullptr; return FPSCHED_ENOMEM; }
  if (!p->d_mb_rows && hipMalloc(&p->d_mb_rows, n_rows * sizeof(int32_t)) != hipSuccess) { p->d_mb_rows = nullptr; return FPSCHED_ENOMEM; }
  if (hipMemcpy(p->d_mb_raw, dur_mb, n_raw * sizeof(int32_t), hipMemcpyHostToDevice) != hipSuccess ||
      hipMemcpy(p->d_mb_rows, rows.data(), n_rows * sizeof(int32_t), hipMemcpyHostToDevice) != hipSuccess)
    return FPSCHED_EHIP;
  if (p->slots_ok && fits_slots &&
      hipFuncSetAttribute(reinterpret_cast<const void*>(slot_kernel_of<kSlotPerMicrobatch>(p->slot_v, p->slot_deg2, p->stab.n_classes == 1)),
                          hipFuncAttributeMaxDynamicSharedMemorySize, p->max_lds) != hipSuccess)
    return FPSCHED_EHIP;
  // Costs of one or two bytes in LDS next to the metadata, if that leaves room for at least six wavefronts
  // per compute unit: [block][chunk < V][lanes per candidate][row of m values], padded to 2 KB.  Kinds
  // whose costs are the same (a forward pass whether its activation is kept or dropped, a
  // recomputation, ...) share a block.
  bool in_lds = false;
  if (p->slots_ok && fits_slots && max_dur < 65536 && !getenv("FPSCHED_MB_GLOBAL")) {
    const SlotTables& ST = p->stab;
    const int V = p->slot_v;
    int block_of[kNKinds] = {0}, n_blocks = 0, kind_of_block[kNKinds] = {0};
    for (int kind = 1; kind < kNKinds; ++kind) {
      int found = -1;
      for (int b = 0; b < n_blocks && found < 0; ++b)
        if (std::equal(dur_mb + (size_t)kind * S * m, dur_mb + (size_t)(kind + 1) * S * m, dur_mb + (size_t)kind_of_block[b] * S * m)) found = b;
      if (found < 0) { found = n_blocks; kind_of_block[n_blocks++] = kind; }
      block_of[kind] = found;
    }
    uint32_t kind_map = 0;
    for (int kind = 1; kind < kNKinds; ++kind) kind_map |= (uint32_t)block_of[kind] << (4 * kind);
    const int value_bytes = max_dur < 256 ? 1 : 2;
    const int64_t row_dwords = slot_mb_row_dwords(m, value_bytes);   // of one device
    const int64_t table_ints = ((int64_t)n_blocks * V * lpc * row_dwords + 511) & ~511ll;
    const int64_t shared = ST.n_shared_ints + table_ints;
    const SlotGeometry geo = slot_geometry(shared, lpc, ST.state_words, ST.slots_per_cand, p->max_lds, ST.cands_per_wave);
    if (geo.waves * geo.groups >= 6 && geo.cands_per_wave == ST.cands_per_wave) {
      std::vector<int32_t> J((size_t)shared + (p->slot_ints.size() - ST.n_shared_ints), 0);
      std::copy(p->slot_ints.begin(), p->slot_ints.begin() + ST.n_shared_ints, J.begin());
      std::copy(p->slot_ints.begin() + ST.n_shared_ints, p->slot_ints.end(), J.begin() + shared);
      unsigned char* t8 = reinterpret_cast<unsigned char*>(J.data() + ST.n_shared_ints);
      for (int b = 0; b < n_blocks; ++b)
        for (int c = 0; c < V; ++c)
          for (int d = 0; d < D; ++d) {
            if (c >= p->n_chunks[d]) continue;
            const int s = p->local_stage[(size_t)d * kMaxChunks + c];
            unsigned char* row = t8 + (((size_t)b * V + c) * lpc + d) * row_dwords * 4;
            for (int j = 0; j < m; ++j) {
              const uint32_t value = (uint32_t)dur_mb[((size_t)kind_of_block[b] * S + s) * m + j];
              if (value_bytes == 1) row[j] = (unsigned char)value;
              else { row[2 * j] = (unsigned char)value; row[2 * j + 1] = (unsigned char)(value >> 8); }
            }
          }
      if (J.size() > p->mb_image_ints) {   // tables with more distinct kinds need a larger image
        if (p->d_mb_image) (void)hipFree(p->d_mb_image);
        p->d_mb_image = nullptr;
        p->mb_image_ints = 0;
        if (hipMalloc(&p->d_mb_image, J.size() * sizeof(int32_t)) != hipSuccess) { p->d_mb_image = nullptr; return FPSCHED_ENOMEM; }
        p->mb_image_ints = J.size();
      }
      if (hipMemcpy(p->d_mb_image, J.data(), J.size() * sizeof(int32_t), hipMemcpyHostToDevice) != hipSuccess) return FPSCHED_EHIP;
      p->mb_image_host = J;
      p->stab_mb = ST;
      p->stab_mb.ints = p->d_mb_image;
      p->stab_mb.off_mb = ST.n_shared_ints;
      p->stab_mb.mb_kind_map = kind_map;
      p->stab_mb.mb_value_bytes = value_bytes;
      p->stab_mb.n_shared_ints = (int32_t)shared;
      p->stab_mb.off_dev = ST.off_dev + (int32_t)table_ints;
      p->stab_mb.off_expect = ST.off_expect + (int32_t)table_ints;
      p->stab_mb.cands_per_wave = geo.cands_per_wave;
      p->stab_mb.wave_ints = geo.wave_ints;
      p->mb_waves = geo.waves;
      p->mb_grid = p->n_cu * geo.groups;
      p->mb_lds_bytes = (int32_t)(4ll * (shared + (int64_t)geo.waves * geo.wave_ints));
      if (hipFuncSetAttribute(reinterpret_cast<const void*>(slot_kernel_of<kSlotPerMicrobatchLds>(p->slot_v, p->slot_deg2, ST.n_classes == 1)),
                              hipFuncAttributeMaxDynamicSharedMemorySize, p->max_lds) != hipSuccess)
        return FPSCHED_EHIP;
      in_lds = true;
    }
  }
  p->mb_in_lds = in_lds;
  if (p->links_on) {   // both variants: only with the table in LDS; else the handle stays on the links alone
    const int rc = build_combined_tables(p);
    if (rc != FPSCHED_OK) return rc;
  }
  if (getenv("FPSCHED_VERBOSE"))
    fprintf(stderr, "[fpsched] costs per micro-batch: %s; slot kernel %d x %d wavefronts per compute unit (plain: %d x %d), LDS limit %d bytes\n",
            !(p->slots_ok && fits_slots) ? "general kernel" : (in_lds ? "slot kernel, table in LDS" : "slot kernel, table in device memory"),
            in_lds ? p->mb_grid / std::max(p->n_cu, 1) : p->slot_grid / std::max(p->n_cu, 1), in_lds ? p->mb_waves : p->slot_waves,
            p->slot_grid / std::max(p->n_cu, 1), p->slot_waves, p->max_lds);
  p->mb_set = true;
  p->mb_slots_ok = p->slots_ok && fits_slots;
  p->mb_max_dur = max_dur;
  return FPSCHED_OK;
}

int fpsched_problem_set_link_occupancy(fpsched_problem* p, int32_t on) {
  if (!p) return FPSCHED_EINVAL;
  if (!on) {
    p->links_on = false;   // the table image stays allocated for the next call
    return FPSCHED_OK;
  }
  if (p->sync_on || p->copy_depth > 0) return FPSCHED_EUNSUPPORTED;   // those models read transfers as latencies
  const int D = p->D, S = p->S;
  // every finish time is at most the sum of all costs and of all transfers (at most two per op here)
  const int64_t bound = (int64_t)D * p->max_stride * ((p->mb_set ? p->mb_max_dur : p->max_dur) + 2 * p->max_comm);
  if (bound >= (int64_t)1 << 31) return FPSCHED_EOVERFLOW;
  if (p->device_id < 0) {
    p->links_on = true;
    return FPSCHED_OK;
  }
  if (!p->slots_ok || bound >= (1ll << 24)) return FPSCHED_EUNSUPPORTED;
  if (p->d_links_image) {   // built by an earlier call
    if (p->mb_set) {        // both variants: the cost table's image with this form's device rows
      const int rc = build_combined_tables(p);
      if (rc != FPSCHED_OK) return rc;
    }
    p->links_on = true;
    return FPSCHED_OK;
  }
  // links of a device: the devices its stages send to (activations to successor stages, gradients to
  // predecessor stages), numbered in the order they are met
  const std::vector<int32_t>& I = p->host_ints;
  const DevTables& T = p->tables;
  const SlotTables& ST = p->stab;
  const int V = p->slot_v, lpc = ST.lanes_per_cand;
  std::vector<std::vector<int>> sends_to(D);
  auto link_of = [&](int d, int to) {
    for (size_t i = 0; i < sends_to[d].size(); ++i) if (sends_to[d][i] == to) return (int)i;
    sends_to[d].push_back(to);
    return (int)sends_to[d].size() - 1;
  };
  struct OutEdge { int to, comm; };
  auto out_edge = [&](int s, bool forward, int k, OutEdge* e) {
    const int off = forward ? T.off_succ_off : T.off_pred_off;
    const int at = I[off + s] + k;
    if (at >= I[off + s + 1]) return false;
    e->to = p->stage_device[I[(forward ? T.off_succ_stage : T.off_pred_stage) + at]];
    e->comm = I[(forward ? T.off_succ_comm : T.off_pred_comm) + at];
    return true;
  };
  for (int s = 0; s < S; ++s)
    for (int fwd = 0; fwd < 2; ++fwd)
      for (int k = 0; k < 2; ++k) {
        OutEdge e;
        if (out_edge(s, fwd != 0, k, &e) && e.to != p->stage_device[s]) (void)link_of(p->stage_device[s], e.to);
      }
  // two more words per lane: one for values that stay on the device (latency 0; it only ever holds
  // earlier finish times of the device, so nothing waits for it) and one that takes what ops without an
  // out-edge write
  int link_words = 2;
  for (int d = 0; d < D; ++d) link_words = std::max(link_words, (int)sends_to[d].size() + 2);
  if (link_words * 256 > 0xffff) return FPSCHED_EUNSUPPORTED;
  const uint32_t spare = (uint32_t)(link_words - 2) * 256u;
  // (this form of the kernel needs no dump region behind the slots: ops without an out-edge write the
  // lane's last link word)
  const int slots_per_cand = (2 * ST.n_classes * p->m + 7) & ~7;
  // (as many candidates per wavefront as the plain tables: the per-lane constants are shared)
  SlotGeometry geo = slot_geometry(ST.n_shared_ints, lpc, ST.state_words + link_words, slots_per_cand, p->max_lds,
                                   ST.cands_per_wave);
  if (geo.waves < 1 || geo.cands_per_wave != ST.cands_per_wave) return FPSCHED_EUNSUPPORTED;
  // never more wavefronts than the plain kernel runs with: where this form would fit more (batches of
  // short candidates), more segments only lengthen the ragged end of a batch
  const int plain_groups = std::max(p->slot_grid / std::max(p->n_cu, 1), 1);
  if (geo.waves * geo.groups > p->slot_waves * plain_groups &&
      4ll * (ST.n_shared_ints + (int64_t)p->slot_waves * geo.wave_ints) + 256 <= p->max_lds / plain_groups) {
    geo.waves = p->slot_waves;
    geo.groups = plain_groups;
  }
  // a table image (the plain one, or the timing pass's) with longer dev rows:
  // [.. 2 + 4V ints as before ..][4V out-edges]
  const int dev_ints = ST.dev_ints + 4 * V;
  auto with_links = [&](const std::vector<int32_t>& base) {
  std::vector<int32_t> J((size_t)ST.n_shared_ints + (size_t)lpc * dev_ints + (size_t)lpc * ST.state_words, 0);
  std::copy(base.begin(), base.begin() + ST.n_shared_ints, J.begin());
  for (int d = 0; d < lpc; ++d) {
    int32_t* row = &J[(size_t)ST.n_shared_ints + (size_t)d * dev_ints];
    std::copy(base.begin() + ST.off_dev + (size_t)d * ST.dev_ints,
              base.begin() + ST.off_dev + (size_t)(d + 1) * ST.dev_ints, row);
    for (int i = 0; i < 4 * V; ++i) row[ST.dev_ints + i] = (int32_t)spare;
    if (d >= D) continue;
    for (int c = 0; c < p->n_chunks[d]; ++c) {
      const int s = p->local_stage[(size_t)d * kMaxChunks + c];
      for (int fwd = 0; fwd < 2; ++fwd)
        for (int k = 0; k < 2; ++k) {
          OutEdge e;
          if (!out_edge(s, fwd != 0, k, &e) || e.to == d) continue;
          // first forward / first backward / second forward / second backward
          row[ST.dev_ints + (2 * k + (fwd ? 0 : 1)) * V + c] =
              (int32_t)(((uint32_t)e.comm << 16) | (uint32_t)link_of(d, e.to) * 256u);
        }
    }
  }
  std::copy(base.begin() + ST.off_expect, base.end(), J.begin() + ST.n_shared_ints + (size_t)lpc * dev_ints);
  return J;
  };
  const std::vector<int32_t> J = with_links(p->slot_ints);
  DeviceGuard g(p->device_id);
  if (!g.ok) return FPSCHED_EHIP;
  int32_t* image = nullptr;
  if (hipMalloc(&image, J.size() * sizeof(int32_t)) != hipSuccess) return FPSCHED_ENOMEM;
  const SlotKernel kernel = slot_kernel_of<kSlotLinks>(p->slot_v, p->slot_deg2, ST.n_classes == 1);
  const int32_t lds_bytes = (int32_t)(4ll * (ST.n_shared_ints + (int64_t)geo.waves * geo.wave_ints));
  if (hipMemcpy(image, J.data(), J.size() * sizeof(int32_t), hipMemcpyHostToDevice) != hipSuccess ||
      hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, p->max_lds) != hipSuccess) {
    (void)hipFree(image);
    return FPSCHED_EHIP;
  }
  p->d_links_image = image;
  p->stab_links = ST;
  p->stab_links.ints = image;
  p->stab_links.link_words = link_words;
  p->stab_links.slots_per_cand = slots_per_cand;
  p->stab_links.dev_ints = dev_ints;
  p->stab_links.off_expect = ST.n_shared_ints + lpc * dev_ints;
  p->stab_links.cands_per_wave = geo.cands_per_wave;
  p->stab_links.wave_ints = geo.wave_ints;
  p->links_waves = geo.waves;
  p->links_grid = p->n_cu * geo.groups;
  p->links_lds_bytes = lds_bytes;
  p->link_words = link_words;
  p->link_rows.assign((size_t)lpc * 4 * V, 0);
  for (int d = 0; d < lpc; ++d)
    std::copy(J.begin() + ST.n_shared_ints + (size_t)d * dev_ints + ST.dev_ints,
              J.begin() + ST.n_shared_ints + (size_t)(d + 1) * dev_ints, p->link_rows.begin() + (size_t)d * 4 * V);
  // the sliding pass's timing kernel under the link model: the timing image, widened the same way; it
  // needs 16 bytes of LDS more
  if (p->slide_ok && !p->times_ints.empty() && (int64_t)lds_bytes + 16 <= p->max_lds / geo.groups) {
    const std::vector<int32_t> JT = with_links(p->times_ints);
    int32_t* timg = nullptr;
    if (hipMalloc(&timg, JT.size() * sizeof(int32_t)) == hipSuccess &&
        hipMemcpy(timg, JT.data(), JT.size() * sizeof(int32_t), hipMemcpyHostToDevice) == hipSuccess &&
        hipFuncSetAttribute(reinterpret_cast<const void*>(slot_kernel_of<kSlotTimesLinks>(p->slot_v, p->slot_deg2, ST.n_classes == 1)),
                            hipFuncAttributeMaxDynamicSharedMemorySize, p->max_lds) == hipSuccess) {
      p->d_times_links_image = timg;
      p->stab_times_links = p->stab_links;
      p->stab_times_links.ints = timg;
      p->links_slide_ok = true;
      // the one-kernel form of the pass under the link model: the same image with the W items' costs behind it
      if (p->slide_eval_ok && !p->slide_w_table.empty()) {
        std::vector<int32_t> JS = JT;
        JS.insert(JS.end(), p->slide_w_table.begin(), p->slide_w_table.end());
        int32_t* simg = nullptr;
        if (hipMalloc(&simg, JS.size() * sizeof(int32_t)) == hipSuccess &&
            hipMemcpy(simg, JS.data(), JS.size() * sizeof(int32_t), hipMemcpyHostToDevice) == hipSuccess &&
            hipFuncSetAttribute(reinterpret_cast<const void*>(slot_kernel_of<kSlotSlideLinks>(p->slot_v, p->slot_deg2, ST.n_classes == 1)),
                                hipFuncAttributeMaxDynamicSharedMemorySize, p->max_lds) == hipSuccess) {
          p->d_slide_links_image = simg;
          p->stab_slide_links = p->stab_links;
          p->stab_slide_links.ints = simg;
          p->stab_slide_links.off_w = (int32_t)JT.size();
          p->links_slide_eval_ok = true;
        } else {
          (void)hipGetLastError();
          if (simg) (void)hipFree(simg);
        }
      }
    } else {
      (void)hipGetLastError();
      if (timg) (void)hipFree(timg);
    }
  }
  if (p->mb_set) {   // both variants (the link tables stay built whatever comes of it)
    const int rc = build_combined_tables(p);
    if (rc != FPSCHED_OK) return rc;
  }
  p->links_on = true;
  if (getenv("FPSCHED_VERBOSE"))
    fprintf(stderr, "[fpsched] link occupancy: %d link words per lane, %d x %d wavefronts per compute unit (plain: %d x %d)\n",
            link_words, geo.groups, geo.waves, p->slot_grid / std::max(p->n_cu, 1), p->slot_waves);
  return FPSCHED_OK;
}

// The table image and workgroup shape of eval_sync_kernel for one setting of the handle: groups and pairs
// (fpsched_problem_set_sync) or the copy-engine form (fpsched_problem_set_copy_engine, copy_depth > 0).
// On success the handle's table is replaced; on failure the handle is back on the plain model.
static int install_table_model(fpsched_problem* p, const std::vector<int32_t>& grp, const std::vector<int32_t>& items,
                               int32_t n_pairs, const fpsched_dependency* pairs, bool wants_w, int copy_depth) {
  const int D = p->D, S = p->S, m = p->m;
  const std::vector<int32_t>& I = p->host_ints;
  const DevTables& T = p->tables;
  std::vector<int32_t> J;
  SyncTables ST{};
  ST.D = D; ST.S = S; ST.m = m; ST.has_w = p->has_w;
  ST.lanes_per_cand = T.lanes_per_cand;
  ST.n_fin_tables = wants_w ? 3 : 2;
  ST.copy_depth = copy_depth;
  auto append = [&](const int32_t* src, size_t n) { const int32_t off = (int32_t)J.size(); J.insert(J.end(), src, src + n); return off; };
  ST.off_dur = append(&I[T.off_dur], (size_t)kNKinds * S);
  ST.off_mem_units = append(&I[T.off_mem_units], S);
  ST.off_group = append(grp.data(), S);
  ST.off_items = append(items.data(), S);
  // one dependency list per (kind, stage): the edges of the stage DAG, then the pairs
  std::vector<int32_t> dep_off((size_t)kNKinds * S + 1, 0), dep;
  for (int kind = 0; kind < kNKinds; ++kind)
    for (int s = 0; s < S; ++s) {
      dep_off[(size_t)kind * S + s] = (int32_t)(dep.size() / 3);
      if (kind == kF || kind == kFD)
        for (int e = I[T.off_pred_off + s]; e < I[T.off_pred_off + s + 1]; ++e) {
          dep.push_back(0); dep.push_back(I[T.off_pred_stage + e]); dep.push_back(I[T.off_pred_comm + e]);
        }
      if (kind == kB)
        for (int e = I[T.off_succ_off + s]; e < I[T.off_succ_off + s + 1]; ++e) {
          dep.push_back(1); dep.push_back(I[T.off_succ_stage + e]); dep.push_back(I[T.off_succ_comm + e]);
        }
      for (int i = 0; i < n_pairs; ++i) {
        const fpsched_dependency& q = pairs[i];
        if (q.stage_to != s || !(q.kind_to == kind || (q.kind_to == FPSCHED_F && kind == kFD))) continue;
        dep.push_back(q.kind_from == FPSCHED_F ? 0 : (q.kind_from == FPSCHED_B ? 1 : 2));
        dep.push_back(q.stage_from);
        dep.push_back(p->stage_device[q.stage_from] != p->stage_device[s] ? q.latency : 0);
      }
    }
  dep_off[(size_t)kNKinds * S] = (int32_t)(dep.size() / 3);
  ST.off_dep_off = append(dep_off.data(), dep_off.size());
  ST.off_dep = append(dep.data(), dep.size());
  ST.off_local_stage = append(p->local_stage.data(), (size_t)D * kMaxChunks);
  ST.off_n_chunks = append(p->n_chunks.data(), D);
  ST.off_mem_cap = append(&I[T.off_mem_cap], D);
  ST.n_table_ints = (int32_t)J.size();
  // candidates per wavefront: whole finish-time tables (and reload times) and state bytes of each in LDS;
  // the copy-engine form adds three rings of eight dwords per lane
  const int64_t SM = (int64_t)S * m;
  const int64_t per_cand = 4 * ((ST.n_fin_tables + (copy_depth > 0 ? 1 : 0)) * SM + ((SM + 3) >> 2));
  const int64_t fixed_bytes = 4ll * ST.n_table_ints + (copy_depth > 0 ? 3 * 8 * 64 * 4 : 0);
  int cpw = 64 / ST.lanes_per_cand;
  while (cpw > 1 && fixed_bytes + cpw * per_cand > p->max_lds) cpw >>= 1;
  if (fixed_bytes + cpw * per_cand > p->max_lds) return FPSCHED_EUNSUPPORTED;
  ST.cands_per_wave = cpw;
  DeviceGuard g(p->device_id);
  if (!g.ok) return FPSCHED_EHIP;
  if (hipDeviceSynchronize() != hipSuccess) return FPSCHED_EHIP;   // an earlier table may be in use
  auto back_to_plain = [&]() {
    p->sync_on = false;
    p->copy_depth = 0;
    p->sync_items.assign(S, m);
  };
  if (J.size() > p->sync_ints_capacity) {
    int32_t* fresh = nullptr;
    if (hipMalloc(&fresh, J.size() * sizeof(int32_t)) != hipSuccess) { (void)hipGetLastError(); return FPSCHED_ENOMEM; }
    if (p->d_sync_ints) (void)hipFree(p->d_sync_ints);
    p->d_sync_ints = fresh;
    p->sync_ints_capacity = J.size();
    back_to_plain();   // the table the handle ran on is gone
  }
  if (hipMemcpy(p->d_sync_ints, J.data(), J.size() * sizeof(int32_t), hipMemcpyHostToDevice) != hipSuccess ||
      hipFuncSetAttribute(reinterpret_cast<const void*>(&eval_sync_kernel<false>), hipFuncAttributeMaxDynamicSharedMemorySize,
                          p->max_lds) != hipSuccess ||
      hipFuncSetAttribute(reinterpret_cast<const void*>(&eval_sync_kernel<true>), hipFuncAttributeMaxDynamicSharedMemorySize,
                          p->max_lds) != hipSuccess) {
    back_to_plain();
    return FPSCHED_EHIP;
  }
  ST.ints = p->d_sync_ints;
  p->sync_tab = ST;
  p->sync_lds_bytes = (int32_t)(fixed_bytes + cpw * per_cand);
  return FPSCHED_OK;
}

// The slot kernel's form of the synchronisation model (mode kSlotSync): possible when every dependency pair runs
// forward-to-forward or backward-to-backward, no stage has more than two inputs or outputs in either direction
// (pairs included), and the neighbours of a stage with more than one micro-batch per item all have one.  The
// table image has the plain layout; a pair is an edge of a slot class of its own that exists in one direction.
// Leaves p->sync_slots_ok false when the setting does not fit.
static void build_sync_slot_tables(fpsched_problem* p, const std::vector<int32_t>& grp, const std::vector<int32_t>& items,
                                   int32_t n_pairs, const fpsched_dependency* pairs, int64_t max_lat) {
  p->sync_slots_ok = false;
  if (!p->slots_ok) return;   // (units, stage count and word format were checked for the plain tables)
  const int D = p->D, S = p->S, m = p->m;
  const std::vector<int32_t>& I = p->host_ints;
  const DevTables& T = p->tables;
  if ((int64_t)D * p->max_stride * (p->max_dur + max_lat) >= (1ll << 24) || max_lat >= (1ll << 16)) return;
  struct In { int from, lat, cls; };
  std::vector<std::vector<In>> fwd_in(S), bwd_in(S);
  std::vector<std::vector<int>> fwd_out(S), bwd_out(S), partners(S);
  // classes of the DAG's edges: chains, as for the plain tables
  std::vector<std::vector<int>> out_cls(S);
  int n_classes = 0;
  {
    std::vector<int> indeg(S, 0), order;
    std::vector<std::vector<int>> arriving(S);
    for (int s = 0; s < S; ++s) indeg[s] = I[T.off_pred_off + s + 1] - I[T.off_pred_off + s];
    for (int s = 0; s < S; ++s) if (!indeg[s]) order.push_back(s);
    for (size_t i = 0; i < order.size(); ++i) {
      const int s = order[i];
      size_t used = 0;
      for (int e = I[T.off_succ_off + s]; e < I[T.off_succ_off + s + 1]; ++e) {
        const int v = I[T.off_succ_stage + e], lat = I[T.off_succ_comm + e];
        const int cls = used < arriving[s].size() ? arriving[s][used++] : n_classes++;
        arriving[v].push_back(cls);
        fwd_out[s].push_back(cls); fwd_in[v].push_back(In{s, lat, cls});
        bwd_in[s].push_back(In{v, lat, cls}); bwd_out[v].push_back(cls);
        partners[s].push_back(v); partners[v].push_back(s);
        if (--indeg[v] == 0) order.push_back(v);
      }
    }
  }
  for (int i = 0; i < n_pairs; ++i) {
    const fpsched_dependency& q = pairs[i];
    const int a = q.stage_from, b = q.stage_to;
    const int lat = p->stage_device[a] != p->stage_device[b] ? q.latency : 0;
    const int cls = n_classes++;
    if (q.kind_from == FPSCHED_F && q.kind_to == FPSCHED_F) {
      fwd_out[a].push_back(cls); fwd_in[b].push_back(In{a, lat, cls});
    } else if (q.kind_from == FPSCHED_B && q.kind_to == FPSCHED_B) {
      bwd_out[a].push_back(cls); bwd_in[b].push_back(In{a, lat, cls});
    } else {
      return;   // a pair the mail slots cannot carry
    }
    partners[a].push_back(b); partners[b].push_back(a);
  }
  if (n_classes == 0) n_classes = 1;
  bool deg2 = false;
  for (int s = 0; s < S; ++s) {
    const size_t most = std::max({fwd_in[s].size(), fwd_out[s].size(), bwd_in[s].size(), bwd_out[s].size()});
    if (most > 2) return;
    if (most > 1) deg2 = true;
    if (grp[s] > 1)
      for (int t : partners[s]) if (grp[t] != 1) return;
  }
  const int V = p->slot_v, lpc = T.lanes_per_cand;
  const int slot_stride = ((2 * n_classes + 1) * m + 7) & ~7;
  if (4ll * slot_stride > 0xffff) return;
  const int64_t unit_scale = p->stab.unit_scale;
  const int n_meta = kNKinds * kMaxChunks * lpc * 4;
  const int n_meta2 = deg2 ? (2 * kMaxChunks + 1) * lpc * 2 : 0;
  const int n_shared = (n_meta + n_meta2 + 511) & ~511;
  const unsigned dump_bytes = (unsigned)(2 * n_classes * m) * 4u;
  const int dev_ints = 2 + 5 * V;
  const int words_per_chunk = (m + 7) / 8;
  const int state_words = V * words_per_chunk;
  std::vector<int32_t> J((size_t)n_shared + (size_t)lpc * dev_ints + (size_t)lpc * state_words, 0);
  static const int need_of[kNKinds] = {15, kAbsent, kRes, kBDone, kDisc, kRes, kOff, kAbsent};
  static const int next_of[kNKinds] = {0, kRes, kBDone, kDone, kRes, kOff, kRes, kDisc};
  auto fwd_slot = [&](int cls) { return (unsigned)((n_classes + cls) * m) * 4u; };
  auto bwd_slot = [&](int cls) { return (unsigned)(cls * m) * 4u; };
  for (int kind = 0; kind < kNKinds; ++kind)
    for (int c = 0; c < kMaxChunks; ++c)
      for (int d = 0; d < lpc; ++d) {
        int32_t* e = &J[(((size_t)kind * kMaxChunks + c) * lpc + d) * 4];
        e[2] = (int32_t)(15u | (dump_bytes << 16));
        if (d >= D || c >= p->n_chunks[d] || kind == kEnd || (kind == kW && !p->has_w)) continue;
        const int st = p->local_stage[(size_t)d * kMaxChunks + c];
        const unsigned units = (unsigned)(I[T.off_mem_units + st] / unit_scale);
        const bool allocs = kind == kF || kind == kFD || kind == kR || kind == kL;
        const bool frees = kind == kFD || kind == kO || kind == (p->has_w ? kW : kB);
        unsigned has_in = 0, tag = 0, prod = dump_bytes, comm = 0;
        if (kind == kF || kind == kFD) {
          if (!fwd_in[st].empty()) { has_in = 0xffu; tag = (unsigned)fwd_in[st][0].from; comm = (unsigned)fwd_in[st][0].lat; }
          if (!fwd_out[st].empty()) prod = fwd_slot(fwd_out[st][0]);
        } else if (kind == kB) {
          if (!bwd_in[st].empty()) { has_in = 0xffu; tag = (unsigned)bwd_in[st][0].from; comm = (unsigned)bwd_in[st][0].lat; }
          if (!bwd_out[st].empty()) prod = bwd_slot(bwd_out[st][0]);
        }
        e[0] = (int32_t)((unsigned)I[T.off_dur + kind * S + st] << 8);
        e[1] = (int32_t)((comm << 8) - tag);
        e[2] = (int32_t)((unsigned)need_of[kind] | ((unsigned)(need_of[kind] ^ next_of[kind]) << 8) | (prod << 16));
        e[3] = (int32_t)((allocs ? units : 0u) | ((frees ? units : 0u) << 8) | ((unsigned)st << 16) | (has_in << 24));
      }
  for (int dir = 0; dir < 2 && deg2; ++dir)
    for (int c = 0; c < kMaxChunks; ++c)
      for (int d = 0; d < D; ++d) {
        if (c >= p->n_chunks[d]) continue;
        const int st = p->local_stage[(size_t)d * kMaxChunks + c];
        int32_t* e = &J[(size_t)n_meta + (((size_t)dir * kMaxChunks + c) * lpc + d) * 2];
        const std::vector<In>& in = dir == 0 ? fwd_in[st] : bwd_in[st];
        const std::vector<int>& out = dir == 0 ? fwd_out[st] : bwd_out[st];
        unsigned y = 0;
        if (in.size() > 1) { y |= kMetaHasCons; e[0] = (int32_t)(((unsigned)in[1].lat << 8) - (unsigned)in[1].from); }
        if (out.size() > 1) y |= kMetaHasProd | (dir == 0 ? fwd_slot(out[1]) : bwd_slot(out[1]));
        e[1] = (int32_t)y;
      }
  for (int d = 0; d < D; ++d) {
    // state words of device d once every item placed on it is consumed
    int32_t* x = &J[(size_t)n_shared + (size_t)lpc * dev_ints + (size_t)d * state_words];
    const unsigned terminal = p->has_w ? kDone : kBDone;
    for (int c = 0; c < p->n_chunks[d]; ++c) {
      const int st = p->local_stage[(size_t)d * kMaxChunks + c];
      for (int g = 0; g < items[st]; ++g) x[c * words_per_chunk + (g >> 3)] |= (int32_t)(terminal << ((g & 7) * 4));
    }
    int32_t* e = &J[(size_t)n_shared + (size_t)d * dev_ints];
    e[0] = p->n_chunks[d];
    e[1] = (int32_t)(I[T.off_mem_cap + d] / unit_scale);
    for (int c = 0; c < p->n_chunks[d]; ++c) {
      const int st = p->local_stage[(size_t)d * kMaxChunks + c];
      e[2 + c] = !fwd_in[st].empty() ? (n_classes + fwd_in[st][0].cls) * m : 0;
      e[2 + V + c] = !bwd_in[st].empty() ? bwd_in[st][0].cls * m : 0;
      e[2 + 2 * V + c] = fwd_in[st].size() > 1 ? (n_classes + fwd_in[st][1].cls) * m : 0;
      e[2 + 3 * V + c] = bwd_in[st].size() > 1 ? bwd_in[st][1].cls * m : 0;
      e[2 + 4 * V + c] = grp[st] | (items[st] << 16);
    }
    for (int c = p->n_chunks[d]; c < V; ++c) e[2 + 4 * V + c] = 1;   // (no such chunk: no item is valid)
  }
  SlotTables ST = p->stab;
  ST.n_classes = n_classes;
  ST.slots_per_cand = slot_stride;
  ST.state_words = state_words;
  ST.n_shared_ints = n_shared;
  ST.off_meta2 = n_meta;
  ST.off_dev = n_shared;
  ST.dev_ints = dev_ints;
  ST.off_expect = n_shared + lpc * dev_ints;
  ST.off_mb = 0; ST.link_words = 0; ST.mb_kind_map = 0; ST.copy_depth = 0;
  const SlotGeometry geo = slot_geometry(n_shared, lpc, state_words, slot_stride, p->max_lds);
  if (geo.waves < 1) return;
  ST.cands_per_wave = geo.cands_per_wave;
  ST.wave_ints = geo.wave_ints;
  DeviceGuard g(p->device_id);
  if (!g.ok) return;
  if (J.size() > p->sync_slot_image_ints) {
    if (p->d_sync_slot_image) (void)hipFree(p->d_sync_slot_image);
    p->d_sync_slot_image = nullptr;
    p->sync_slot_image_ints = 0;
    if (hipMalloc(&p->d_sync_slot_image, J.size() * sizeof(int32_t)) != hipSuccess) { (void)hipGetLastError(); p->d_sync_slot_image = nullptr; return; }
    p->sync_slot_image_ints = J.size();
  }
  if (hipMemcpy(p->d_sync_slot_image, J.data(), J.size() * sizeof(int32_t), hipMemcpyHostToDevice) != hipSuccess ||
      hipFuncSetAttribute(reinterpret_cast<const void*>(slot_kernel_of<kSlotSync>(V, deg2, n_classes == 1)),
                          hipFuncAttributeMaxDynamicSharedMemorySize, p->max_lds) != hipSuccess) {
    (void)hipGetLastError();
    return;
  }
  ST.ints = p->d_sync_slot_image;
  p->stab_sync = ST;
  p->sync_deg2 = deg2;
  p->sync_slot_waves = geo.waves;
  p->sync_slot_grid = p->n_cu * geo.groups;
  p->sync_slot_lds_bytes = (int32_t)(4ll * (n_shared + (int64_t)geo.waves * geo.wave_ints));
  p->sync_slots_ok = true;
}

int fpsched_problem_set_sync(fpsched_problem* p, const int32_t* group, int32_t n_pairs,
                             const fpsched_dependency* pairs) {
  if (!p || n_pairs < 0 || (n_pairs > 0 && !pairs)) return FPSCHED_EINVAL;
  const int D = p->D, S = p->S, m = p->m;
  bool trivial = n_pairs == 0;
  for (int s = 0; s < S && group; ++s) {
    if (group[s] < 1) return FPSCHED_EINVAL;
    if (group[s] != 1) trivial = false;
  }
  if (trivial) {   // back to the plain model; the table stays allocated for the next call
    if (p->sync_on) p->sync_items.assign(S, m);
    p->sync_on = false;
    return FPSCHED_OK;
  }
  if (p->mb_set || p->links_on || p->copy_depth > 0) return FPSCHED_EUNSUPPORTED;
  int64_t max_lat = p->max_comm;
  bool wants_w = false;
  for (int i = 0; i < n_pairs; ++i) {
    const fpsched_dependency& q = pairs[i];
    if (q.kind_from != FPSCHED_F && q.kind_from != FPSCHED_B && q.kind_from != FPSCHED_W) return FPSCHED_EINVAL;
    if (q.kind_to <= FPSCHED_END || q.kind_to >= FPSCHED_NKINDS) return FPSCHED_EINVAL;
    if ((q.kind_from == FPSCHED_W || q.kind_to == FPSCHED_W) && !p->has_w) return FPSCHED_EINVAL;
    if (q.stage_from < 0 || q.stage_from >= S || q.stage_to < 0 || q.stage_to >= S || q.latency < 0) return FPSCHED_EINVAL;
    if (q.stage_from == q.stage_to && (q.kind_from == q.kind_to || (q.kind_from == FPSCHED_F && q.kind_to == FPSCHED_FD)))
      return FPSCHED_EINVAL;
    max_lat = std::max<int64_t>(max_lat, q.latency);
    wants_w = wants_w || q.kind_from == FPSCHED_W;
  }
  if ((int64_t)D * p->max_stride * (p->max_dur + max_lat) >= (int64_t)1 << 31) return FPSCHED_EOVERFLOW;
  std::vector<int32_t> grp(S, 1), items(S, m);
  for (int s = 0; s < S; ++s) {
    grp[s] = group ? std::min(group[s], m) : 1;
    items[s] = (m + grp[s] - 1) / grp[s];
  }
  if (p->device_id >= 0) {
    const int rc = install_table_model(p, grp, items, n_pairs, pairs, wants_w, 0);
    if (rc != FPSCHED_OK) return rc;
    build_sync_slot_tables(p, grp, items, n_pairs, pairs, max_lat);
  }
  p->sync_items = items;
  p->sync_on = true;
  return FPSCHED_OK;
}

int fpsched_problem_set_copy_engine(fpsched_problem* p, int32_t depth) {
  if (!p || depth < 0 || depth > FPSCHED_MAX_COPY_DEPTH) return FPSCHED_EINVAL;
  if (depth == 0) {
    p->copy_depth = 0;
    return FPSCHED_OK;
  }
  if (p->mb_set || p->links_on || p->sync_on) return FPSCHED_EUNSUPPORTED;
  // a transfer takes time: with a cost of zero any number of them could end at one instant
  const std::vector<int32_t>& I = p->host_ints;
  for (int s = 0; s < p->S; ++s)
    if (I[p->tables.off_dur + kO * p->S + s] < 1 || I[p->tables.off_dur + kL * p->S + s] < 1) return FPSCHED_EINVAL;
  if (p->device_id >= 0) {
    const std::vector<int32_t> grp(p->S, 1), items(p->S, p->m);
    const int rc = install_table_model(p, grp, items, 0, nullptr, false, depth);
    if (rc != FPSCHED_OK) return rc;
    // the slot kernel has a form of this model too: the plain tables, 32 more dwords of LDS per lane for
    // the rings of the copy timeline
    p->copy_slots_ok = false;
    if (p->slots_ok) {
      const SlotTables& PT = p->stab;
      const SlotGeometry geo = slot_geometry(PT.n_shared_ints, PT.lanes_per_cand, PT.state_words + kSlotCopyWords,
                                             PT.slots_per_cand, p->max_lds, PT.cands_per_wave);
      DeviceGuard g(p->device_id);
      if (g.ok && geo.waves >= 1 && geo.cands_per_wave == PT.cands_per_wave &&
          hipFuncSetAttribute(reinterpret_cast<const void*>(slot_kernel_of<kSlotCopy>(p->slot_v, p->slot_deg2, PT.n_classes == 1)),
                              hipFuncAttributeMaxDynamicSharedMemorySize, p->max_lds) == hipSuccess) {
        p->stab_copy = PT;
        p->stab_copy.link_words = kSlotCopyWords;
        p->stab_copy.copy_depth = depth;
        p->stab_copy.wave_ints = geo.wave_ints;
        p->copy_waves = geo.waves;
        p->copy_grid = p->n_cu * geo.groups;
        p->copy_lds_bytes = (int32_t)(4ll * (PT.n_shared_ints + (int64_t)geo.waves * geo.wave_ints));
        p->copy_slots_ok = true;
      }
    }
  }
  p->copy_depth = depth;
  return FPSCHED_OK;
}

using GenKernel = void (*)(DevTables, const int32_t*, const int32_t*, const long long*, long long, long long, int, uint16_t*,
                           int32_t*, unsigned char*, unsigned long long*, GenResults);
static int gen_waves_per_cu() {
  // tuning knob: FPSCHED_GEN_WAVES = resident wavefronts per compute unit
  int waves_per_cu = 24;
  if (const char* env = getenv("FPSCHED_GEN_WAVES")) {
    const int v = atoi(env);
    if (v >= 1 && v <= 32) waves_per_cu = v;
  }
  return waves_per_cu;
}
static int gen_max_chunks(const fpsched_problem* p) {
  int max_chunks = 0;
  for (int d = 0; d < p->D; ++d) max_chunks = std::max(max_chunks, p->n_chunks[d]);
  return max_chunks;
}

static int run_generate(const fpsched_problem* p, const fpsched_actor_policy* d_policy, const int32_t* d_inflight,
                 const int64_t* d_select, int64_t n_src, int64_t n_sets, int32_t stride_words, uint16_t* d_ops, int32_t* d_steps,
                 uint8_t* d_status, void* d_workspace, size_t workspace_bytes, void* hip_stream) {
  if (!p || n_sets < 0) return FPSCHED_EINVAL;
  if (p->device_id < 0) return FPSCHED_ENODEV;
  if (n_sets == 0) return FPSCHED_OK;
  if (!d_policy || !d_inflight || !d_ops || !d_steps || !d_status) return FPSCHED_EINVAL;
  if (p->sync_on) return FPSCHED_EUNSUPPORTED;   // the generator schedules one item per micro-batch
  const int max_chunks = gen_max_chunks(p);
  const int64_t longest = (int64_t)max_chunks * p->m * (p->has_w ? 3 : 2);
  if (stride_words < 8 || (stride_words & 7) || stride_words < longest) return FPSCHED_EINVAL;
  if (reinterpret_cast<uintptr_t>(d_ops) & 15) return FPSCHED_EINVAL;
  // the first 8 bytes of the workspace hold the counter the segments draw parameter sets from
  if (!d_workspace || (reinterpret_cast<uintptr_t>(d_workspace) & 15)) return FPSCHED_EINVAL;
  if (workspace_bytes < 256) return FPSCHED_ENOMEM;
  const int lpc = p->tables.lanes_per_cand;
  const int cpw = 64 / lpc;
  const int deg = p->max_degree <= 1 ? 1 : (p->max_degree == 2 ? 2 : 0);
  // tables (if walked), counters and the constant words (a multiple of four), 8 staging dwords per lane
  const int64_t lds_bytes = 4ll * ((deg == 0 ? p->tables.n_table_ints : 0) +
                                   (((int64_t)cpw * 3 * p->S + 2 * p->S + 1 + 3) & ~3ll) + 8 * 64);
  if (lds_bytes > p->max_lds) return FPSCHED_EUNSUPPORTED;
  // persistent grid: as many single-wavefront workgroups as stay resident
  const int64_t blocks = std::min<int64_t>((n_sets + cpw - 1) / cpw, (int64_t)p->n_cu * gen_waves_per_cu());
  DeviceGuard g(p->device_id);
  if (!g.ok) return FPSCHED_EHIP;
  const int V = max_chunks <= 1 ? 1 : (max_chunks <= 2 ? 2 : 4);
  static const GenKernel table[3][3] = {
      {&generate_kernel<1, 0, kGenPlain>, &generate_kernel<1, 1, kGenPlain>, &generate_kernel<1, 2, kGenPlain>},
      {&generate_kernel<2, 0, kGenPlain>, &generate_kernel<2, 1, kGenPlain>, &generate_kernel<2, 2, kGenPlain>},
      {&generate_kernel<4, 0, kGenPlain>, &generate_kernel<4, 1, kGenPlain>, &generate_kernel<4, 2, kGenPlain>}};
  const GenKernel kernel = table[V == 1 ? 0 : (V == 2 ? 1 : 2)][deg];
  if (lds_bytes > 64 * 1024 &&
      hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                          p->max_lds) != hipSuccess)
    return FPSCHED_EHIP;
  unsigned long long* counter = static_cast<unsigned long long*>(d_workspace);
  // segment g starts on set g; the counter hands out the sets after those
  hipLaunchKernelGGL(reset_counter_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(hip_stream), counter,
                     (unsigned long long)(blocks * cpw));
  hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(64), (size_t)lds_bytes,
                     static_cast<hipStream_t>(hip_stream), p->tables, reinterpret_cast<const int32_t*>(d_policy),
                     d_inflight, reinterpret_cast<const long long*>(d_select), (long long)n_src, (long long)n_sets, (int)stride_words,
                     d_ops, d_steps, d_status, counter, GenResults{nullptr, nullptr, nullptr, nullptr});
  return check_hip(hipGetLastError());
}

int fpsched_generate(const fpsched_problem* p, const fpsched_actor_policy* d_policy, const int32_t* d_inflight,
                     int64_t n_sets, int32_t stride_words, uint16_t* d_ops, int32_t* d_steps, uint8_t* d_status,
                     void* d_workspace, size_t workspace_bytes, void* hip_stream) {
  return run_generate(p, d_policy, d_inflight, nullptr, n_sets, n_sets, stride_words, d_ops, d_steps, d_status, d_workspace,
                      workspace_bytes, hip_stream);
}

int fpsched_generate_selected(const fpsched_problem* p, const fpsched_actor_policy* d_policy,
                              const int32_t* d_inflight, int64_t n_sets, const int64_t* d_select, int64_t n_selected,
                              int32_t stride_words, uint16_t* d_ops, int32_t* d_steps, uint8_t* d_status,
                              void* d_workspace, size_t workspace_bytes, void* hip_stream) {
  if (n_sets < 0 || (n_selected > 0 && !d_select)) return FPSCHED_EINVAL;
  return run_generate(p, d_policy, d_inflight, d_select, n_sets, n_selected, stride_words, d_ops, d_steps, d_status,
                      d_workspace, workspace_bytes, hip_stream);
}

// generator and evaluator in one kernel; slide: with the weight-gradient sliding pass in it
static int run_generate_evaluate(const fpsched_problem* p, const fpsched_actor_policy* d_policy,
                                 const int32_t* d_inflight, int64_t n_sets, fpsched_results out, int32_t* d_steps,
                                 uint8_t* d_status, void* d_workspace, size_t workspace_bytes, void* hip_stream,
                                 bool slide) {
  if (!p || n_sets < 0) return FPSCHED_EINVAL;
  if (p->device_id < 0) return FPSCHED_ENODEV;
  if (slide && !p->has_w) return FPSCHED_EINVAL;
  if (n_sets == 0) return FPSCHED_OK;
  if (!d_policy || !d_inflight || !d_steps || !d_status || !out.makespan || !out.idle || !out.peak || !out.flags)
    return FPSCHED_EINVAL;
  // the plain cost model only: one cost per (type, stage), transfers as latencies
  if (p->sync_on || p->copy_depth > 0 || p->mb_set || p->links_on) return FPSCHED_EUNSUPPORTED;
  if (p->tables.off_gen_rows < 0) return FPSCHED_EUNSUPPORTED;
  if (!d_workspace || (reinterpret_cast<uintptr_t>(d_workspace) & 15)) return FPSCHED_EINVAL;
  if (workspace_bytes < 256) return FPSCHED_ENOMEM;
  // finish times stay below 2^30: every item starts at most (items before it) * (largest cost + latency) late
  if (3ll * p->S * p->m * (p->max_dur + p->max_comm) >= (1ll << 30)) return FPSCHED_EOVERFLOW;
  const int lpc = p->tables.lanes_per_cand;
  const int cpw = 64 / lpc;
  const int V = p->tables.gen_row_chunks;
  // cost rows shared by the workgroup; per wavefront its counters and its sets' slots
  const int64_t shared_ints = 3ll * V * p->D * 8;
  // (slide: a ring of queue words per lane for stashes deeper than two words: one bit per entry at two stages per
  // device, two at four, none at one; a power of two that holds every W item of a device)
  DevTables tables = p->tables;
  tables.gen_spill_words = 0;
  if (slide) {
    const int64_t bits = V == 1 ? 0 : (V == 2 ? 1 : 2);
    int words = 1;
    while ((int64_t)words * 32 < (int64_t)V * p->m * bits + 32) words <<= 1;
    tables.gen_spill_words = words;
  }
  const int64_t wave_ints = (((int64_t)cpw * 3 * p->S + 2 * p->S + 1 + 3) & ~3ll) + (int64_t)cpw * p->tables.gen_slot_words +
                            64ll * tables.gen_spill_words;
  const int64_t lds_ints = p->max_lds / 4;
  if (shared_ints + wave_ints > lds_ints) return FPSCHED_EUNSUPPORTED;
  // wavefronts per workgroup and workgroups per compute unit: as many resident wavefronts as asked for
  // and as LDS holds, in as few workgroups as possible (each keeps a copy of the rows)
  const int want = gen_waves_per_cu();
  int best_waves = 1, best_groups = 1;
  for (int groups = 1; groups <= 8; ++groups) {
    int wv = (int)std::min<int64_t>((lds_ints / groups - shared_ints - 64) / wave_ints, kGenTimedThreads / 64);
    wv = std::min(wv, (want + groups - 1) / groups);
    if (wv >= 1 && wv * groups > best_waves * best_groups) { best_waves = wv; best_groups = groups; }
  }
  const int64_t segments = (n_sets + cpw - 1) / cpw;
  // (a small batch is spread over the compute units: fewer wavefronts per workgroup)
  const int64_t grid = (int64_t)p->n_cu * best_groups;
  best_waves = (int)std::clamp<int64_t>((segments + grid - 1) / grid, 1, best_waves);
  const int64_t blocks = std::min<int64_t>((segments + best_waves - 1) / best_waves, grid);
  const int64_t lds_bytes = 4 * (shared_ints + best_waves * wave_ints);
  DeviceGuard g(p->device_id);
  if (!g.ok) return FPSCHED_EHIP;
  const int deg = p->max_degree <= 1 ? 1 : 2;
  static const GenKernel table[2][3][2] = {
      {{&generate_kernel<1, 1, kGenTimed>, &generate_kernel<1, 2, kGenTimed>},
       {&generate_kernel<2, 1, kGenTimed>, &generate_kernel<2, 2, kGenTimed>},
       {&generate_kernel<4, 1, kGenTimed>, &generate_kernel<4, 2, kGenTimed>}},
      {{&generate_kernel<1, 1, kGenSlide>, &generate_kernel<1, 2, kGenSlide>},
       {&generate_kernel<2, 1, kGenSlide>, &generate_kernel<2, 2, kGenSlide>},
       {&generate_kernel<4, 1, kGenSlide>, &generate_kernel<4, 2, kGenSlide>}}};
  const GenKernel kernel = table[slide ? 1 : 0][V == 1 ? 0 : (V == 2 ? 1 : 2)][deg - 1];
  if (lds_bytes > 64 * 1024 &&
      hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                          p->max_lds) != hipSuccess)
    return FPSCHED_EHIP;
  unsigned long long* counter = static_cast<unsigned long long*>(d_workspace);
  hipLaunchKernelGGL(reset_counter_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(hip_stream), counter,
                     (unsigned long long)(blocks * best_waves * cpw));
  hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(64 * best_waves), (size_t)lds_bytes,
                     static_cast<hipStream_t>(hip_stream), tables, reinterpret_cast<const int32_t*>(d_policy),
                     d_inflight, nullptr, (long long)n_sets, (long long)n_sets, 0, nullptr, d_steps, d_status, counter,
                     GenResults{reinterpret_cast<long long*>(out.makespan), reinterpret_cast<long long*>(out.idle),
                                out.peak, out.flags});
  return check_hip(hipGetLastError());
}

int fpsched_generate_evaluate(const fpsched_problem* p, const fpsched_actor_policy* d_policy,
                              const int32_t* d_inflight, int64_t n_sets, fpsched_results out, int32_t* d_steps,
                              uint8_t* d_status, void* d_workspace, size_t workspace_bytes, void* hip_stream) {
  return run_generate_evaluate(p, d_policy, d_inflight, n_sets, out, d_steps, d_status, d_workspace, workspace_bytes,
                               hip_stream, false);
}

int fpsched_generate_slide_evaluate(const fpsched_problem* p, const fpsched_actor_policy* d_policy,
                                    const int32_t* d_inflight, int64_t n_sets, fpsched_results out, int32_t* d_steps,
                                    uint8_t* d_status, void* d_workspace, size_t workspace_bytes, void* hip_stream) {
  return run_generate_evaluate(p, d_policy, d_inflight, n_sets, out, d_steps, d_status, d_workspace, workspace_bytes,
                               hip_stream, true);
}

// k smallest (key, index) among the entries whose flag byte is 0: tile sort, then a tree of merges
static int run_topk(const long long* keys, const unsigned char* flags, int64_t n_cand, int32_t k, int64_t* d_idx,
                    int64_t* d_key, int32_t* d_count, char* key_buffers, hipStream_t st) {
  int64_t cap_a = 0, cap_b = 0;
  topk_level_sizes(n_cand, k, &cap_a, &cap_b);
  Key* buf_a = reinterpret_cast<Key*>(key_buffers);
  Key* buf_b = buf_a + cap_a;
  long long* f_idx = reinterpret_cast<long long*>(d_idx);
  long long* f_ms = reinterpret_cast<long long*>(d_key);

  int64_t n = n_cand;
  const Key* src = nullptr;  // level 0 reads keys / flags
  Key* dst = buf_a;
  for (;;) {
    const int64_t tiles = std::max<int64_t>(1, (n + kTile - 1) / kTile);
    const bool last = tiles == 1;
    hipLaunchKernelGGL(topk_tile_kernel, dim3((unsigned)tiles), dim3(kTopkThreads), 0, st, keys, flags, src,
                       (long long)n, (int)k, last ? nullptr : dst, last ? f_idx : nullptr, last ? f_ms : nullptr,
                       last ? d_count : nullptr);
    if (hipGetLastError() != hipSuccess) return FPSCHED_EHIP;
    if (last) break;
    n = tiles * k;
    src = dst;
    dst = (dst == buf_a) ? buf_b : buf_a;
  }
  return FPSCHED_OK;
}

int fpsched_topk(const fpsched_problem* p, fpsched_results in, int64_t n_cand, int32_t k,
                 int64_t* d_idx, int64_t* d_makespan, int32_t* d_count, void* d_workspace,
                 size_t workspace_bytes, void* hip_stream) {
  if (!p || n_cand < 0 || k < 1 || k > 1024 || !d_idx || !d_makespan || !d_count) return FPSCHED_EINVAL;
  if (p->device_id < 0) return FPSCHED_ENODEV;
  if (n_cand > 0 && (!in.makespan || !in.flags)) return FPSCHED_EINVAL;
  if (!d_workspace || (reinterpret_cast<uintptr_t>(d_workspace) & 15)) return FPSCHED_EINVAL;
  if (workspace_bytes < fpsched_workspace_bytes(p, n_cand, k)) return FPSCHED_ENOMEM;
  DeviceGuard g(p->device_id);
  if (!g.ok) return FPSCHED_EHIP;
  return run_topk(reinterpret_cast<const long long*>(in.makespan), in.flags, n_cand, k, d_idx, d_makespan, d_count,
                  static_cast<char*>(d_workspace) + 256, static_cast<hipStream_t>(hip_stream));
}

size_t fpsched_static_scratch_bytes(void) { return kStaticScratchBytes; }

int fpsched_evaluate_topk_static(const fpsched_problem* p, const uint16_t* d_ops, int64_t n_cand,
                                 int32_t stride_words, fpsched_results out, int32_t k, int64_t* d_idx,
                                 int64_t* d_makespan, int32_t* d_count, void* hip_stream) {
  if (!p || n_cand < 0 || k < 1 || k > 1024) return FPSCHED_EINVAL;
  if (p->device_id < 0) return FPSCHED_ENODEV;
  if (!p->d_static_scratch) return FPSCHED_EHIP;
  // the same layout as a caller's workspace: [256 bytes: work counter][top-k key buffers]
  if (fpsched_workspace_bytes(p, n_cand, k) > kStaticScratchBytes) return FPSCHED_ESCRATCH;
  // (the counter is preset by a kernel and every key that is read was written by the level before: nothing
  // of an earlier call's contents is ever looked at)
  const int rc = fpsched_evaluate(p, d_ops, n_cand, stride_words, out, p->d_static_scratch, kStaticScratchBytes,
                                  hip_stream);
  if (rc != FPSCHED_OK) return rc;
  return fpsched_topk(p, out, n_cand, k, d_idx, d_makespan, d_count, p->d_static_scratch, kStaticScratchBytes,
                      hip_stream);
}

size_t fpsched_rank_workspace_bytes(const fpsched_problem* p, int64_t n_cand, int32_t k) {
  if (!p || n_cand < 0) return 0;
  const size_t base = (fpsched_workspace_bytes(p, n_cand, k) + 15) & ~(size_t)15;
  return base + (size_t)n_cand * 8 + (((size_t)n_cand + 15) & ~(size_t)15);
}

int fpsched_rank(const fpsched_problem* p, fpsched_results in, int64_t n_cand, int32_t k, int32_t mode,
                 int32_t include_over_cap, int64_t* d_idx, int64_t* d_key, int32_t* d_count, void* d_workspace,
                 size_t workspace_bytes, void* hip_stream) {
  if (!p || n_cand < 0 || k < 1 || k > 1024 || !d_idx || !d_key || !d_count) return FPSCHED_EINVAL;
  if (mode < FPSCHED_RANK_MAKESPAN || mode > FPSCHED_RANK_IDLE) return FPSCHED_EINVAL;
  if (p->device_id < 0) return FPSCHED_ENODEV;
  if (n_cand > 0 && (!in.makespan || !in.idle || !in.peak || !in.flags)) return FPSCHED_EINVAL;
  if (!d_workspace || (reinterpret_cast<uintptr_t>(d_workspace) & 15)) return FPSCHED_EINVAL;
  if (workspace_bytes < fpsched_rank_workspace_bytes(p, n_cand, k)) return FPSCHED_ENOMEM;
  DeviceGuard g(p->device_id);
  if (!g.ok) return FPSCHED_EHIP;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const size_t base = (fpsched_workspace_bytes(p, n_cand, k) + 15) & ~(size_t)15;
  long long* keys = reinterpret_cast<long long*>(static_cast<char*>(d_workspace) + base);
  unsigned char* excluded = reinterpret_cast<unsigned char*>(keys + n_cand);
  if (n_cand > 0) {
    const int64_t blocks = (n_cand + 255) / 256;
    if (blocks > 0x7fffffffll) return FPSCHED_EINVAL;
    hipLaunchKernelGGL(rank_keys_kernel, dim3((unsigned)blocks), dim3(256), 0, st,
                       reinterpret_cast<const long long*>(in.makespan), reinterpret_cast<const long long*>(in.idle),
                       in.peak, in.flags, (long long)n_cand, (int)p->D, (int)mode, (int)(include_over_cap != 0), keys,
                       excluded);
    if (hipGetLastError() != hipSuccess) return FPSCHED_EHIP;
  }
  return run_topk(keys, excluded, n_cand, k, d_idx, d_key, d_count, static_cast<char*>(d_workspace) + 256, st);
}

// workspace of the sliding pass: [256 bytes: candidate counter][low halves of the start times: 16 bits per op
// word and lane of a candidate][escape lists: escape_cap dwords per row][stop positions: int32 per row]
// [flags of the timing pass: one byte per candidate]
static size_t wslide_starts_bytes(const fpsched_problem* p, int64_t n_cand, int32_t stride_words) {
  return (size_t)n_cand * p->tables.lanes_per_cand * (size_t)stride_words * sizeof(uint16_t);
}
// entries of a row's escape list: an op that waits 2^16 time units or more for its inputs; each such wait
// uses up 2^16 of the largest possible finish time (links: two transfers per op at most), plus the end mark
static int wslide_escape_cap(const fpsched_problem* p) {
  const int64_t bound = (int64_t)p->D * p->max_stride * (p->max_dur + 2 * p->max_comm);
  return (int)std::min<int64_t>(bound >> 16, 255) + 2;
}
static size_t wslide_escape_bytes(const fpsched_problem* p, int64_t n_cand) {
  return (((size_t)n_cand * p->D * wslide_escape_cap(p) * sizeof(uint32_t)) + 15) & ~(size_t)15;
}

size_t fpsched_wslide_workspace_bytes(const fpsched_problem* p, int64_t n_cand, int32_t stride_words) {
  if (!p || n_cand < 0 || stride_words < 8) return 0;
  const size_t rows = (size_t)n_cand * p->D;
  return 256 + wslide_starts_bytes(p, n_cand, stride_words) + wslide_escape_bytes(p, n_cand) +
         ((rows * sizeof(int32_t) + 15) & ~(size_t)15) + (((size_t)n_cand + 15) & ~(size_t)15);
}

int fpsched_wslide(const fpsched_problem* p, const uint16_t* d_ops, int64_t n_cand, int32_t stride_words,
                   uint16_t* d_ops_out, int32_t stride_out_words, fpsched_results out, void* d_workspace,
                   size_t workspace_bytes, void* hip_stream) {
  if (!p || n_cand < 0) return FPSCHED_EINVAL;
  if (p->device_id < 0) return FPSCHED_ENODEV;
  if (!p->has_w) return FPSCHED_EINVAL;
  // the pass knows one cost per (type, stage)
  if (!p->slide_ok || p->mb_set || p->sync_on || p->copy_depth > 0 || (p->links_on && !p->links_slide_ok)) return FPSCHED_EUNSUPPORTED;
  if (n_cand == 0) return FPSCHED_OK;
  if (!d_ops || !d_ops_out || !out.makespan || !out.idle || !out.peak || !out.flags) return FPSCHED_EINVAL;
  if (stride_words < 8 || (stride_words & 7) || stride_words > p->max_stride) return FPSCHED_EINVAL;
  if (stride_out_words < 8 || (stride_out_words & 7) || stride_out_words > p->max_stride) return FPSCHED_EINVAL;
  if ((reinterpret_cast<uintptr_t>(d_ops) & 15) || (reinterpret_cast<uintptr_t>(d_ops_out) & 15)) return FPSCHED_EINVAL;
  if (!d_workspace || (reinterpret_cast<uintptr_t>(d_workspace) & 15)) return FPSCHED_EINVAL;
  if (workspace_bytes < fpsched_wslide_workspace_bytes(p, n_cand, stride_words)) return FPSCHED_ENOMEM;
  const int lpc = p->stab.lanes_per_cand;
  // (a small batch is spread over the compute units: fewer wavefronts per workgroup)
  const int64_t place_waves_all = (n_cand * lpc + 63) / 64;
  const int place_threads = 64 * (int)std::clamp<int64_t>((place_waves_all + std::max(p->n_cu, 1) - 1) / std::max(p->n_cu, 1),
                                                          1, kSlideThreads / 64);
  const int64_t place_blocks = (n_cand * lpc + place_threads - 1) / place_threads;
  if (place_blocks > 0x7fffffffll) return FPSCHED_EINVAL;
  DeviceGuard g(p->device_id);
  if (!g.ok) return FPSCHED_EHIP;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  char* ws = static_cast<char*>(d_workspace);
  unsigned long long* counter = reinterpret_cast<unsigned long long*>(ws);
  uint32_t* starts = reinterpret_cast<uint32_t*>(ws + 256);
  uint32_t* escapes = reinterpret_cast<uint32_t*>(ws + 256 + wslide_starts_bytes(p, n_cand, stride_words));
  const int escape_cap = wslide_escape_cap(p);
  int32_t* stops = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(escapes) + wslide_escape_bytes(p, n_cand));
  unsigned char* timed_flags = reinterpret_cast<unsigned char*>(stops) + (((size_t)n_cand * p->D * sizeof(int32_t) + 15) & ~(size_t)15);
  // pass 1: the lists without their W items, timed by the evaluation kernel (launched as in fpsched_evaluate)
  // (under the link model: that model's tables and workgroup shape; W items send nothing, so the second
  // pass is the same)
  const bool links = p->links_on;
  const SlotTables& times_tab = links ? p->stab_times_links : p->stab_times;
  const int waves = links ? p->links_waves : p->slot_waves;
  const int grid = links ? p->links_grid : p->slot_grid;
  const size_t times_lds = (size_t)(links ? p->links_lds_bytes : p->slot_lds_bytes) + 16;
  const SlotLaunch L = slot_launch(times_tab, waves, grid, times_lds, n_cand);
  const int per_block = times_tab.cands_per_wave * L.waves;
  const int64_t blocks = L.blocks;
  const int64_t row_words = (int64_t)p->D * stride_words;
  const int draw_block = (int)std::clamp<int64_t>((12288 + row_words - 1) / row_words, 1, times_tab.cands_per_wave);
  const bool one_class = p->stab.n_classes == 1;
  hipLaunchKernelGGL(reset_counter_kernel, dim3(1), dim3(64), 0, st, counter, (unsigned long long)(blocks * per_block));
  hipLaunchKernelGGL(links ? slot_kernel_of<kSlotTimesLinks>(p->slot_v, p->slot_deg2, one_class)
                           : slot_kernel_of<kSlotTimes>(p->slot_v, p->slot_deg2, one_class),
                     dim3((unsigned)blocks), dim3(64 * L.waves), L.lds_bytes, st, times_tab, d_ops, (long long)n_cand,
                     (int)stride_words, (long long*)nullptr, (long long*)nullptr, (int*)nullptr, timed_flags, counter,
                     draw_block, starts, stops, (const int32_t*)nullptr, escapes, escape_cap);
  if (hipGetLastError() != hipSuccess) return FPSCHED_EHIP;
  // pass 2: every row places its W items on its own
  hipLaunchKernelGGL(wslide_place_kernel, dim3((unsigned)place_blocks), dim3(place_threads),
                     (size_t)kNKinds * kMaxChunks * lpc * 16 + (place_threads / 64) * kSlideWaveLdsBytes, st, p->stab, d_ops,
                     (long long)n_cand, (int)stride_words,
                     starts, escapes, escape_cap, stops, timed_flags, d_ops_out, (int)stride_out_words,
                     reinterpret_cast<long long*>(out.makespan), reinterpret_cast<long long*>(out.idle), out.peak,
                     out.flags);
  return check_hip(hipGetLastError());
}

int fpsched_wslide_evaluate(const fpsched_problem* p, const uint16_t* d_ops, int64_t n_cand, int32_t stride_words,
                            fpsched_results out, void* d_workspace, size_t workspace_bytes, void* hip_stream) {
  if (!p || n_cand < 0) return FPSCHED_EINVAL;
  if (p->device_id < 0) return FPSCHED_ENODEV;
  if (!p->has_w) return FPSCHED_EINVAL;
  if (!p->slide_eval_ok || p->mb_set || p->sync_on || p->copy_depth > 0 || (p->links_on && !p->links_slide_eval_ok))
    return FPSCHED_EUNSUPPORTED;
  if (n_cand == 0) return FPSCHED_OK;
  if (!d_ops || !out.makespan || !out.idle || !out.peak || !out.flags) return FPSCHED_EINVAL;
  if (stride_words < 8 || (stride_words & 7) || stride_words > p->max_stride) return FPSCHED_EINVAL;
  if (reinterpret_cast<uintptr_t>(d_ops) & 15) return FPSCHED_EINVAL;
  if (!d_workspace || (reinterpret_cast<uintptr_t>(d_workspace) & 15)) return FPSCHED_EINVAL;
  if (workspace_bytes < 256) return FPSCHED_ENOMEM;
  DeviceGuard g(p->device_id);
  if (!g.ok) return FPSCHED_EHIP;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  unsigned long long* counter = static_cast<unsigned long long*>(d_workspace);
  // launched as fpsched_evaluate launches the plain form, or the link form (same workgroup shape; 16 bytes of LDS more)
  const bool links = p->links_on;
  const SlotTables& tab = links ? p->stab_slide_links : p->stab_slide;
  const SlotLaunch L = slot_launch(tab, links ? p->links_waves : p->slot_waves, links ? p->links_grid : p->slot_grid,
                                   (size_t)(links ? p->links_lds_bytes : p->slot_lds_bytes) + 16, n_cand);
  const int per_block = tab.cands_per_wave * L.waves;
  const int64_t blocks = L.blocks;
  const int64_t row_words = (int64_t)p->D * stride_words;
  const int draw_block = (int)std::clamp<int64_t>((12288 + row_words - 1) / row_words, 1, tab.cands_per_wave);
  hipLaunchKernelGGL(reset_counter_kernel, dim3(1), dim3(64), 0, st, counter, (unsigned long long)(blocks * per_block));
  hipLaunchKernelGGL(links ? slot_kernel_of<kSlotSlideLinks>(p->slot_v, p->slot_deg2, tab.n_classes == 1)
                           : slot_kernel_of<kSlotSlide>(p->slot_v, p->slot_deg2, tab.n_classes == 1), dim3((unsigned)blocks),
                     dim3(64 * L.waves), L.lds_bytes, st, tab, d_ops, (long long)n_cand,
                     (int)stride_words, reinterpret_cast<long long*>(out.makespan), reinterpret_cast<long long*>(out.idle),
                     out.peak, out.flags, counter, draw_block, (uint32_t*)nullptr, (int32_t*)nullptr,
                     (const int32_t*)nullptr, (uint32_t*)nullptr, 0);
  return check_hip(hipGetLastError());
}

static int64_t pareto_tiles(int64_t n_cand) { return (n_cand + kTile - 1) / kTile; }

size_t fpsched_pareto_workspace_bytes(const fpsched_problem* p, int64_t n_cand) {
  if (!p || n_cand < 0) return 0;
  const size_t tiles = (size_t)pareto_tiles(n_cand);
  // [256 reserved][tile fronts: Key, then peak, kTile entries per tile][entries per tile front]
  return 256 + tiles * kTile * (sizeof(Key) + sizeof(int32_t)) + ((tiles * sizeof(int32_t) + 15) & ~(size_t)15);
}

int fpsched_pareto(const fpsched_problem* p, fpsched_results in, int64_t n_cand, int32_t kmax, int64_t* d_idx,
                   int64_t* d_makespan, int32_t* d_peak, int32_t* d_count, void* d_workspace,
                   size_t workspace_bytes, void* hip_stream) {
  if (!p || n_cand < 0 || kmax < 1 || kmax > 1024 || !d_idx || !d_makespan || !d_peak || !d_count)
    return FPSCHED_EINVAL;
  if (pareto_tiles(n_cand) > kParetoMaxTiles) return FPSCHED_EINVAL;
  if (p->device_id < 0) return FPSCHED_ENODEV;
  if (n_cand > 0 && (!in.makespan || !in.peak || !in.flags)) return FPSCHED_EINVAL;
  if (!d_workspace || (reinterpret_cast<uintptr_t>(d_workspace) & 15)) return FPSCHED_EINVAL;
  if (workspace_bytes < fpsched_pareto_workspace_bytes(p, n_cand)) return FPSCHED_ENOMEM;
  DeviceGuard g(p->device_id);
  if (!g.ok) return FPSCHED_EHIP;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int64_t tiles = pareto_tiles(n_cand);
  Key* front_keys = reinterpret_cast<Key*>(static_cast<char*>(d_workspace) + 256);
  int* front_peak = reinterpret_cast<int*>(front_keys + tiles * kTile);
  int* tile_count = front_peak + tiles * kTile;
  if (tiles > 0) {
    hipLaunchKernelGGL(pareto_tile_kernel, dim3((unsigned)tiles), dim3(kTopkThreads), 0, st,
                       reinterpret_cast<const long long*>(in.makespan), in.peak, in.flags, (long long)n_cand,
                       (int)p->D, front_keys, front_peak, tile_count);
    if (hipGetLastError() != hipSuccess) return FPSCHED_EHIP;
  }
  hipLaunchKernelGGL(pareto_merge_kernel, dim3(1), dim3(kParetoMergeThreads), 0, st, front_keys, front_peak,
                     tile_count, (int)tiles, (int)kmax, reinterpret_cast<long long*>(d_idx),
                     reinterpret_cast<long long*>(d_makespan), d_peak, d_count);
  if (hipGetLastError() != hipSuccess) return FPSCHED_EHIP;
  return FPSCHED_OK;
}

int fpsched_apply_caps(const fpsched_problem* p, const int32_t* d_peak, const int32_t* d_caps,
                       int32_t per_candidate, int64_t n_cand, uint8_t* d_flags, void* hip_stream) {
  if (!p || n_cand < 0 || !d_caps) return FPSCHED_EINVAL;
  if (p->device_id < 0) return FPSCHED_ENODEV;
  if (n_cand == 0) return FPSCHED_OK;
  if (!d_peak || !d_flags) return FPSCHED_EINVAL;
  const int64_t blocks = (n_cand + 255) / 256;
  if (blocks > 0x7fffffffll) return FPSCHED_EINVAL;
  DeviceGuard g(p->device_id);
  if (!g.ok) return FPSCHED_EHIP;
  hipLaunchKernelGGL(apply_caps_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                     d_peak, d_caps, (int)(per_candidate != 0), (long long)n_cand, (int)p->D, d_flags);
  if (hipGetLastError() != hipSuccess) return FPSCHED_EHIP;
  return FPSCHED_OK;
}

int fpsched_encode(const fpsched_problem* p, const int32_t* ksm, int32_t device, int32_t n,
                   uint16_t* out_words) {
  if (!p || n < 0 || device < 0 || device >= p->D || (n > 0 && (!ksm || !out_words))) return FPSCHED_EINVAL;
  for (int i = 0; i < n; ++i) {
    const int kind = ksm[3 * i], s = ksm[3 * i + 1], j = ksm[3 * i + 2];
    if (kind <= FPSCHED_END || kind >= FPSCHED_NKINDS || s < 0 || s >= p->S || j < 0 || j >= p->sync_items[s])
      return FPSCHED_EINVAL;
    if (p->stage_device[s] != device) return FPSCHED_EINVAL;
    if (kind == FPSCHED_W && !p->has_w) return FPSCHED_EINVAL;
    out_words[i] = FPSCHED_WORD(kind, p->stage_chunk[s], j);
  }
  return FPSCHED_OK;
}

int64_t fpsched_validate(const fpsched_problem* p, const uint16_t* h_ops, int64_t n_cand,
                         int32_t stride_words) {
  if (!p || n_cand < 0 || stride_words < 1 || (n_cand > 0 && !h_ops)) return FPSCHED_EINVAL;
  int64_t bad = 0;
  for (int64_t c = 0; c < n_cand; ++c) {
    bool cand_bad = false;
    for (int d = 0; d < p->D && !cand_bad; ++d) {
      const uint16_t* row = h_ops + ((size_t)c * p->D + d) * stride_words;
      for (int i = 0; i < stride_words; ++i) {
        const unsigned w = row[i];
        const int kind = w >> 13;
        if (kind == FPSCHED_END) break;
        const int c = (int)((w >> 11) & 3);
        if (c >= p->n_chunks[d] || (int)(w & 0x7ff) >= p->sync_items[p->local_stage[(size_t)d * kMaxChunks + c]] ||
            (kind == FPSCHED_W && !p->has_w)) { cand_bad = true; break; }
      }
    }
    bad += cand_bad;
  }
  return bad;
}

}  // extern "C"

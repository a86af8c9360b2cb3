// Host side of the C ABI declared in include/triaccel.h: argument validation, workspace,
// pointer-table upload and the sequence of kernel launches of one optimizer step
// (control loop of Sec. 3.4).  No device synchronisation happens inside triaccel_step.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "../../include/triaccel.h"
#include "kernels.h"
#include "power.h"

using namespace triaccel;

namespace {

thread_local std::string g_last_error;

int hip_fail(hipError_t e, const char* what) {
  g_last_error = std::string(what) + ": " + hipGetErrorString(e);
  return TRIACCEL_E_HIP;
}

#define TA_HIP(call)                                   \
  do {                                                 \
    hipError_t e_ = (call);                            \
    if (e_ != hipSuccess) return hip_fail(e_, #call);  \
  } while (0)

constexpr int kRing = 4;  // pinned staging buffers for the pointer table
constexpr int kTableSlots = 8;  // device copies of the pointer table kept per handle
constexpr uint64_t kMemSampleEvery = 16;  // calls between two hipMemGetInfo samples when the caller passes no figures

bool valid_dtype(int32_t d) { return d == TRIACCEL_FP16 || d == TRIACCEL_BF16 || d == TRIACCEL_FP32; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

struct StepGraph {
  hipGraph_t graph = nullptr;
  hipGraphExec_t exec = nullptr;
  hipGraphNode_t root = nullptr;  // the node that writes the per-step scalars
};

struct triaccel_ctx {
  hipStream_t stream = nullptr;
  int device = 0;
  triaccel_config cfg{};
  Hyper hp{};
  uint32_t n = 0;
  std::vector<int64_t> numel;
  std::vector<int32_t> grad_dtype;
  DeviceTables t{};
  std::vector<TensorDesc> desc;       // the table of the step being enqueued
  // Device copies of the table.  A caller that alternates between a few sets of buffers (double-buffered
  // gradients, a probe on some steps only) finds each of its tables already on the device; a table seen
  // for the first time replaces the one used longest ago (the copy is ordered on the stream).
  struct TableSlot {
    TensorDesc* dev = nullptr;
    std::vector<TensorDesc> sent;  // what the device copy holds
    bool valid = false;            // `sent` has been enqueued for upload
    uint64_t last_used = 0;
  };
  TableSlot tables[kTableSlots];
  TensorDesc* staging[kRing] = {};
  hipEvent_t staging_ev[kRing] = {};
  bool staging_used[kRing] = {};
  int ring_pos = 0;
  GlobalDev* pinned_res = nullptr;
  uint64_t step_index = 0;
  uint64_t mem_used_cached = 0, mem_total_cached = 0;  // last hipMemGetInfo sample (0: none yet)
  bool result_valid = false;  // a step has been enqueued since init / set_state
  int32_t next_batch = 0;
  int profiling = 0;  // 0 off, 1 every stage boundary, 2 only the boundaries of the update kernel
  hipEvent_t ev[TRIACCEL_PROFILE_RING][TRIACCEL_N_STAGES + 1] = {};
  uint64_t ev_step[TRIACCEL_PROFILE_RING] = {};  // step_index recorded in each ring slot (0 = none)
  int ev_level[TRIACCEL_PROFILE_RING] = {};      // profiling level that slot was recorded with
  std::vector<LayerDev> layer_host;
  std::vector<void*> device_allocs;
  bool use_graph = false;
  // One captured step per (variant, device copy of the table): [0][s] steps without a curvature
  // refresh, [1][s] with; the kernels of a captured step hold the address of table copy s.
  StepGraph graphs[2][kTableSlots];
  // power iteration (only with cfg.power_k > 0)
  PowerTables pt{};
  PowerDesc* power_staging[kRing] = {};
  hipEvent_t power_ev[kRing] = {};
  bool power_used[kRing] = {};
  int power_pos = 0;
  bool power_called = false;
  hipEvent_t power_prof[4] = {};
  bool power_timed = false;  // the last call recorded its kernel boundaries
  std::vector<PowerLayer> power_host;
};

namespace {

template <typename T>
int dev_alloc(triaccel_ctx* c, T** out, size_t count) {
  void* p = nullptr;
  const size_t bytes = (count ? count : 1) * sizeof(T);
  hipError_t e = hipMalloc(&p, bytes);
  if (e != hipSuccess) {
    g_last_error = std::string("hipMalloc: ") + hipGetErrorString(e);
    return TRIACCEL_E_NO_MEMORY;
  }
  c->device_allocs.push_back(p);
  e = hipMemset(p, 0, bytes);
  if (e != hipSuccess) return hip_fail(e, "hipMemset");
  *out = static_cast<T*>(p);
  return TRIACCEL_OK;
}

int validate_config(const triaccel_config* cfg) {
  if (!cfg) return TRIACCEL_E_NULL_PTR;
  if (cfg->struct_size != sizeof(triaccel_config)) return TRIACCEL_E_INVALID_ARG;
  auto unit = [](float b) { return b >= 0.0f && b < 1.0f; };
  if (!unit(cfg->beta_var) || !unit(cfg->beta_curv)) return TRIACCEL_E_INVALID_ARG;
  if (!(cfg->tau_low <= cfg->tau_high)) return TRIACCEL_E_INVALID_ARG;
  if (!(cfg->alpha >= 0.0f) || !std::isfinite(cfg->alpha) || !std::isfinite(cfg->tau_curv)) return TRIACCEL_E_INVALID_ARG;
  if (cfg->sparsity_ppm > 1000000u) return TRIACCEL_E_INVALID_ARG;
  if (!(cfg->momentum >= 0.0f && cfg->momentum < 1.0f)) return TRIACCEL_E_INVALID_ARG;
  if (!(cfg->weight_decay >= 0.0f) || !std::isfinite(cfg->weight_decay)) return TRIACCEL_E_INVALID_ARG;
  if (cfg->ctrl_interval < 1 || cfg->growth_interval < 1) return TRIACCEL_E_INVALID_ARG;
  if (!(cfg->scale_backoff > 0.0f && cfg->scale_backoff <= 1.0f) || !(cfg->scale_growth >= 1.0f)) return TRIACCEL_E_INVALID_ARG;
  if (!(cfg->rho_low >= 0.0 && cfg->rho_low <= cfg->rho_high && cfg->rho_high <= 1.0)) return TRIACCEL_E_INVALID_ARG;
  if (cfg->delta_up < 0 || cfg->delta_down < 0 || cfg->b_min < 1 || cfg->b_max < cfg->b_min) return TRIACCEL_E_INVALID_ARG;
  if (cfg->power_k < 0 || cfg->power_k > kMaxPowerK) return TRIACCEL_E_INVALID_ARG;
  if (cfg->lambda_source != 0 && cfg->lambda_source != 1) return TRIACCEL_E_INVALID_ARG;
  if (cfg->lambda_source == 1 && cfg->power_k == 0) return TRIACCEL_E_INVALID_ARG;
  if (cfg->curvature_source != 0 && cfg->curvature_source != 1) return TRIACCEL_E_INVALID_ARG;
  if (cfg->elementwise_scale != 0 && cfg->elementwise_scale != 1) return TRIACCEL_E_INVALID_ARG;
  return TRIACCEL_OK;
}

// Checks one tensor entry of a step (or of init, where probe pointers are not required).
int validate_tensor(const triaccel_tensor& t, bool need_mom) {
  if (!t.param || !t.grad || !t.curv || !t.mask) return TRIACCEL_E_NULL_PTR;
  if (need_mom && !t.mom) return TRIACCEL_E_NULL_PTR;
  if ((t.z == nullptr) != (t.hz == nullptr)) return TRIACCEL_E_NULL_PTR;
  if (t.numel <= 0 || t.numel >= (int64_t(1) << 31)) return TRIACCEL_E_INVALID_ARG;
  if (!valid_dtype(t.grad_dtype)) return TRIACCEL_E_BAD_DTYPE;
  if (!aligned16(t.param) || !aligned16(t.grad) || !aligned16(t.curv) || !aligned16(t.mask) || !aligned16(t.mom) ||
      !aligned16(t.z) || !aligned16(t.hz))
    return TRIACCEL_E_ALIGNMENT;
  return TRIACCEL_OK;
}

void free_ctx(triaccel_ctx* c) {
  if (!c) return;
  for (void* p : c->device_allocs) (void)hipFree(p);
  for (int i = 0; i < kRing; ++i) {
    if (c->staging[i]) (void)hipHostFree(c->staging[i]);
    if (c->staging_ev[i]) (void)hipEventDestroy(c->staging_ev[i]);
    if (c->power_staging[i]) (void)hipHostFree(c->power_staging[i]);
    if (c->power_ev[i]) (void)hipEventDestroy(c->power_ev[i]);
    if (c->power_prof[i]) (void)hipEventDestroy(c->power_prof[i]);
  }
  for (auto& variant : c->graphs)
    for (auto& g : variant) {
      if (g.exec) (void)hipGraphExecDestroy(g.exec);
      if (g.graph) (void)hipGraphDestroy(g.graph);
    }
  if (c->pinned_res) (void)hipHostFree(c->pinned_res);
  for (auto& set : c->ev)
    for (auto& e : set)
      if (e) (void)hipEventDestroy(e);
  delete c;
}

// The kernels of one optimizer step, in order, on the handle's stream.  `ev` (eight events) records
// the stage boundaries.  Order of the stages: the per-layer assignment needs only the gradient
// moments and lambda_l = max |h_i| (known after the EMA pass), so it runs before the threshold is
// final; the mask is an output that nothing in the per-layer update depends on.
int enqueue_step(triaccel_ctx* h, const StepArg& sa, bool any_probe, hipEvent_t* ev, int level) {
  const float beta_h = h->cfg.beta_curv;
  const float omb_h = 1.0f - beta_h;
  const DeviceTables& T = h->t;
  hipStream_t s = h->stream;
  const bool fisher = h->cfg.curvature_source == 1;
  if (ev && level == 1) TA_HIP(hipEventRecord(ev[0], s));
  TA_HIP(launch_grad_stats(T, sa, s));
  if (ev && level == 1) TA_HIP(hipEventRecord(ev[1], s));
  if (any_probe) TA_HIP(launch_curv_ema(T, sa, beta_h, omb_h, fisher ? 1 : 0, s));
  if (ev && level == 1) TA_HIP(hipEventRecord(ev[2], s));
  TA_HIP(launch_layer(T, sa, h->hp, s));
  if (ev && level == 1) TA_HIP(hipEventRecord(ev[3], s));
  if (any_probe) {
    // fallback radix select: two rounds at full width (a first window, then a refinement or the
    // other side of a window that missed); rarer further rounds are made inside the second launch.
    // Each launch leaves at once when no tensor is (still) in histogram mode.
    // A set bound by its number of launches gets one: rounds beyond the first are then made by the
    // scanning workgroup alone.
    if (T.total_chunks >= kLaunchBoundChunks) TA_HIP(launch_hist_pass(T, sa, 0, s));
    TA_HIP(launch_hist_pass(T, sa, 8, s));
  }
  const bool elem = h->cfg.elementwise_scale == 1;
  if (elem && any_probe) {
    // element-wise step sizes need the final threshold: finish the mask and the selection first
    TA_HIP(launch_mask_pass(T, sa, s));
    TA_HIP(launch_select_finish(T, sa, h->hp.beta_curv, s));
  }
  if (ev) TA_HIP(hipEventRecord(ev[4], s));
  TA_HIP(launch_update(T, sa, h->cfg.weight_decay, h->cfg.momentum, h->cfg.alpha, elem, s));
  if (ev) TA_HIP(hipEventRecord(ev[5], s));
  TA_HIP(launch_update_resize(T, sa, h->cfg.weight_decay, h->cfg.momentum, h->cfg.alpha, elem, s));
  if (ev && level == 1) TA_HIP(hipEventRecord(ev[6], s));
  if (any_probe && !elem) TA_HIP(launch_select_finish(T, sa, h->hp.beta_curv, s));
  if (ev && level == 1) TA_HIP(hipEventRecord(ev[7], s));
  return TRIACCEL_OK;
}

// Graph form of the same step: captured once per variant (with / without a curvature refresh) and
// device copy of the tensor table (`slot`, the one h->t.tensors points to) from the launches above,
// with the kernels reading the per-step scalars from device memory; a replay updates the one node
// that writes those scalars and launches the graph.
int replay_step(triaccel_ctx* h, const StepScalars& sc, bool any_probe, int slot) {
  StepGraph& g = h->graphs[any_probe ? 1 : 0][slot];
  hipStream_t s = h->stream;
  if (!g.exec) {
    hipGraph_t graph = nullptr;
    TA_HIP(hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal));
    int rc = TRIACCEL_OK;
    hipError_t e = launch_set_scalars(h->t, sc, s);
    if (e != hipSuccess) rc = hip_fail(e, "launch_set_scalars");
    if (!rc) rc = enqueue_step(h, StepArg{sc, h->t.scalars}, any_probe, nullptr, 0);
    e = hipStreamEndCapture(s, &graph);  // always ends the capture, also after a failure above
    if (rc) {
      if (graph) (void)hipGraphDestroy(graph);
      return rc;
    }
    if (e != hipSuccess) return hip_fail(e, "hipStreamEndCapture");
    size_t n_roots = 0;
    hipGraphNode_t root = nullptr;
    e = hipGraphGetRootNodes(graph, nullptr, &n_roots);
    if (e == hipSuccess && n_roots == 1) e = hipGraphGetRootNodes(graph, &root, &n_roots);
    if (e == hipSuccess && n_roots != 1) {
      (void)hipGraphDestroy(graph);
      g_last_error = "captured step graph does not start with a single node";
      return TRIACCEL_E_HIP;
    }
    hipGraphExec_t exec = nullptr;
    if (e == hipSuccess) e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
    if (e != hipSuccess) {
      (void)hipGraphDestroy(graph);
      return hip_fail(e, "hipGraphInstantiate");
    }
    g.graph = graph;
    g.exec = exec;
    g.root = root;
  }
  hipKernelNodeParams params{};
  void* args[2];
  StepScalars* dst = h->t.scalars;
  set_scalars_node_params(&params, args, &sc, &dst);
  TA_HIP(hipGraphExecKernelNodeSetParams(g.exec, g.root, &params));
  TA_HIP(hipGraphLaunch(g.exec, s));
  return TRIACCEL_OK;
}

// Kernels are launched on the current device: it must be the one the handle was created on.
int check_device(const triaccel_ctx* h) {
  int dev = -1;
  TA_HIP(hipGetDevice(&dev));
  if (dev != h->device) {
    g_last_error = "the current HIP device is not the one the handle was created on";
    return TRIACCEL_E_HIP;
  }
  return TRIACCEL_OK;
}

int32_t batch_rule(const triaccel_config& cfg, int32_t batch, uint64_t used, uint64_t total) {
  // Sec. 3.3: strict comparisons as printed, then the clamp.
  const double u = (double)used, m = (double)total;
  int64_t b = batch;
  if (u < cfg.rho_low * m) b += cfg.delta_up;
  else if (u > cfg.rho_high * m) b -= cfg.delta_down;
  if (b < cfg.b_min) b = cfg.b_min;
  if (b > cfg.b_max) b = cfg.b_max;
  return (int32_t)b;
}

}  // namespace

extern "C" {

int triaccel_init(triaccel_handle* out, const triaccel_config* config, const triaccel_tensor* tensors, int32_t n,
                  void* hip_stream) {
  if (!out) return TRIACCEL_E_NULL_PTR;
  *out = nullptr;
  int rc = validate_config(config);
  if (rc) return rc;
  if (!tensors) return TRIACCEL_E_NULL_PTR;
  if (n <= 0) return TRIACCEL_E_INVALID_ARG;
  const bool need_mom = config->momentum != 0.0f;
  uint64_t total_chunks = 0;
  for (int32_t i = 0; i < n; ++i) {
    rc = validate_tensor(tensors[i], need_mom);
    if (rc) return rc;
    if (!valid_dtype(tensors[i].param_dtype)) return TRIACCEL_E_BAD_DTYPE;
    total_chunks += (uint64_t)((tensors[i].numel + kChunk - 1) / kChunk);
  }
  if (total_chunks >= (uint64_t(1) << 31)) return TRIACCEL_E_INVALID_ARG;

  triaccel_ctx* c = new (std::nothrow) triaccel_ctx();
  if (!c) return TRIACCEL_E_NO_MEMORY;
  c->stream = static_cast<hipStream_t>(hip_stream);
  c->cfg = *config;
  c->n = (uint32_t)n;
  c->hp = Hyper{config->beta_var,     config->beta_curv,     config->tau_low,       config->tau_high,
                config->tau_curv,     config->alpha,         config->sparsity_ppm,  config->momentum,
                config->weight_decay, config->ctrl_interval, config->scale_backoff, config->scale_growth,
                config->growth_interval, config->lambda_source, config->elementwise_scale,
                config->topk_abs};
  auto fail = [&](int code) {
    free_ctx(c);
    return code;
  };
  hipError_t e = hipGetDevice(&c->device);
  if (e != hipSuccess) return fail(hip_fail(e, "hipGetDevice"));
  hipDeviceProp_t prop;
  e = hipGetDeviceProperties(&prop, c->device);
  if (e != hipSuccess) return fail(hip_fail(e, "hipGetDeviceProperties"));
  const uint32_t cus = prop.multiProcessorCount > 0 ? (uint32_t)prop.multiProcessorCount : 256u;

  // chunk list and per-tensor table
  std::vector<ChunkRef> chunks;
  chunks.reserve(total_chunks);
  c->desc.resize(n);
  c->numel.resize(n);
  c->grad_dtype.resize(n);
  c->layer_host.resize(n);
  uint64_t cand_total = 0;
  uint32_t max_chunks = 0;
  for (int32_t i = 0; i < n; ++i) {
    const triaccel_tensor& t = tensors[i];
    const uint32_t nc = (uint32_t)((t.numel + kChunk - 1) / kChunk);
    TensorDesc& d = c->desc[i];
    std::memset(&d, 0, sizeof(d));
    d.numel = t.numel;
    d.first_chunk = (uint32_t)chunks.size();
    d.n_chunks = nc;
    d.grad_dtype = t.grad_dtype;
    d.cand_offset = cand_total;
    d.cand_cap = t.numel < (int64_t)kCandCap ? (uint32_t)t.numel : kCandCap;
    d.sub_cap = (d.cand_cap + kCandLists - 1) / kCandLists;
    d.list_all = t.numel <= (int64_t)kListAllMax ? 1u : 0u;
    cand_total += (uint64_t)kCandLists * d.sub_cap + d.cand_cap;
    for (uint32_t k = 0; k < nc; ++k) chunks.push_back(ChunkRef{(uint32_t)i, k});
    if (nc > max_chunks) max_chunks = nc;
    c->numel[i] = t.numel;
    c->grad_dtype[i] = t.grad_dtype;
    LayerDev& ls = c->layer_host[i];
    std::memset(&ls, 0, sizeof(ls));
    ls.code = ls.prev_code = t.param_dtype;
    ls.mode = kSelHist;  // first probed step: histogram over the full key range
    ls.win_lo = 0;
    ls.win_shift = kFullShift;
    ls.win_bins = kHistBins;
    ls.win_hi = 0x80000000u;
    ls.var_ext = 3.0e38f;  // no extrapolation error measured yet
  }
  DeviceTables& T = c->t;
  T.n_tensors = (uint32_t)n;
  T.total_chunks = (uint32_t)chunks.size();
  T.max_chunks_per_tensor = max_chunks;
  T.persistent_grid = cus * 8;
  for (auto& slot : c->tables)
    if ((rc = dev_alloc(c, &slot.dev, (size_t)n))) return fail(rc);
  T.tensors = c->tables[0].dev;
  if ((rc = dev_alloc(c, &T.chunks, chunks.size()))) return fail(rc);
  if ((rc = dev_alloc(c, &T.partials, chunks.size()))) return fail(rc);
  if ((rc = dev_alloc(c, &T.ema_partials, chunks.size()))) return fail(rc);
  if ((rc = dev_alloc(c, &T.layers, (size_t)n))) return fail(rc);
  if ((rc = dev_alloc(c, &T.glob, 1))) return fail(rc);
  if ((rc = dev_alloc(c, &T.hist, (size_t)n * kHistBins))) return fail(rc);
  if ((rc = dev_alloc(c, &T.cands, (size_t)cand_total))) return fail(rc);
  if ((rc = dev_alloc(c, &T.cand_counters, (size_t)n * (kCandLists + 1) * kCandCounterStride))) return fail(rc);
  if ((rc = dev_alloc(c, &T.trans_list, (size_t)n * 2))) return fail(rc);
  if ((rc = dev_alloc(c, &T.scalars, 1))) return fail(rc);
  e = hipMemcpy(T.chunks, chunks.data(), chunks.size() * sizeof(ChunkRef), hipMemcpyHostToDevice);
  if (e != hipSuccess) return fail(hip_fail(e, "hipMemcpy(chunks)"));
  // shapes and chunk ranges are valid from now on; the pointers arrive with every step
  for (auto& slot : c->tables) {
    e = hipMemcpy(slot.dev, c->desc.data(), (size_t)n * sizeof(TensorDesc), hipMemcpyHostToDevice);
    if (e != hipSuccess) return fail(hip_fail(e, "hipMemcpy(tensor table)"));
  }
  e = hipMemcpy(T.layers, c->layer_host.data(), (size_t)n * sizeof(LayerDev), hipMemcpyHostToDevice);
  if (e != hipSuccess) return fail(hip_fail(e, "hipMemcpy(layers)"));
  for (int i = 0; i < kRing; ++i) {
    e = hipHostMalloc(reinterpret_cast<void**>(&c->staging[i]), (size_t)n * sizeof(TensorDesc), hipHostMallocDefault);
    if (e != hipSuccess) return fail(hip_fail(e, "hipHostMalloc(staging)"));
    e = hipEventCreateWithFlags(&c->staging_ev[i], hipEventDisableTiming);
    if (e != hipSuccess) return fail(hip_fail(e, "hipEventCreate"));
  }
  if (config->power_k > 0) {
    // workspace of the power iteration: segment table, per-segment sums, per-layer records
    std::vector<SegRef> segs;
    std::vector<uint32_t> seg_first((size_t)n);
    for (int32_t i = 0; i < n; ++i) {
      seg_first[i] = (uint32_t)segs.size();
      const uint32_t ns = (c->desc[i].n_chunks + kPowerSeg - 1) / kPowerSeg;
      for (uint32_t k = 0; k < ns; ++k) segs.push_back(SegRef{(uint32_t)i, k});
    }
    PowerTables& P = c->pt;
    P.tensors = T.tensors;
    P.chunks = T.chunks;
    P.layers = T.layers;
    P.n_tensors = (uint32_t)n;
    P.total_chunks = T.total_chunks;
    P.total_segs = (uint32_t)segs.size();
    if ((rc = dev_alloc(c, &P.descs, (size_t)n))) return fail(rc);
    if ((rc = dev_alloc(c, &P.segs, segs.size()))) return fail(rc);
    if ((rc = dev_alloc(c, &P.seg_first, (size_t)n))) return fail(rc);
    if ((rc = dev_alloc(c, &P.partials, segs.size() * (size_t)power_partial_len(config->power_k)))) return fail(rc);
    if ((rc = dev_alloc(c, &P.state, (size_t)n))) return fail(rc);
    e = hipMemcpy(P.segs, segs.data(), segs.size() * sizeof(SegRef), hipMemcpyHostToDevice);
    if (e != hipSuccess) return fail(hip_fail(e, "hipMemcpy(segments)"));
    e = hipMemcpy(P.seg_first, seg_first.data(), (size_t)n * sizeof(uint32_t), hipMemcpyHostToDevice);
    if (e != hipSuccess) return fail(hip_fail(e, "hipMemcpy(segment index)"));
    for (int i = 0; i < kRing; ++i) {
      e = hipHostMalloc(reinterpret_cast<void**>(&c->power_staging[i]), (size_t)n * sizeof(PowerDesc), hipHostMallocDefault);
      if (e != hipSuccess) return fail(hip_fail(e, "hipHostMalloc(power staging)"));
      e = hipEventCreateWithFlags(&c->power_ev[i], hipEventDisableTiming);
      if (e != hipSuccess) return fail(hip_fail(e, "hipEventCreate"));
    }
    c->power_host.resize((size_t)n);
  }
  e = hipHostMalloc(reinterpret_cast<void**>(&c->pinned_res), sizeof(GlobalDev), hipHostMallocDefault);
  if (e != hipSuccess) return fail(hip_fail(e, "hipHostMalloc(result)"));
  std::memset(c->pinned_res, 0, sizeof(GlobalDev));
  e = hipHostGetDevicePointer(reinterpret_cast<void**>(&T.host_result), c->pinned_res, 0);
  if (e != hipSuccess) return fail(hip_fail(e, "hipHostGetDevicePointer(result)"));
  e = hipDeviceSynchronize();
  if (e != hipSuccess) return fail(hip_fail(e, "hipDeviceSynchronize"));
  *out = c;
  return TRIACCEL_OK;
}

int triaccel_step(triaccel_handle h, const triaccel_tensor* tensors, int32_t n, const triaccel_step_args* args) {
  if (!h) return TRIACCEL_E_NOT_INITIALISED;
  if (!tensors || !args) return TRIACCEL_E_NULL_PTR;
  if (args->struct_size != sizeof(triaccel_step_args)) return TRIACCEL_E_INVALID_ARG;
  if ((uint32_t)n != h->n) return TRIACCEL_E_SHAPE_MISMATCH;
  if (!(args->loss_scale > 0.0f) || !std::isfinite(args->loss_scale) || !std::isfinite(args->lr))
    return TRIACCEL_E_INVALID_ARG;
  if (int drc = check_device(h)) return drc;
  const bool need_mom = h->cfg.momentum != 0.0f;
  const bool fisher = h->cfg.curvature_source == 1;
  bool any_probe = false;
  for (int32_t i = 0; i < n; ++i) {
    const triaccel_tensor& t = tensors[i];
    if (t.numel != h->numel[i] || t.grad_dtype != h->grad_dtype[i]) return TRIACCEL_E_SHAPE_MISMATCH;
    const int rc = validate_tensor(t, need_mom);
    if (rc) return rc;
    if (fisher && t.z != nullptr) return TRIACCEL_E_INVALID_ARG;  // no probe pairs in this mode
    any_probe = any_probe || t.z != nullptr;
  }
  if (fisher) any_probe = args->update_curvature != 0;
  // stage (4) of the control loop: batch size from memory usage, on the host
  uint64_t used = args->mem_used_bytes, total = args->mem_total_bytes;
  if (total == 0) {
    // the runtime's figures cost a driver round trip: they are sampled on the first call and then on
    // every kMemSampleEvery-th one, and the last sample is used in between
    if (h->mem_total_cached == 0 || h->step_index % kMemSampleEvery == 0) {
      size_t free_b = 0, total_b = 0;
      TA_HIP(hipMemGetInfo(&free_b, &total_b));
      h->mem_total_cached = total_b;
      h->mem_used_cached = total_b - free_b;
    }
    total = h->mem_total_cached;
    used = h->mem_used_cached;
  }
  const int32_t next_batch = batch_rule(h->cfg, args->batch_size, used, total);
  // ---- nothing below can fail on the arguments ----
  for (int32_t i = 0; i < n; ++i) {
    const triaccel_tensor& t = tensors[i];
    TensorDesc& d = h->desc[i];
    d.param = t.param;
    d.grad = t.grad;
    d.z = t.z;
    d.hz = t.hz;
    d.curv = t.curv;
    d.mom = need_mom ? t.mom : nullptr;
    d.mask = t.mask;
    d.has_probe = fisher ? (any_probe ? 1 : 0) : (t.z != nullptr);
  }
  const size_t table_bytes = (size_t)n * sizeof(TensorDesc);
  const uint64_t index = h->step_index + 1;
  int use = -1, victim = 0;
  for (int i = 0; i < kTableSlots; ++i) {
    triaccel_ctx::TableSlot& slot = h->tables[i];
    if (slot.valid && std::memcmp(h->desc.data(), slot.sent.data(), table_bytes) == 0) {
      use = i;
      break;
    }
    if (!slot.valid) {
      if (h->tables[victim].valid) victim = i;
    } else if (h->tables[victim].valid && slot.last_used < h->tables[victim].last_used) {
      victim = i;
    }
  }
  if (use < 0) {
    triaccel_ctx::TableSlot& slot = h->tables[victim];
    const int stage = h->ring_pos;
    if (h->staging_used[stage]) TA_HIP(hipEventSynchronize(h->staging_ev[stage]));
    std::memcpy(h->staging[stage], h->desc.data(), table_bytes);
    slot.valid = false;  // until the copy below is known to be enqueued
    TA_HIP(hipMemcpyAsync(slot.dev, h->staging[stage], table_bytes, hipMemcpyHostToDevice, h->stream));
    TA_HIP(hipEventRecord(h->staging_ev[stage], h->stream));
    h->ring_pos = (h->ring_pos + 1) % kRing;
    h->staging_used[stage] = true;
    slot.sent = h->desc;
    slot.valid = true;
    use = victim;
  }
  h->tables[use].last_used = index;
  h->t.tensors = h->tables[use].dev;

  // the call counts, and its result can be read, only once all of its work is enqueued
  StepScalars sc{};
  sc.lr = args->lr;
  sc.loss_scale = args->loss_scale;
  sc.inv_scale = 1.0f / args->loss_scale;
  sc.step_id = index;
  const bool prof = h->profiling != 0;
  h->ev_step[index % TRIACCEL_PROFILE_RING] = 0;
  if (h->use_graph && !prof) {
    const int rc = replay_step(h, sc, any_probe, use);
    if (rc) return rc;
  } else {
    hipEvent_t* ev = prof ? h->ev[index % TRIACCEL_PROFILE_RING] : nullptr;
    const int rc = enqueue_step(h, StepArg{sc, nullptr}, any_probe, ev, h->profiling);
    if (rc) return rc;
    if (prof) {
      h->ev_step[index % TRIACCEL_PROFILE_RING] = index;
      h->ev_level[index % TRIACCEL_PROFILE_RING] = h->profiling;
    }
  }
  h->step_index = index;
  h->next_batch = next_batch;
  h->result_valid = true;
  return TRIACCEL_OK;
}

int triaccel_result(triaccel_handle h, triaccel_step_result* out) {
  if (!h) return TRIACCEL_E_NOT_INITIALISED;
  if (!out) return TRIACCEL_E_NULL_PTR;
  if (out->struct_size != sizeof(triaccel_step_result)) return TRIACCEL_E_INVALID_ARG;
  if (h->step_index == 0 || !h->result_valid) return TRIACCEL_E_NOT_INITIALISED;
  TA_HIP(hipStreamSynchronize(h->stream));
  out->skipped = h->pinned_res->res_skipped;
  out->step_index = h->step_index;
  out->next_loss_scale = h->pinned_res->res_next_scale;
  out->next_batch_size = h->next_batch;
  return TRIACCEL_OK;
}

int triaccel_layer_state(triaccel_handle h, triaccel_layer_info* out, int32_t n) {
  if (!h) return TRIACCEL_E_NOT_INITIALISED;
  if (!out) return TRIACCEL_E_NULL_PTR;
  if ((uint32_t)n != h->n) return TRIACCEL_E_SHAPE_MISMATCH;
  TA_HIP(hipStreamSynchronize(h->stream));
  TA_HIP(hipMemcpy(h->layer_host.data(), h->t.layers, (size_t)n * sizeof(LayerDev), hipMemcpyDeviceToHost));
  for (int32_t i = 0; i < n; ++i) {
    const LayerDev& ls = h->layer_host[i];
    triaccel_layer_info& o = out[i];
    o.numel = h->numel[i];
    o.mean = ls.mean;
    o.var = ls.var;
    o.v = ls.v;
    o.theta = ls.theta;
    o.nnz = ls.nnz;
    o.lambda = ls.lambda;
    o.lambda_ctrl = ls.lambda_ctrl;
    o.eta = ls.eta;
    o.code = ls.code;
    o.prev_code = ls.prev_code;
    o.found_inf = ls.found_inf;
    o.curv_nonfinite = ls.curv_nonfinite;
    o.sel_passes = ls.sel_passes;
    o.sel_listed = ls.sel_listed;
    o.sel_outcome = ls.sel_outcome;
  }
  return TRIACCEL_OK;
}

namespace {
struct StateHeader {
  uint64_t magic;       // "TRIACCL1"
  uint32_t layer_size;  // sizeof(LayerDev): guards against a blob from another build
  uint32_t n;
  uint64_t step_index;
  int32_t next_batch;
  int32_t good_steps;
  uint64_t shape_hash;  // over numel and gradient dtypes
  uint64_t config_hash; // over the hyper-parameters
};
constexpr uint64_t kStateMagic = 0x314c434341495254ull;

uint64_t fnv1a(const void* data, size_t bytes, uint64_t h = 1469598103934665603ull) {
  const unsigned char* p = static_cast<const unsigned char*>(data);
  for (size_t i = 0; i < bytes; ++i) h = (h ^ p[i]) * 1099511628211ull;
  return h;
}
uint64_t shape_hash(const triaccel_ctx* c) {
  uint64_t h = fnv1a(c->numel.data(), c->numel.size() * sizeof(int64_t));
  return fnv1a(c->grad_dtype.data(), c->grad_dtype.size() * sizeof(int32_t), h);
}
}  // namespace

int64_t triaccel_state_size(triaccel_handle h) {
  if (!h) return TRIACCEL_E_NOT_INITIALISED;
  return (int64_t)(sizeof(StateHeader) + (size_t)h->n * sizeof(LayerDev));
}

int triaccel_get_state(triaccel_handle h, void* buf, int64_t size) {
  if (!h) return TRIACCEL_E_NOT_INITIALISED;
  if (!buf) return TRIACCEL_E_NULL_PTR;
  if (size != triaccel_state_size(h)) return TRIACCEL_E_INVALID_ARG;
  TA_HIP(hipStreamSynchronize(h->stream));
  GlobalDev g;
  TA_HIP(hipMemcpy(&g, h->t.glob, sizeof(g), hipMemcpyDeviceToHost));
  StateHeader hd{};
  hd.magic = kStateMagic;
  hd.layer_size = (uint32_t)sizeof(LayerDev);
  hd.n = h->n;
  hd.step_index = h->step_index;
  hd.next_batch = h->next_batch;
  hd.good_steps = g.good_steps;
  hd.shape_hash = shape_hash(h);
  hd.config_hash = fnv1a(&h->hp, sizeof(h->hp));
  std::memcpy(buf, &hd, sizeof(hd));
  TA_HIP(hipMemcpy(static_cast<char*>(buf) + sizeof(hd), h->t.layers, (size_t)h->n * sizeof(LayerDev),
                   hipMemcpyDeviceToHost));
  return TRIACCEL_OK;
}

int triaccel_set_state(triaccel_handle h, const void* buf, int64_t size) {
  if (!h) return TRIACCEL_E_NOT_INITIALISED;
  if (!buf) return TRIACCEL_E_NULL_PTR;
  if (size != triaccel_state_size(h)) return TRIACCEL_E_SHAPE_MISMATCH;
  StateHeader hd;
  std::memcpy(&hd, buf, sizeof(hd));
  if (hd.magic != kStateMagic || hd.layer_size != sizeof(LayerDev)) return TRIACCEL_E_INVALID_ARG;
  if (hd.n != h->n || hd.shape_hash != shape_hash(h)) return TRIACCEL_E_SHAPE_MISMATCH;
  if (hd.config_hash != fnv1a(&h->hp, sizeof(h->hp))) return TRIACCEL_E_INVALID_ARG;
  TA_HIP(hipStreamSynchronize(h->stream));
  // the small global record starts clean (both parities of its per-step words are zero between steps)
  GlobalDev g;
  std::memset(&g, 0, sizeof(g));
  g.good_steps = hd.good_steps;
  TA_HIP(hipMemcpy(h->t.glob, &g, sizeof(g), hipMemcpyHostToDevice));
  TA_HIP(hipMemcpy(h->t.layers, static_cast<const char*>(buf) + sizeof(hd), (size_t)h->n * sizeof(LayerDev),
                   hipMemcpyHostToDevice));
  h->step_index = hd.step_index;
  h->next_batch = hd.next_batch;
  std::memset(h->pinned_res, 0, sizeof(GlobalDev));
  h->result_valid = false;
  for (auto& s : h->ev_step) s = 0;  // stage timings of the other run do not apply
  return TRIACCEL_OK;
}

int triaccel_power_iter(triaccel_handle h, const triaccel_power_tensor* vectors, int32_t n, int32_t k, int32_t latch) {
  if (!h) return TRIACCEL_E_NOT_INITIALISED;
  if (!vectors) return TRIACCEL_E_NULL_PTR;
  if ((uint32_t)n != h->n) return TRIACCEL_E_SHAPE_MISMATCH;
  if (k < 1 || k > h->cfg.power_k) return TRIACCEL_E_INVALID_ARG;
  if (int drc = check_device(h)) return drc;
  for (int32_t i = 0; i < n; ++i) {
    const triaccel_power_tensor& v = vectors[i];
    if (!v.u || !v.hu) return TRIACCEL_E_NULL_PTR;
    if (v.stride < h->numel[i] || (v.stride & 3) != 0) return TRIACCEL_E_INVALID_ARG;
    if (!aligned16(v.u) || !aligned16(v.hu)) return TRIACCEL_E_ALIGNMENT;
  }
  const int slot = h->power_pos;
  h->power_pos = (h->power_pos + 1) % kRing;
  if (h->power_used[slot]) TA_HIP(hipEventSynchronize(h->power_ev[slot]));
  for (int32_t i = 0; i < n; ++i) h->power_staging[slot][i] = PowerDesc{vectors[i].u, vectors[i].hu, vectors[i].stride};
  TA_HIP(hipMemcpyAsync(h->pt.descs, h->power_staging[slot], (size_t)n * sizeof(PowerDesc), hipMemcpyHostToDevice,
                        h->stream));
  TA_HIP(hipEventRecord(h->power_ev[slot], h->stream));
  h->power_used[slot] = true;
  if (h->profiling)
    for (auto& e : h->power_prof)
      if (!e) TA_HIP(hipEventCreate(&e));
  TA_HIP(launch_power_iter(h->pt, k, latch ? 1 : 0, h->stream, h->profiling ? h->power_prof : nullptr));
  h->power_timed = h->profiling;
  h->power_called = true;
  return TRIACCEL_OK;
}

static_assert(sizeof(PowerInfoOut) == sizeof(triaccel_power_info), "the device record is the public one");
static_assert(TRIACCEL_STATIC_MAX_TENSORS == kStaticMaxTensors && TRIACCEL_STATIC_MAX_CHUNKS == kStaticMaxChunks,
              "limits of the header");

int triaccel_power_iter_static(const triaccel_power_tensor* vectors, const int64_t* numel, int32_t n, int32_t k,
                               triaccel_power_info* info, void* hip_stream) {
  if (n < 0 || n > kStaticMaxTensors) {
    g_last_error = "triaccel_power_iter_static: at most 256 tensors per call";
    return TRIACCEL_E_INVALID_ARG;
  }
  if (n == 0) {  // set-up only: look up the fixed array of the current device
    TA_HIP(power_static_prepare());
    return TRIACCEL_OK;
  }
  if (!vectors || !numel || !info) return TRIACCEL_E_NULL_PTR;
  if (k < 1 || k > kMaxPowerK) return TRIACCEL_E_INVALID_ARG;
  StaticTensor ts[kStaticMaxTensors];
  int64_t chunks = 0;
  for (int32_t i = 0; i < n; ++i) {
    const triaccel_power_tensor& v = vectors[i];
    if (!v.u || !v.hu) return TRIACCEL_E_NULL_PTR;
    if (numel[i] <= 0 || numel[i] >= (int64_t(1) << 31)) return TRIACCEL_E_INVALID_ARG;
    if (v.stride < numel[i] || (v.stride & 3) != 0) return TRIACCEL_E_INVALID_ARG;
    if (!aligned16(v.u) || !aligned16(v.hu)) return TRIACCEL_E_ALIGNMENT;
    chunks += (numel[i] + kChunk - 1) / kChunk;
    ts[i] = StaticTensor{v.u, v.hu, v.stride, numel[i]};
  }
  if (chunks > kStaticMaxChunks) {
    g_last_error = "triaccel_power_iter_static: the tensors of one call may hold at most 65536 pieces of 4096 "
                   "elements (268,435,456 elements); split the call";
    return TRIACCEL_E_INVALID_ARG;
  }
  if ((reinterpret_cast<uintptr_t>(info) & 3u) != 0) return TRIACCEL_E_ALIGNMENT;
  TA_HIP(launch_power_iter_static(ts, n, k, reinterpret_cast<PowerInfoOut*>(info), static_cast<hipStream_t>(hip_stream)));
  return TRIACCEL_OK;
}

int triaccel_power_state(triaccel_handle h, triaccel_power_info* out, int32_t n) {
  if (!h) return TRIACCEL_E_NOT_INITIALISED;
  if (!out) return TRIACCEL_E_NULL_PTR;
  if ((uint32_t)n != h->n) return TRIACCEL_E_SHAPE_MISMATCH;
  if (h->cfg.power_k == 0 || !h->power_called) return TRIACCEL_E_NOT_INITIALISED;
  TA_HIP(hipStreamSynchronize(h->stream));
  TA_HIP(hipMemcpy(h->power_host.data(), h->pt.state, (size_t)n * sizeof(PowerLayer), hipMemcpyDeviceToHost));
  TA_HIP(hipMemcpy(h->layer_host.data(), h->t.layers, (size_t)n * sizeof(LayerDev), hipMemcpyDeviceToHost));
  for (int32_t i = 0; i < n; ++i) {
    const PowerLayer& p = h->power_host[i];
    triaccel_power_info& o = out[i];
    for (int j = 0; j < kMaxPowerK; ++j) {
      o.rayleigh[j] = p.rayleigh[j];
      o.resid[j] = p.resid[j];
      o.hnorm[j] = p.hnorm[j];
    }
    o.deficient = p.deficient;
    o.lambda_max = p.lambda_max;
    o.lambda_latched = h->layer_host[i].lambda_power;
  }
  return TRIACCEL_OK;
}

int32_t triaccel_batch_next(const triaccel_config* config, int32_t batch_size, uint64_t mem_used_bytes,
                            uint64_t mem_total_bytes) {
  if (!config) return batch_size;
  return batch_rule(*config, batch_size, mem_used_bytes, mem_total_bytes);
}

void triaccel_destroy(triaccel_handle h) {
  if (!h) return;
  (void)hipStreamSynchronize(h->stream);
  free_ctx(h);
}

const char* triaccel_strerror(int code) {
  switch (code) {
    case TRIACCEL_OK: return "success";
    case TRIACCEL_E_INVALID_ARG: return "invalid argument";
    case TRIACCEL_E_BAD_DTYPE: return "dtype code must be 0 (FP16), 1 (BF16) or 2 (FP32)";
    case TRIACCEL_E_SHAPE_MISMATCH: return "tensor list does not match the one given at init";
    case TRIACCEL_E_NULL_PTR: return "required pointer is NULL";
    case TRIACCEL_E_ALIGNMENT: return "device pointer is not 16-byte aligned";
    case TRIACCEL_E_HIP: return "HIP runtime error (see triaccel_last_error)";
    case TRIACCEL_E_NOT_INITIALISED: return "handle not initialised or no step enqueued yet";
    case TRIACCEL_E_NO_MEMORY: return "out of memory";
    default: return "unknown error code";
  }
}

const char* triaccel_last_error(void) { return g_last_error.c_str(); }

int triaccel_set_graph(triaccel_handle h, int32_t on) {
  if (!h) return TRIACCEL_E_NOT_INITIALISED;
  if (on && h->stream == nullptr) {
    g_last_error = "graph replay needs a stream of its own: the default stream cannot be captured";
    return TRIACCEL_E_HIP;
  }
  h->use_graph = on != 0;
  return TRIACCEL_OK;
}

int triaccel_set_profiling(triaccel_handle h, int32_t on) {
  if (!h) return TRIACCEL_E_NOT_INITIALISED;
  if (on) {
    for (auto& set : h->ev)
      for (auto& e : set)
        if (!e) TA_HIP(hipEventCreate(&e));
  }
  if (on < 0 || on > 2) return TRIACCEL_E_INVALID_ARG;
  h->profiling = on;
  return TRIACCEL_OK;
}

int triaccel_stage_times_get(triaccel_handle h, int32_t steps_back, triaccel_stage_times* out) {
  if (!h) return TRIACCEL_E_NOT_INITIALISED;
  if (!out) return TRIACCEL_E_NULL_PTR;
  if (steps_back < 0 || steps_back >= TRIACCEL_PROFILE_RING || (uint64_t)steps_back >= h->step_index)
    return TRIACCEL_E_INVALID_ARG;
  const uint64_t step = h->step_index - (uint64_t)steps_back;
  const int slot = (int)(step % TRIACCEL_PROFILE_RING);
  if (h->ev_step[slot] != step) return TRIACCEL_E_NOT_INITIALISED;
  TA_HIP(hipStreamSynchronize(h->stream));
  for (int i = 0; i < TRIACCEL_N_STAGES; ++i) {
    out->ms[i] = 0.0f;
    if (h->ev_level[slot] == 1 || i == 4) TA_HIP(hipEventElapsedTime(&out->ms[i], h->ev[slot][i], h->ev[slot][i + 1]));
  }
  return TRIACCEL_OK;
}

int triaccel_power_times_get(triaccel_handle h, float* ms) {
  if (!h) return TRIACCEL_E_NOT_INITIALISED;
  if (!ms) return TRIACCEL_E_NULL_PTR;
  if (!h->power_called || !h->power_timed) return TRIACCEL_E_NOT_INITIALISED;
  TA_HIP(hipStreamSynchronize(h->stream));
  for (int i = 0; i < 3; ++i) TA_HIP(hipEventElapsedTime(&ms[i], h->power_prof[i], h->power_prof[i + 1]));
  return TRIACCEL_OK;
}

int triaccel_cast_f32(const float* src, void* dst, int64_t n, int32_t dtype, void* hip_stream) {
  if (!src || !dst) return TRIACCEL_E_NULL_PTR;
  if (n < 0 || n > (int64_t)0x7fffffff * kChunk) return TRIACCEL_E_INVALID_ARG;  // one workgroup per chunk
  if (!valid_dtype(dtype)) return TRIACCEL_E_BAD_DTYPE;
  if (!aligned16(src) || !aligned16(dst)) return TRIACCEL_E_ALIGNMENT;
  if (n == 0) return TRIACCEL_OK;
  TA_HIP(launch_cast(src, dst, n, dtype, static_cast<hipStream_t>(hip_stream)));
  return TRIACCEL_OK;
}

}  // extern "C"

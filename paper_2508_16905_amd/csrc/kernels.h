// Host-callable launchers of the gfx950 kernels (defined in kernels.hip).
#pragma once
#include <hip/hip_runtime.h>

#include "common.h"

namespace triaccel {

// Device pointers and sizes of a handle's workspace.
struct DeviceTables {
  TensorDesc* tensors;
  ChunkRef* chunks;
  StatPartial* partials;
  EmaPartial* ema_partials;  // one record per chunk, written by the EMA kernel
  LayerDev* layers;
  GlobalDev* glob;
  GlobalDev* host_result;  // pinned host memory (device-visible address): the per-layer kernel leaves the step's result record there
  uint32_t* hist;        // n_tensors x kHistBins
  Candidate* cands;      // pool: per tensor kCandLists * sub_cap + cand_cap entries
  uint32_t* cand_counters;  // n_tensors x (kCandLists + 1) counters, kCandCounterStride words apart
  uint32_t* trans_list;  // 2 x n_tensors
  StepScalars* scalars;  // device copy of the per-step scalars, read by the kernels of a replayed graph
  uint32_t n_tensors;
  uint32_t total_chunks;
  uint32_t max_chunks_per_tensor;
  uint32_t persistent_grid;  // workgroups of the persistent streaming kernels
};

hipError_t launch_grad_stats(const DeviceTables& t, const StepArg& sa, hipStream_t s);
hipError_t launch_curv_ema(const DeviceTables& t, const StepArg& sa, float beta_h, float omb_h, int fisher,
                           hipStream_t s);
hipError_t launch_hist_pass(const DeviceTables& t, const StepArg& sa, int serial_rounds, hipStream_t s);
hipError_t launch_select_finish(const DeviceTables& t, const StepArg& sa, float beta_h, hipStream_t s);
hipError_t launch_layer(const DeviceTables& t, const StepArg& sa, const Hyper& hp, hipStream_t s);
hipError_t launch_update(const DeviceTables& t, const StepArg& sa, float wd, float mu, float alpha, bool elem,
                         hipStream_t s);
hipError_t launch_mask_pass(const DeviceTables& t, const StepArg& sa, hipStream_t s);
hipError_t launch_update_resize(const DeviceTables& t, const StepArg& sa, float wd, float mu, float alpha,
                                bool elem, hipStream_t s);
// Writes the per-step scalars to device memory (first node of a captured step).
hipError_t launch_set_scalars(const DeviceTables& t, const StepScalars& sc, hipStream_t s);
// Kernel-node parameters of that launch, for updating an instantiated graph; `args` must hold two
// pointers and outlive the call that consumes the parameters.
void set_scalars_node_params(hipKernelNodeParams* p, void** args, const StepScalars* sc, StepScalars* const* dst);
hipError_t launch_cast(const float* src, void* dst, int64_t n, int dtype, hipStream_t s);

}  // namespace triaccel

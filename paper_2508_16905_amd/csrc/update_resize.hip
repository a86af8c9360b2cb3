// gfx950 kernels: the later launches of the in-place update of tensors whose storage size changes
// (2 <-> 4 bytes per element), and the stand-alone conversion utility.
#include "resize_body.h"

namespace triaccel {

// Launches 1 .. n_stages - 1 of the in-place resize (launch 0 is part of the update kernel's grid).
template <bool ELEM>
__global__ __launch_bounds__(kThreads) void k_update_resize(const TensorDesc* __restrict__ tds, const LayerDev* layers,
                                                            const GlobalDev* glob, const uint32_t* trans_list,
                                                            uint32_t n_tensors, ResizePlan plan, uint32_t launch,
                                                            uint32_t slots, StepArg sa, float wd, float mu, float alpha) {
  const StepScalars sc = step_scalars(sa);
  if (step_skipped(glob, sc.step_id)) return;
  resize_items<ELEM>(tds, layers, glob, trans_list, n_tensors, plan, launch, slots, blockIdx.x, gridDim.x, sc, wd, mu,
                     alpha);
}

// ---------------------------------------------------------------------------------------------
// Utility: fp32 -> {fp16, bf16, fp32} array conversion with the store path of the update kernel.
// ---------------------------------------------------------------------------------------------
template <int ND>
__global__ __launch_bounds__(kThreads) void k_cast(const float* __restrict__ src, void* dst, int64_t n) {
  // same shape as the step kernels: one workgroup per chunk, all loads of the chunk before its stores
  const int64_t base = (int64_t)blockIdx.x * kChunk;
  float v[kRows][4];
  if (base + kChunk <= n) {
#pragma unroll
    for (int r = 0; r < kRows; ++r) load4<kFP32>(src, base + r * kRowElems + (int64_t)threadIdx.x * kVec, v[r]);
#pragma unroll
    for (int r = 0; r < kRows; ++r) store4<ND>(dst, base + r * kRowElems + (int64_t)threadIdx.x * kVec, v[r]);
  } else {
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
      const int64_t idx = base + r * kRowElems + (int64_t)threadIdx.x * kVec;
      if (idx < n) {
        load4_guard<kFP32>(src, idx, n, 0.0f, v[r]);
        store4_guard<ND>(dst, idx, n, v[r]);
      }
    }
  }
}

hipError_t launch_update_resize(const DeviceTables& t, const StepArg& sa, float wd, float mu, float alpha,
                                bool elem, hipStream_t s) {
  const ResizePlan plan = make_resize_plan(t.max_chunks_per_tensor, t.total_chunks);
  for (uint32_t launch = 1; launch < plan.n_stages; ++launch) {
    const ResizeGrid rg = resize_grid(plan, launch, t.n_tensors);
    if (elem)
      hipLaunchKernelGGL(k_update_resize<true>, dim3(rg.grid), dim3(kThreads), 0, s, t.tensors, t.layers, t.glob,
                         t.trans_list, t.n_tensors, plan, launch, rg.slots, sa, wd, mu, alpha);
    else
      hipLaunchKernelGGL(k_update_resize<false>, dim3(rg.grid), dim3(kThreads), 0, s, t.tensors, t.layers, t.glob,
                         t.trans_list, t.n_tensors, plan, launch, rg.slots, sa, wd, mu, alpha);
    TA_LAUNCH_CHECK();
  }
  return hipSuccess;
}

__global__ void k_set_scalars(StepScalars v, StepScalars* dst) {
  if (threadIdx.x == 0 && blockIdx.x == 0) *dst = v;
}

hipError_t launch_set_scalars(const DeviceTables& t, const StepScalars& sc, hipStream_t s) {
  hipLaunchKernelGGL(k_set_scalars, dim3(1), dim3(kWave), 0, s, sc, t.scalars);
  TA_LAUNCH_CHECK();
  return hipSuccess;
}

void set_scalars_node_params(hipKernelNodeParams* p, void** args, const StepScalars* sc, StepScalars* const* dst) {
  args[0] = const_cast<StepScalars*>(sc);
  args[1] = const_cast<StepScalars**>(dst);
  p->func = reinterpret_cast<void*>(k_set_scalars);
  p->gridDim = dim3(1);
  p->blockDim = dim3(kWave);
  p->sharedMemBytes = 0;
  p->kernelParams = args;
  p->extra = nullptr;
}

hipError_t launch_cast(const float* src, void* dst, int64_t n, int dtype, hipStream_t s) {
  int64_t blocks = (n + kChunk - 1) / kChunk;
  if (blocks < 1) blocks = 1;
  switch (dtype) {
    case kFP32: hipLaunchKernelGGL(k_cast<kFP32>, dim3((uint32_t)blocks), dim3(kThreads), 0, s, src, dst, n); break;
    case kBF16: hipLaunchKernelGGL(k_cast<kBF16>, dim3((uint32_t)blocks), dim3(kThreads), 0, s, src, dst, n); break;
    default: hipLaunchKernelGGL(k_cast<kFP16>, dim3((uint32_t)blocks), dim3(kThreads), 0, s, src, dst, n); break;
  }
  TA_LAUNCH_CHECK();
  return hipSuccess;
}

}  // namespace triaccel

// gfx950 kernels: in-place update of tensors whose storage size changes (2 <-> 4 bytes per element),
// and the stand-alone conversion utility.
#include "resize_schedule.h"
#include "update_body.h"

namespace triaccel {

// Tensors whose storage size changes (2 <-> 4 bytes per element) are rewritten in place, in the
// order resize_schedule.h lays down: stage 0 (the first chunks of a tensor, one workgroup, a barrier
// between the loads and the stores of every chunk), then subtree stages in which every workgroup
// walks the levels of its own subtree of chunks with a barrier between levels.  No workgroup waits
// for another; what a stage depends on was done by an earlier launch.  Launch q performs stage q for
// the narrowing tensors of the step's list and stage n_stages - 1 - q for the widening ones.
//
// Work items of a launch are (list entry, workgroup of that tensor) pairs, `slots` per entry (the
// larger of the two stages' workgroup counts); a workgroup takes the items blockIdx.x,
// blockIdx.x + gridDim.x, ...  The list and its length are written on the device by the per-layer
// kernel, so every launch is made on every step and leaves at once when the list is empty.
template <bool ELEM>
__global__ __launch_bounds__(kThreads) void k_update_resize(const TensorDesc* __restrict__ tds, const LayerDev* layers,
                                                            const GlobalDev* glob, const uint32_t* trans_list,
                                                            uint32_t n_tensors, ResizePlan plan, uint32_t launch,
                                                            uint32_t slots, StepArg sa, float wd, float mu, float alpha) {
  const StepScalars sc = step_scalars(sa);
  if (step_skipped(glob, sc.step_id)) return;
  const uint32_t count = glob->trans_count[sc.step_id & 1u];
  const uint32_t* list = trans_list + (sc.step_id & 1u) * n_tensors;
  const int tid = (int)threadIdx.x;
  const uint64_t items = (uint64_t)count * slots;
  for (uint64_t item = blockIdx.x; item < items; item += gridDim.x) {
    const uint32_t l = list[item / slots];
    const uint32_t r = (uint32_t)(item % slots);
    const LayerDev& ls = layers[l];
    const int pd = ls.prev_code, nd = ls.code;
    const bool narrowing = elem_size(nd) < elem_size(pd);
    const uint32_t stage = resize_stage_of_launch(plan, launch, narrowing);
    if (r >= resize_stage_roots(plan, stage)) continue;
    const TensorDesc td = tds[l];
    const StepSize ss{-ls.eta, sc.lr, alpha, ls.theta_key};
    if (stage == 0) {
      resize_walk_top(plan, td.n_chunks, narrowing, [&](uint32_t c) {
        ChunkRegs regs;
        update_load_any<ELEM>(td, pd, (int64_t)c * kChunk, sc.inv_scale, wd, mu, ss, tid, regs);
        __syncthreads();  // chunk 0 overwrites itself; a later chunk overwrites what an earlier one loaded
        update_store_any(td, nd, (int64_t)c * kChunk, tid, regs);
      });
    } else {
      if (plan.root[stage] + r >= td.n_chunks) continue;
      resize_walk_subtree(
          plan, stage, r, td.n_chunks, narrowing,
          [&](uint32_t c) { update_any<ELEM>(td, pd, nd, (int64_t)c * kChunk, sc.inv_scale, wd, mu, ss, tid); },
          [&]() { __syncthreads(); });
    }
  }
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
  for (uint32_t launch = 0; launch < plan.n_stages; ++launch) {
    // a narrowing tensor is at stage `launch`, a widening one at the mirrored stage
    const uint32_t a = resize_stage_roots(plan, launch), b = resize_stage_roots(plan, plan.n_stages - 1u - launch);
    const uint32_t slots = a > b ? a : b;
    uint64_t grid = (uint64_t)t.n_tensors * slots;
    if (grid > 65536u) grid = 65536u;
    if (elem)
      hipLaunchKernelGGL(k_update_resize<true>, dim3((uint32_t)grid), dim3(kThreads), 0, s, t.tensors, t.layers, t.glob,
                         t.trans_list, t.n_tensors, plan, launch, slots, sa, wd, mu, alpha);
    else
      hipLaunchKernelGGL(k_update_resize<false>, dim3((uint32_t)grid), dim3(kThreads), 0, s, t.tensors, t.layers, t.glob,
                         t.trans_list, t.n_tensors, plan, launch, slots, sa, wd, mu, alpha);
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

// gfx950 kernels: in-place update of tensors whose storage size changes (2 <-> 4 bytes per element),
// and the stand-alone conversion utility.
#include "update_body.h"

namespace triaccel {

// Tensors whose storage size changes (2 <-> 4 bytes per element) are rewritten in place in
// phases: phase 0 is chunk 0, phase p >= 1 the chunks [2^(p-1), 2^p).  Inside a phase the bytes
// written (element range [lo, hi) at the new size) never overlap the bytes read (same range at
// the old size) because hi <= 2 lo.  Narrowing runs the phases in ascending order, so every
// write lands on bytes whose old contents were consumed by an earlier phase; widening runs them
// in descending order for the same reason.
//
// The phases up to kSerialPhase (the first kSerialChunks chunks) are done by ONE workgroup per
// tensor in a single launch: a workgroup of 1024 threads takes four consecutive chunks per
// iteration (every 256-thread part loads its chunk, the workgroup synchronises, then stores), in
// ascending order when narrowing and in descending order when widening; what such a group of four
// overwrites was read by an earlier iteration, or by the same one before its barrier.  Each later
// phase is a launch of its own.  With L = the last phase of the largest tensor there are
// n_launch = 1 + max(0, L - kSerialPhase) launches:
//   narrowing:  launch 0 = serial part, launch j >= 1 = phase kSerialPhase + j;
//   widening:   launch j < n_launch - 1 = phase L - j, launch n_launch - 1 = serial part.
// A tensor with fewer phases than the largest one skips the launches beyond its own.  The first
// and the last launch run with 1024 threads per workgroup (their phase work is then spread over
// the four parts of a workgroup), the others with 256.
constexpr uint32_t kSerialPhase = 8;
constexpr uint32_t kSerialChunks = 1u << kSerialPhase;  // 256 chunks = 1,048,576 elements
constexpr int kSerialParts = 4;                          // 256-thread parts of the serial workgroup

template <bool ELEM>
__global__ __launch_bounds__(kSerialParts * kThreads) void k_update_resize(
    const TensorDesc* __restrict__ tds, const LayerDev* layers, const GlobalDev* glob, const uint32_t* trans_list,
    uint32_t n_tensors, uint32_t launch, uint32_t n_launch, StepArg sa, float wd, float mu, float alpha) {
  const StepScalars sc = step_scalars(sa);
  if (step_skipped(glob, sc.step_id)) return;
  const uint32_t count = glob->trans_count[sc.step_id & 1u];
  const uint32_t* list = trans_list + (sc.step_id & 1u) * n_tensors;
  const uint32_t parts = blockDim.x / kThreads;  // 1 or kSerialParts
  const uint32_t part = threadIdx.x / kThreads;
  const int lane = (int)(threadIdx.x % kThreads);
  for (uint32_t i = 0; i < count; ++i) {
    const uint32_t l = list[i];
    const TensorDesc td = tds[l];
    const LayerDev& ls = layers[l];
    const int pd = ls.prev_code, nd = ls.code;
    const bool narrowing = elem_size(nd) < elem_size(pd);
    const StepSize ss{-ls.eta, sc.lr, alpha, ls.theta_key};
    const bool serial = narrowing ? launch == 0 : launch == n_launch - 1u;
    if (serial) {
      if (i % gridDim.x != blockIdx.x) continue;  // one workgroup per tensor
      const uint32_t n_ser = min(kSerialChunks, td.n_chunks);
      const uint32_t n_it = (n_ser + parts - 1u) / parts;
      for (uint32_t it = 0; it < n_it; ++it) {
        const uint32_t c = (narrowing ? it : n_it - 1u - it) * parts + part;
        // every thread of the workgroup meets exactly one barrier per iteration
        if (c < n_ser) update_any<ELEM>(td, pd, nd, (int64_t)c * kChunk, sc.inv_scale, wd, mu, ss, true, lane);
        else __syncthreads();
      }
      continue;
    }
    // number of phases: 1 + ceil(log2(n_chunks))
    const uint32_t last_phase = td.n_chunks <= 1 ? 0u : 32u - (uint32_t)__clz(td.n_chunks - 1u);
    const uint32_t phase = narrowing ? kSerialPhase + launch : kSerialPhase + (n_launch - 1u - launch);
    if (phase > last_phase) continue;
    const uint32_t c_lo = 1u << (phase - 1u);  // phase > kSerialPhase >= 1
    const uint32_t c_hi = min(1u << phase, td.n_chunks);
    // a chunk c >= 1 reads and writes disjoint bytes (its element range at the old and at the new
    // size do not meet), so these phases need no synchronisation between its loads and its stores
    for (uint32_t c = c_lo + blockIdx.x * parts + part; c < c_hi; c += gridDim.x * parts)
      update_any<ELEM>(td, pd, nd, (int64_t)c * kChunk, sc.inv_scale, wd, mu, ss, false, lane);
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
  // last phase of the largest tensor: ceil(log2(chunks)); a phase holds at most half the chunks of a tensor
  uint32_t last_phase = 0;
  while ((1u << last_phase) < t.max_chunks_per_tensor) ++last_phase;
  const uint32_t n_launch = 1u + (last_phase > kSerialPhase ? last_phase - kSerialPhase : 0u);
  uint32_t grid = (t.max_chunks_per_tensor + 1) / 2;
  if (grid < 1) grid = 1;
  if (grid > t.persistent_grid) grid = t.persistent_grid;
  for (uint32_t launch = 0; launch < n_launch; ++launch) {
    // the launches that hold a serial part use the wide workgroup
    const uint32_t threads = (launch == 0 || launch == n_launch - 1u) ? kSerialParts * kThreads : kThreads;
    if (elem)
      hipLaunchKernelGGL(k_update_resize<true>, dim3(grid), dim3(threads), 0, s, t.tensors, t.layers, t.glob,
                         t.trans_list, t.n_tensors, launch, n_launch, sa, wd, mu, alpha);
    else
      hipLaunchKernelGGL(k_update_resize<false>, dim3(grid), dim3(threads), 0, s, t.tensors, t.layers, t.glob,
                         t.trans_list, t.n_tensors, launch, n_launch, sa, wd, mu, alpha);
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

// gfx950 kernels of the fused update + cast (stage 5 of the optimizer step) and the stand-alone
// mask pass.  Compiled as a translation unit of its own: the update body is specialised for every
// (gradient, old, new) precision triple, which dominates the build time.
#include "resize_body.h"

namespace triaccel {

// Mask pass as a kernel of its own, for the element-wise form of the update, where the threshold
// must be final before the update runs: the tensors whose mask the EMA kernel did not settle get
// their mask written and their range keys listed here, before k_select_finish.  Leaves at once
// when no tensor needs it (the steady state).
__global__ __launch_bounds__(kThreads) void k_mask_pass(const TensorDesc* __restrict__ tds,
                                                        const ChunkRef* __restrict__ chunks, uint32_t total_chunks,
                                                        const LayerDev* layers, const GlobalDev* glob, Candidate* cands,
                                                        uint32_t* counters, StepArg sa) {
  const StepScalars sc = step_scalars(sa);
  if (step_skipped(glob, sc.step_id)) return;
  if (glob->mask_pending[sc.step_id & 1u] == 0) return;
  for (uint32_t c = blockIdx.x; c < total_chunks; c += gridDim.x) {
    const ChunkRef cr = chunks[c];
    const TensorDesc td = tds[cr.tensor];
    const LayerDev& ls = layers[cr.tensor];
    const uint32_t mode = ls.mode;
    if (!td.has_probe || ls.mask_done || mode == kSelHist) continue;
    const int64_t base = (int64_t)cr.index * kChunk;
    if (base + kChunk <= td.numel)
      mask_chunk<true>(td, base, mode, ls.theta_key, ls.rng_lo, ls.rng_hi, cr.index, cr.tensor, cands, counters);
    else
      mask_chunk<false>(td, base, mode, ls.theta_key, ls.rng_lo, ls.rng_hi, cr.index, cr.tensor, cands, counters);
  }
}

// Tensors whose storage size does not change: element i is read and written at the same address
// by the same lane, so the update is in place.  One workgroup per chunk.  The same workgroup then
// runs the fallback mask pass of its chunk when the tensor's mask was not settled by the EMA
// kernel (nothing in the update depends on the mask, and a separate launch would cost a full
// grid of idle workgroups on every step that needs no fallback).
//
// The first `resize_wgs` workgroups of the grid do something else: the first launch of the in-place
// resize of the tensors whose storage size does change (resize_body.h).  It depends on the per-layer
// kernel only, like the update itself, so it needs no launch of its own; it comes first in the grid
// because its work items are the longer ones.
//
// In the element-wise form (ELEM) the threshold must be final before the update, so the mask and
// the listed keys are completed by the kernels before this one and no mask pass runs here.
template <bool ELEM>
__global__ __launch_bounds__(kThreads) void k_update(const TensorDesc* __restrict__ tds,
                                                     const ChunkRef* __restrict__ chunks, LayerDev* layers,
                                                     const GlobalDev* glob, Candidate* cands, uint32_t* counters,
                                                     const uint32_t* trans_list, uint32_t n_tensors, ResizePlan plan,
                                                     uint32_t resize_slots, uint32_t resize_wgs, StepArg sa, float wd,
                                                     float mu, float alpha) {
  const StepScalars sc = step_scalars(sa);
  if (step_skipped(glob, sc.step_id)) return;
  if (blockIdx.x < resize_wgs) {
    resize_items<ELEM>(tds, layers, glob, trans_list, n_tensors, plan, 0u, resize_slots, blockIdx.x, resize_wgs, sc, wd, mu,
                       alpha);
    return;
  }
  const ChunkRef cr = chunks[blockIdx.x - resize_wgs];
  LayerDev& ls = layers[cr.tensor];
  const int pd = ls.prev_code, nd = ls.code;
  const TensorDesc td = tds[cr.tensor];
  const int64_t base = (int64_t)cr.index * kChunk;
  const StepSize ss{-ls.eta, sc.lr, alpha, ls.theta_key};
  if (elem_size(pd) == elem_size(nd)) update_any<ELEM>(td, pd, nd, base, sc.inv_scale, wd, mu, ss, (int)threadIdx.x);
  if constexpr (ELEM) return;
  // kSelHist cannot remain after the last scan; never write a mask from a stale range
  const uint32_t mode = ls.mode;
  if (td.has_probe && !ls.mask_done && mode != kSelHist) {
    if (base + kChunk <= td.numel)
      mask_chunk<true>(td, base, mode, ls.theta_key, ls.rng_lo, ls.rng_hi, cr.index, cr.tensor, cands, counters);
    else
      mask_chunk<false>(td, base, mode, ls.theta_key, ls.rng_lo, ls.rng_hi, cr.index, cr.tensor, cands, counters);
  }
}

hipError_t launch_update(const DeviceTables& t, const StepArg& sa, float wd, float mu, float alpha, bool elem,
                         hipStream_t s) {
  const ResizePlan plan = make_resize_plan(t.max_chunks_per_tensor, t.total_chunks);
  const ResizeGrid rg = resize_grid(plan, 0u, t.n_tensors);
  const dim3 grid(t.total_chunks + rg.grid);
  if (elem)
    hipLaunchKernelGGL(k_update<true>, grid, dim3(kThreads), 0, s, t.tensors, t.chunks, t.layers, t.glob, t.cands,
                       t.cand_counters, t.trans_list, t.n_tensors, plan, rg.slots, rg.grid, sa, wd, mu, alpha);
  else
    hipLaunchKernelGGL(k_update<false>, grid, dim3(kThreads), 0, s, t.tensors, t.chunks, t.layers, t.glob, t.cands,
                       t.cand_counters, t.trans_list, t.n_tensors, plan, rg.slots, rg.grid, sa, wd, mu, alpha);
  TA_LAUNCH_CHECK();
  return hipSuccess;
}

hipError_t launch_mask_pass(const DeviceTables& t, const StepArg& sa, hipStream_t s) {
  const uint32_t grid = t.total_chunks < t.persistent_grid ? t.total_chunks : t.persistent_grid;
  hipLaunchKernelGGL(k_mask_pass, dim3(grid), dim3(kThreads), 0, s, t.tensors, t.chunks, t.total_chunks, t.layers,
                     t.glob, t.cands, t.cand_counters, sa);
  TA_LAUNCH_CHECK();
  return hipSuccess;
}

}  // namespace triaccel

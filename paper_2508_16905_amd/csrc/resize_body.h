// Work of one launch of the in-place resize (tensors whose storage size changes between 2 and 4
// bytes per element), as a device function: the first launch rides in the grid of the update kernel,
// the later ones are launches of their own (update_resize.hip).
#pragma once
#include "resize_schedule.h"
#include "update_body.h"

namespace triaccel {

// The tensors are rewritten in place in the order resize_schedule.h lays down: stage 0 (the first
// chunks of a tensor, one workgroup, a barrier between the loads and the stores of every chunk), then
// subtree stages in which every workgroup walks the levels of its own subtree of chunks with a
// barrier between levels.  No workgroup waits for another; what a stage depends on was done by an
// earlier launch.  Launch q performs stage q for the narrowing tensors of the step's list and stage
// n_stages - 1 - q for the widening ones.
//
// Work items of a launch are (list entry, workgroup of that tensor) pairs, `slots` per entry (the
// larger of the two stages' workgroup counts); workgroup `wg` of `n_wg` takes the items wg,
// wg + n_wg, ...  The list and its length are written on the device by the per-layer kernel, so the
// work is offered on every step and nothing happens when the list is empty.  Uniform over the
// workgroup (it contains barriers).
template <bool ELEM>
__device__ __forceinline__ void resize_items(const TensorDesc* __restrict__ tds, const LayerDev* layers,
                                             const GlobalDev* glob, const uint32_t* trans_list, uint32_t n_tensors,
                                             const ResizePlan& plan, uint32_t launch, uint32_t slots, uint32_t wg,
                                             uint32_t n_wg, const StepScalars& sc, float wd, float mu, float alpha) {
  const uint32_t count = glob->trans_count[sc.step_id & 1u];
  const uint32_t* list = trans_list + (sc.step_id & 1u) * n_tensors;
  const int tid = (int)threadIdx.x;
  const uint64_t items = (uint64_t)count * slots;
  for (uint64_t item = wg; item < items; item += n_wg) {
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

// Work items per list entry and workgroups offered to launch `launch`.
struct ResizeGrid {
  uint32_t slots;
  uint32_t grid;
};
inline ResizeGrid resize_grid(const ResizePlan& plan, uint32_t launch, uint32_t n_tensors) {
  // a narrowing tensor is at stage `launch`, a widening one at the mirrored stage
  const uint32_t a = resize_stage_roots(plan, launch), b = resize_stage_roots(plan, plan.n_stages - 1u - launch);
  const uint32_t slots = a > b ? a : b;
  uint64_t grid = (uint64_t)n_tensors * slots;
  if (grid > 65536u) grid = 65536u;
  return ResizeGrid{slots, (uint32_t)grid};
}

}  // namespace triaccel

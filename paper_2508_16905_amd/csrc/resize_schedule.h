// Order in which the chunks of a tensor are rewritten when its storage size changes in place
// (2 <-> 4 bytes per element), as plain functions that the kernels, their launcher and a host-side
// replay of the schedule all use.
//
// Element range [lo, hi) occupies bytes [s lo, s hi) at element size s.  NARROWING (4 -> 2): chunk c
// writes into bytes that held the old data of chunk c / 2 (its parent), so a chunk may be stored once
// its parent has been loaded.  WIDENING (2 -> 4): chunk c writes over the old data of chunks 2c and
// 2c + 1 (its children), so a chunk may be stored once both children have been loaded.  Chunk 0 is
// its own parent / child: its loads must precede its own stores.
//
// The dependence is a binary tree, and the subtrees rooted at the chunks [A, 2A) are independent of
// each other: level v of the subtree of root r is the contiguous run of chunks [r 2^v, (r + 1) 2^v),
// its stores land on the old bytes of level v - 1 (narrowing) or v + 1 (widening) of the same
// subtree, and never on the old bytes of its own level.  One workgroup walks one subtree, level by
// level with a workgroup barrier between levels (root to leaves when narrowing, leaves to root when
// widening) and without waiting for any other workgroup.  What a root itself depends on lies in
// [A / 2, A) (narrowing) -- chunks done by an earlier launch.  A step therefore needs
//   stage 0      chunks [0, top): one workgroup per tensor, chunk by chunk, barrier in every chunk
//   stage j >= 1 chunks [root_j, root_j 2^depth_j): root_j workgroups per tensor, depth_j levels each
// with root_1 = top and root_{j+1} = root_j 2^depth_j, in this order for a narrowing tensor and in
// the reverse order for a widening one.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define TA_HD __host__ __device__ inline
#else
#define TA_HD inline
#endif

namespace triaccel {

constexpr uint32_t kResizeMaxStages = 8;     // stage 0 plus up to 7 subtree stages
constexpr uint32_t kResizeTop = 16;          // chunks of stage 0 when subtree stages follow
constexpr uint32_t kResizeTopOnly = 128;     // tensors up to this many chunks: stage 0 alone
constexpr uint32_t kResizeBigSet = 16384;    // chunks in the whole set from which a launch more costs nothing
                                             // (= kLaunchBoundChunks of the step's other kernels)

struct ResizePlan {
  uint32_t n_stages;                  // 1 + number of subtree stages
  uint32_t top;                       // chunks [0, top) belong to stage 0
  uint32_t root[kResizeMaxStages];    // stage j >= 1: roots [root[j], 2 root[j])
  uint32_t depth[kResizeMaxStages];   // stage j >= 1: levels 0 .. depth[j] - 1
};

// Plan for a set whose largest tensor has `max_chunks` chunks.  Small sets are bound by the number of
// launches, so they get deep subtrees (up to 6 levels, 63 chunks per workgroup) and as few stages as
// possible; large sets get shallow ones (up to 4 levels, 15 chunks) for parallelism inside a tensor.
TA_HD ResizePlan make_resize_plan(uint32_t max_chunks, uint32_t total_chunks) {
  ResizePlan p{};
  p.n_stages = 1;
  if (max_chunks <= kResizeTopOnly) {
    p.top = max_chunks ? max_chunks : 1u;
    return p;
  }
  p.top = kResizeTop;
  uint32_t levels = 0;  // smallest count with top << levels >= max_chunks
  while (((uint64_t)p.top << levels) < max_chunks) ++levels;
  const uint32_t dmax = total_chunks >= kResizeBigSet ? 4u : 6u;
  const uint32_t n_sub = (levels + dmax - 1) / dmax;
  const uint32_t base = levels / n_sub, rem = levels % n_sub;
  uint32_t root = p.top;
  for (uint32_t j = 1; j <= n_sub; ++j) {
    p.root[j] = root;
    p.depth[j] = base + (j > n_sub - rem ? 1u : 0u);  // the later (wider) stages take the deeper trees
    root <<= p.depth[j];
  }
  p.n_stages = 1 + n_sub;
  return p;
}

// Stage that launch `launch` (0 .. n_stages - 1) performs for a tensor.
TA_HD uint32_t resize_stage_of_launch(const ResizePlan& p, uint32_t launch, bool narrowing) {
  return narrowing ? launch : p.n_stages - 1u - launch;
}

// Workgroups one tensor needs in a stage (stage 0: one).
TA_HD uint32_t resize_stage_roots(const ResizePlan& p, uint32_t stage) { return stage == 0 ? 1u : p.root[stage]; }

// Stage 0: chunks [0, min(top, n_chunks)), ascending when narrowing, descending when widening.
// `chunk_op(c)` must load the chunk, pass a workgroup barrier, then store it.
template <class ChunkOp>
TA_HD void resize_walk_top(const ResizePlan& p, uint32_t n_chunks, bool narrowing, ChunkOp&& chunk_op) {
  const uint32_t n = n_chunks < p.top ? n_chunks : p.top;
  for (uint32_t i = 0; i < n; ++i) chunk_op(narrowing ? i : n - 1u - i);
}

// Stage j >= 1, workgroup `r` (0 <= r < root[j]) of a tensor: the subtree of chunk root[j] + r.
// `chunk_op(c)` loads and stores one chunk (its loads and stores never overlap: c >= 1);
// `level_done()` is the workgroup barrier between two levels.
template <class ChunkOp, class LevelDone>
TA_HD void resize_walk_subtree(const ResizePlan& p, uint32_t stage, uint32_t r, uint32_t n_chunks, bool narrowing,
                               ChunkOp&& chunk_op, LevelDone&& level_done) {
  const uint32_t first = p.root[stage] + r, depth = p.depth[stage];
  for (uint32_t i = 0; i < depth; ++i) {
    const uint32_t v = narrowing ? i : depth - 1u - i;
    const uint64_t lo = (uint64_t)first << v;
    if (lo >= n_chunks) {
      if (narrowing) break;  // deeper levels lie further out still
      continue;
    }
    const uint64_t end = lo + ((uint64_t)1 << v);
    const uint32_t hi = end < n_chunks ? (uint32_t)end : n_chunks;
    for (uint32_t c = (uint32_t)lo; c < hi; ++c) chunk_op(c);
    level_done();
  }
}

}  // namespace triaccel

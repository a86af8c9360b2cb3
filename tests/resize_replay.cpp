// Host-side replay of the in-place resize schedule (csrc/resize_schedule.h): lists, for one tensor,
// every load, barrier and store in the order each workgroup of each launch performs them.
// Compiled with g++ by tests/test_resize_schedule.py; no GPU code.
#include <stdint.h>

#include "../paper_2508_16905_amd/csrc/resize_schedule.h"

using namespace triaccel;

// Rows of five int32: launch, workgroup (of this tensor), kind (0 load, 1 barrier, 2 store), chunk, stage.
// Returns the number of rows (also when it exceeds `cap`; only `cap` rows are written).
extern "C" int64_t resize_replay(uint32_t max_chunks, uint32_t total_chunks, uint32_t n_chunks, int narrowing,
                                 int32_t* out, int64_t cap) {
  const ResizePlan p = make_resize_plan(max_chunks, total_chunks);
  int64_t n = 0;
  auto emit = [&](uint32_t launch, uint32_t wg, int kind, uint32_t chunk, uint32_t stage) {
    if (n < cap) {
      int32_t* row = out + 5 * n;
      row[0] = (int32_t)launch; row[1] = (int32_t)wg; row[2] = kind; row[3] = (int32_t)chunk; row[4] = (int32_t)stage;
    }
    ++n;
  };
  for (uint32_t launch = 0; launch < p.n_stages; ++launch) {
    const uint32_t stage = resize_stage_of_launch(p, launch, narrowing != 0);
    if (stage == 0) {
      resize_walk_top(p, n_chunks, narrowing != 0, [&](uint32_t c) {
        emit(launch, 0, 0, c, stage);
        emit(launch, 0, 1, c, stage);
        emit(launch, 0, 2, c, stage);
      });
    } else {
      for (uint32_t r = 0; r < resize_stage_roots(p, stage); ++r) {
        resize_walk_subtree(p, stage, r, n_chunks, narrowing != 0,
                            [&](uint32_t c) {
                              emit(launch, r, 0, c, stage);
                              emit(launch, r, 2, c, stage);
                            },
                            [&]() { emit(launch, r, 1, 0, stage); });
      }
    }
  }
  return n;
}

extern "C" void resize_plan(uint32_t max_chunks, uint32_t total_chunks, uint32_t* out /* 2 + 2 * 8 words */) {
  const ResizePlan p = make_resize_plan(max_chunks, total_chunks);
  out[0] = p.n_stages;
  out[1] = p.top;
  for (uint32_t j = 0; j < kResizeMaxStages; ++j) {
    out[2 + j] = p.root[j];
    out[2 + kResizeMaxStages + j] = p.depth[j];
  }
}

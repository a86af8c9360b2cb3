// Power iteration for the top-k eigenvalues of each layer's Hessian (Sec. 3.2, third equation):
// device tables and host-callable launchers (defined in power.hip).
#pragma once
#include <hip/hip_runtime.h>

#include "common.h"

namespace triaccel {

constexpr int kMaxPowerK = 8;  // vectors per layer the workspace can be sized for
constexpr int kPowerSeg = 8;   // chunks of one tensor that one workgroup of the Gram pass sums

// Doubles one workgroup of the Gram pass leaves for k vectors: the upper triangle of W^T W
// (W = [H u_0 .. H u_{k-1}]), then u_j . (H u_j), then u_j . u_j.
constexpr int power_partial_len(int k) { return k * (k + 1) / 2 + 2 * k; }

// Per tensor: the k vectors of one call.  Vector j occupies elements [j * stride, j * stride + numel).
struct PowerDesc {
  float* u;
  const float* hu;
  int64_t stride;
};

struct SegRef {
  uint32_t tensor;
  uint32_t index;  // segment number inside the tensor: chunks [index * kPowerSeg, (index + 1) * kPowerSeg)
};

// Per-tensor result of the last call.
struct PowerLayer {
  // q_j = sum_{i <= j} coef[i][j] * (H u_i): the orthonormalisation in terms of the supplied vectors
  double coef[kMaxPowerK][kMaxPowerK];
  float rayleigh[kMaxPowerK];
  float resid[kMaxPowerK];
  float hnorm[kMaxPowerK];
  uint32_t deficient;
  float lambda_max;  // max_j |rayleigh_j| of this call
};

struct PowerTables {
  const TensorDesc* tensors;  // numel and chunk counts (shared with the optimizer step)
  const ChunkRef* chunks;
  LayerDev* layers;
  PowerDesc* descs;
  SegRef* segs;
  uint32_t* seg_first;  // per tensor: index of its first segment
  double* partials;     // total_segs x power_partial_len(k)
  PowerLayer* state;
  uint32_t n_tensors;
  uint32_t total_chunks;
  uint32_t total_segs;
};

// One iteration on k vectors per tensor: Gram pass, per-layer factorisation, apply pass.  With
// `ev` (four events) the boundaries of the three kernels are recorded on the stream.
hipError_t launch_power_iter(const PowerTables& t, int k, int latch, hipStream_t s, hipEvent_t* ev);

// The same iteration without a handle and without any allocation: tables and partial sums live in a
// fixed device array of this library (one per GPU), rebuilt by a small kernel on every call.
constexpr int kStaticMaxTensors = 256;      // tensors per call
constexpr int kStaticMaxChunks = 65536;     // sum over the tensors of ceil(numel / kChunk): 268,435,456 elements
constexpr int kStaticBatch = 64;            // tensor descriptions handed to the table kernel per launch

struct StaticTensor {
  float* u;
  const float* hu;
  int64_t stride;
  int64_t numel;
};

// Exported per-tensor record (layout of triaccel_power_info).
struct PowerInfoOut {
  float rayleigh[kMaxPowerK];
  float resid[kMaxPowerK];
  float hnorm[kMaxPowerK];
  uint32_t deficient;
  float lambda_max;
  float lambda_latched;
};

// Looks up (once per device) the address of the fixed array on the current device.
hipError_t power_static_prepare();
// `tensors` is a host array of n entries; `info` a device array of n records.  The caller has checked
// the limits above.  Calls on one GPU share the array: they must not overlap in time.
hipError_t launch_power_iter_static(const StaticTensor* tensors, int n, int k, PowerInfoOut* info, hipStream_t s);

}  // namespace triaccel

// Body of the fused update + cast, shared by the kernels that apply it in place (update.hip) and
// stage by stage while the storage size changes (update_resize.hip).
#pragma once
#include "device_util.h"

namespace triaccel {

// ---------------------------------------------------------------------------------------------
// Stage 5: fused update + cast.  Per element, fp32:
//   theta = widen(param);  gt = widen(g) * inv_scale;  d = fma(wd, theta, gt);
//   m = fma(mu, m, d) (m = d without a buffer);  theta' = fma(-eta, m, theta);
//   store theta' in the layer's new precision, round to nearest even.
// The body comes in two halves -- load + arithmetic into registers, then the stores -- so that a
// kernel that rewrites a tensor in place at another element size can put its one workgroup barrier
// between them, at a single place that every thread passes.
// ELEM: the step size is scaled per element instead of per layer (Sec. 3.2, "Step size scaling",
// applied to each entry of the sparsified curvature): eta_i = lr / fma(alpha, a_i, 1) with
// a_i = |h_i| if the entry is in the mask (|h_i| >= theta and |h_i| > 0), else 0; reads h once more.
// ---------------------------------------------------------------------------------------------
struct StepSize {
  float neg_eta;       // per-layer form: -eta_l
  float lr, alpha;     // element-wise form
  uint32_t theta_key;  // element-wise form: bit pattern of the mask threshold
};

// New parameter values and momentum of a lane's 16 elements of one chunk.
struct ChunkRegs {
  float th[kRows][4];
  float m[kRows][4];
};

template <int GD, int PD, bool FULL, bool MOM, bool ELEM>
__device__ __forceinline__ void update_load(const TensorDesc& td, int64_t base, float inv_scale, float wd, float mu,
                                            const StepSize& ss, int tid, ChunkRegs& r) {
  float g[kRows][4], h[ELEM ? kRows : 1][4];
  // Row by row, the arrays interleaved.  (Measured over 48 placements of the arrays in memory each,
  // with the accesses in the global address space: issuing the loads array by array instead is 2 %
  // slower on average, rotating the row order between the arrays changes nothing.)
#pragma unroll
  for (int q = 0; q < kRows; ++q) {
    const int64_t idx = base + q * kRowElems + tid * kVec;
    if constexpr (FULL) {
      load4<GD>(td.grad, idx, g[q]);
      load4<PD>(td.param, idx, r.th[q]);
      if constexpr (MOM) load4<kFP32>(td.mom, idx, r.m[q]);
      if constexpr (ELEM) load4<kFP32>(td.curv, idx, h[q]);
    } else {
      load4_guard<GD>(td.grad, idx, td.numel, 0.0f, g[q]);
      load4_guard<PD>(td.param, idx, td.numel, 0.0f, r.th[q]);
      if constexpr (MOM) load4_guard<kFP32>(td.mom, idx, td.numel, 0.0f, r.m[q]);
      if constexpr (ELEM) load4_guard<kFP32>(td.curv, idx, td.numel, 0.0f, h[q]);
    }
  }
#pragma unroll
  for (int q = 0; q < kRows; ++q) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float gt = g[q][i] * inv_scale;
      const float d = fmaf(wd, r.th[q][i], gt);
      const float mm = MOM ? fmaf(mu, r.m[q][i], d) : d;
      r.m[q][i] = mm;
      float neg_eta = ss.neg_eta;
      if constexpr (ELEM) {
        const uint32_t key = f2u(h[q][i]) & 0x7fffffffu;
        const float a = (key >= ss.theta_key && key != 0u) ? u2f(key) : 0.0f;
        const float den = fmaf(ss.alpha, a, 1.0f);
        neg_eta = -(ss.lr / den);
      }
      r.th[q][i] = fmaf(neg_eta, mm, r.th[q][i]);
    }
  }
}

template <int ND, bool FULL, bool MOM>
__device__ __forceinline__ void update_store(const TensorDesc& td, int64_t base, int tid, const ChunkRegs& r) {
#pragma unroll
  for (int q = 0; q < kRows; ++q) {
    const int64_t idx = base + q * kRowElems + tid * kVec;
    if constexpr (FULL) {
      store4<ND>(td.param, idx, r.th[q]);
      if constexpr (MOM) store4<kFP32>(td.mom, idx, r.m[q]);
    } else {
      store4_guard<ND>(td.param, idx, td.numel, r.th[q]);
      if constexpr (MOM) store4_guard<kFP32>(td.mom, idx, td.numel, r.m[q]);
    }
  }
}

// Gradient, old and new precision are uniform over a workgroup: each half branches once per chunk
// into a body specialised for its combination.
template <bool ELEM, int GD, int PD>
__device__ __forceinline__ void update_load2(const TensorDesc& td, int64_t base, float inv_scale, float wd, float mu,
                                             const StepSize& ss, int tid, ChunkRegs& r) {
  const bool full = base + kChunk <= td.numel;
  const bool mom = td.mom != nullptr;
  if (full) {
    if (mom) update_load<GD, PD, true, true, ELEM>(td, base, inv_scale, wd, mu, ss, tid, r);
    else update_load<GD, PD, true, false, ELEM>(td, base, inv_scale, wd, mu, ss, tid, r);
  } else {
    if (mom) update_load<GD, PD, false, true, ELEM>(td, base, inv_scale, wd, mu, ss, tid, r);
    else update_load<GD, PD, false, false, ELEM>(td, base, inv_scale, wd, mu, ss, tid, r);
  }
}

template <bool ELEM, int GD>
__device__ __forceinline__ void update_load1(int pd, const TensorDesc& td, int64_t base, float inv_scale, float wd,
                                             float mu, const StepSize& ss, int tid, ChunkRegs& r) {
  switch (pd) {
    case kFP32: update_load2<ELEM, GD, kFP32>(td, base, inv_scale, wd, mu, ss, tid, r); break;
    case kBF16: update_load2<ELEM, GD, kBF16>(td, base, inv_scale, wd, mu, ss, tid, r); break;
    default: update_load2<ELEM, GD, kFP16>(td, base, inv_scale, wd, mu, ss, tid, r); break;
  }
}

template <bool ELEM>
__device__ __forceinline__ void update_load_any(const TensorDesc& td, int pd, int64_t base, float inv_scale, float wd,
                                                float mu, const StepSize& ss, int tid, ChunkRegs& r) {
  switch (td.grad_dtype) {
    case kFP32: update_load1<ELEM, kFP32>(pd, td, base, inv_scale, wd, mu, ss, tid, r); break;
    case kBF16: update_load1<ELEM, kBF16>(pd, td, base, inv_scale, wd, mu, ss, tid, r); break;
    default: update_load1<ELEM, kFP16>(pd, td, base, inv_scale, wd, mu, ss, tid, r); break;
  }
}

template <int ND>
__device__ __forceinline__ void update_store1(const TensorDesc& td, int64_t base, int tid, const ChunkRegs& r) {
  const bool full = base + kChunk <= td.numel;
  const bool mom = td.mom != nullptr;
  if (full) {
    if (mom) update_store<ND, true, true>(td, base, tid, r);
    else update_store<ND, true, false>(td, base, tid, r);
  } else {
    if (mom) update_store<ND, false, true>(td, base, tid, r);
    else update_store<ND, false, false>(td, base, tid, r);
  }
}

__device__ __forceinline__ void update_store_any(const TensorDesc& td, int nd, int64_t base, int tid,
                                                 const ChunkRegs& r) {
  switch (nd) {
    case kFP32: update_store1<kFP32>(td, base, tid, r); break;
    case kBF16: update_store1<kBF16>(td, base, tid, r); break;
    default: update_store1<kFP16>(td, base, tid, r); break;
  }
}

// One chunk, loads then stores, for the kernels in which they cannot overlap.
template <bool ELEM>
__device__ __forceinline__ void update_any(const TensorDesc& td, int pd, int nd, int64_t base, float inv_scale,
                                           float wd, float mu, const StepSize& ss, int tid) {
  ChunkRegs r;
  update_load_any<ELEM>(td, pd, base, inv_scale, wd, mu, ss, tid, r);
  update_store_any(td, nd, base, tid, r);
}

}  // namespace triaccel

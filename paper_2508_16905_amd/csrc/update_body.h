// Body of the fused update + cast, shared by the kernels that apply it in place (update.hip) and
// phase by phase while the storage size changes (update_resize.hip).
#pragma once
#include "device_util.h"

namespace triaccel {

// ---------------------------------------------------------------------------------------------
// Stage 5: fused update + cast.  Per element, fp32:
//   theta = widen(param);  gt = widen(g) * inv_scale;  d = fma(wd, theta, gt);
//   m = fma(mu, m, d) (m = d without a buffer);  theta' = fma(-eta, m, theta);
//   store theta' in the layer's new precision, round to nearest even.
// All loads of a chunk complete before its first store (needed when the storage size changes
// in place, harmless otherwise).
// ELEM: the step size is scaled per element instead of per layer (Sec. 3.2, "Step size scaling",
// applied to each entry of the sparsified curvature): eta_i = lr / fma(alpha, a_i, 1) with
// a_i = |h_i| if the entry is in the mask (|h_i| >= theta and |h_i| > 0), else 0; reads h once more.
// ---------------------------------------------------------------------------------------------
struct StepSize {
  float neg_eta;       // per-layer form: -eta_l
  float lr, alpha;     // element-wise form
  uint32_t theta_key;  // element-wise form: bit pattern of the mask threshold
};

template <int GD, int PD, int ND, bool FULL, bool MOM, bool ELEM>
__device__ __forceinline__ void update_chunk(const TensorDesc& td, int64_t base, float inv_scale, float wd, float mu,
                                             const StepSize& ss, bool barrier, int tid) {
  float g[kRows][4], th[kRows][4], m[kRows][4], h[ELEM ? kRows : 1][4];
#pragma unroll
  for (int r = 0; r < kRows; ++r) {
    const int64_t idx = base + r * kRowElems + tid * kVec;
    if (FULL) {
      load4<GD>(td.grad, idx, g[r]);
      load4<PD>(td.param, idx, th[r]);
      if (MOM) load4<kFP32>(td.mom, idx, m[r]);
      if constexpr (ELEM) load4<kFP32>(td.curv, idx, h[r]);
    } else {
      load4_guard<GD>(td.grad, idx, td.numel, 0.0f, g[r]);
      load4_guard<PD>(td.param, idx, td.numel, 0.0f, th[r]);
      if (MOM) load4_guard<kFP32>(td.mom, idx, td.numel, 0.0f, m[r]);
      if constexpr (ELEM) load4_guard<kFP32>(td.curv, idx, td.numel, 0.0f, h[r]);
    }
  }
#pragma unroll
  for (int r = 0; r < kRows; ++r) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float gt = g[r][i] * inv_scale;
      const float d = fmaf(wd, th[r][i], gt);
      const float mm = MOM ? fmaf(mu, m[r][i], d) : d;
      m[r][i] = mm;
      float neg_eta = ss.neg_eta;
      if constexpr (ELEM) {
        const uint32_t key = f2u(h[r][i]) & 0x7fffffffu;
        const float a = (key >= ss.theta_key && key != 0u) ? u2f(key) : 0.0f;
        const float den = fmaf(ss.alpha, a, 1.0f);
        neg_eta = -(ss.lr / den);
      }
      th[r][i] = fmaf(neg_eta, mm, th[r][i]);
    }
  }
  if (barrier) __syncthreads();
#pragma unroll
  for (int r = 0; r < kRows; ++r) {
    const int64_t idx = base + r * kRowElems + tid * kVec;
    if (FULL) {
      store4<ND>(td.param, idx, th[r]);
      if (MOM) store4<kFP32>(td.mom, idx, m[r]);
    } else {
      store4_guard<ND>(td.param, idx, td.numel, th[r]);
      if (MOM) store4_guard<kFP32>(td.mom, idx, td.numel, m[r]);
    }
  }
}

template <bool ELEM, int GD, int PD, int ND>
__device__ __forceinline__ void update_dispatch2(const TensorDesc& td, int64_t base, float inv_scale, float wd,
                                                 float mu, const StepSize& ss, bool barrier, int tid) {
  const bool full = base + kChunk <= td.numel;
  const bool mom = td.mom != nullptr;
  if (full) {
    if (mom) update_chunk<GD, PD, ND, true, true, ELEM>(td, base, inv_scale, wd, mu, ss, barrier, tid);
    else update_chunk<GD, PD, ND, true, false, ELEM>(td, base, inv_scale, wd, mu, ss, barrier, tid);
  } else {
    if (mom) update_chunk<GD, PD, ND, false, true, ELEM>(td, base, inv_scale, wd, mu, ss, barrier, tid);
    else update_chunk<GD, PD, ND, false, false, ELEM>(td, base, inv_scale, wd, mu, ss, barrier, tid);
  }
}

template <bool ELEM, int GD, int PD>
__device__ __forceinline__ void update_dispatch1(int nd, const TensorDesc& td, int64_t base, float inv_scale,
                                                 float wd, float mu, const StepSize& ss, bool barrier, int tid) {
  switch (nd) {
    case kFP32: update_dispatch2<ELEM, GD, PD, kFP32>(td, base, inv_scale, wd, mu, ss, barrier, tid); break;
    case kBF16: update_dispatch2<ELEM, GD, PD, kBF16>(td, base, inv_scale, wd, mu, ss, barrier, tid); break;
    default: update_dispatch2<ELEM, GD, PD, kFP16>(td, base, inv_scale, wd, mu, ss, barrier, tid); break;
  }
}

template <bool ELEM, int GD>
__device__ __forceinline__ void update_dispatch0(int pd, int nd, const TensorDesc& td, int64_t base,
                                                 float inv_scale, float wd, float mu, const StepSize& ss,
                                                 bool barrier, int tid) {
  switch (pd) {
    case kFP32: update_dispatch1<ELEM, GD, kFP32>(nd, td, base, inv_scale, wd, mu, ss, barrier, tid); break;
    case kBF16: update_dispatch1<ELEM, GD, kBF16>(nd, td, base, inv_scale, wd, mu, ss, barrier, tid); break;
    default: update_dispatch1<ELEM, GD, kFP16>(nd, td, base, inv_scale, wd, mu, ss, barrier, tid); break;
  }
}

// Gradient, old and new precision are uniform over a workgroup: branch once per chunk into a body
// specialised for the combination.
template <bool ELEM>
__device__ __forceinline__ void update_any(const TensorDesc& td, int pd, int nd, int64_t base, float inv_scale,
                                           float wd, float mu, const StepSize& ss, bool barrier, int tid) {
  switch (td.grad_dtype) {
    case kFP32: update_dispatch0<ELEM, kFP32>(pd, nd, td, base, inv_scale, wd, mu, ss, barrier, tid); break;
    case kBF16: update_dispatch0<ELEM, kBF16>(pd, nd, td, base, inv_scale, wd, mu, ss, barrier, tid); break;
    default: update_dispatch0<ELEM, kFP16>(pd, nd, td, base, inv_scale, wd, mu, ss, barrier, tid); break;
  }
}

}  // namespace triaccel

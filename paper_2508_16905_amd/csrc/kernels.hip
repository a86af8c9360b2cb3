// gfx950 kernels of the Tri-Accel optimizer step.
//
// Every kernel streams tensors in chunks of kChunk = 4096 elements: four rows of 256 lanes, each
// lane holding 4 consecutive elements (one 128-bit access per lane, row and fp32 array).  All
// arithmetic that decides a stored value is fp32 with an explicit operation order (fmaf where a
// fused multiply-add is meant; the file is compiled with -ffp-contract=off); reductions are fp64.
#include "kernels.h"

#include <hip/hip_runtime.h>

#include "numerics.h"

namespace triaccel {

// ---------------------------------------------------------------------------------------------
// wavefront (64 lanes) helpers
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}
__device__ __forceinline__ uint32_t wave_max(uint32_t v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = max(v, (uint32_t)__shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ uint32_t wave_or(uint32_t v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v |= (uint32_t)__shfl_xor(v, o);
  return v;
}

__device__ __forceinline__ bool step_skipped(const GlobalDev* glob, uint32_t step_id) {
  return *reinterpret_cast<const volatile uint32_t*>(&glob->skip_epoch) == step_id;
}

__device__ __forceinline__ uint32_t elem_size(int code) { return code == kFP32 ? 4u : 2u; }

// (count, mean, M2) merge of two disjoint samples (Chan et al.), fp64.
struct Moments {
  double n, mean, m2;
};
__device__ __forceinline__ Moments merge(const Moments& a, const Moments& b) {
  if (b.n == 0.0) return a;
  if (a.n == 0.0) return b;
  Moments r;
  r.n = a.n + b.n;
  const double delta = b.mean - a.mean;
  const double w = b.n / r.n;
  r.mean = a.mean + delta * w;
  r.m2 = a.m2 + b.m2 + delta * delta * a.n * w;
  return r;
}
__device__ __forceinline__ Moments shfl_down(const Moments& m, int o) {
  Moments r;
  r.n = __shfl_down(m.n, o);
  r.mean = __shfl_down(m.mean, o);
  r.m2 = __shfl_down(m.m2, o);
  return r;
}

// ---------------------------------------------------------------------------------------------
// Stage 1: per-chunk gradient moments and non-finite scan (Sec. 3.1, Var[grad_l(t)]).
// One workgroup per chunk.  Each lane accumulates shifted sums of its 16 unscaled values in fp64,
// lanes / wavefronts are merged pairwise in a fixed order, one (mean, M2) partial per chunk.
// ---------------------------------------------------------------------------------------------
template <int GD, bool FULL>
__device__ __forceinline__ void stats_chunk(const TensorDesc& td, int64_t base, float inv_scale, Moments& mom,
                                            uint32_t& bad) {
  const int tid = threadIdx.x;
  float g[kRows][4];
#pragma unroll
  for (int r = 0; r < kRows; ++r) {
    const int64_t idx = base + r * kRowElems + tid * kVec;
    if (FULL) load4<GD>(td.grad, idx, g[r]);
    else load4_guard<GD>(td.grad, idx, td.numel, 0.0f, g[r]);
  }
  double shift = 0.0, s1 = 0.0, s2 = 0.0;
  int cnt = 0;
#pragma unroll
  for (int r = 0; r < kRows; ++r) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int64_t idx = base + r * kRowElems + tid * kVec + i;
      if (FULL || idx < td.numel) {
        const float raw = g[r][i];
        bad |= ((f2u(raw) & 0x7f800000u) == 0x7f800000u) ? 1u : 0u;
        const double x = (double)(raw * inv_scale);
        if (cnt == 0) shift = x;
        const double d = x - shift;
        s1 += d;
        s2 = fma(d, d, s2);
        ++cnt;
      }
    }
  }
  mom.n = (double)cnt;
  if (cnt > 0) {
    mom.mean = shift + s1 / (double)cnt;
    mom.m2 = s2 - s1 * s1 / (double)cnt;
  } else {
    mom.mean = 0.0;
    mom.m2 = 0.0;
  }
}

__global__ __launch_bounds__(kThreads) void k_grad_stats(const TensorDesc* __restrict__ tds,
                                                         const ChunkRef* __restrict__ chunks,
                                                         StatPartial* __restrict__ partials, LayerDev* layers,
                                                         GlobalDev* glob, StepScalars sc) {
  const ChunkRef cr = chunks[blockIdx.x];
  const TensorDesc td = tds[cr.tensor];
  const int64_t base = (int64_t)cr.index * kChunk;
  const bool full = base + kChunk <= td.numel;
  Moments mom;
  uint32_t bad = 0;
  if (full) {
    switch (td.grad_dtype) {
      case kFP32: stats_chunk<kFP32, true>(td, base, sc.inv_scale, mom, bad); break;
      case kBF16: stats_chunk<kBF16, true>(td, base, sc.inv_scale, mom, bad); break;
      default: stats_chunk<kFP16, true>(td, base, sc.inv_scale, mom, bad); break;
    }
  } else {
    switch (td.grad_dtype) {
      case kFP32: stats_chunk<kFP32, false>(td, base, sc.inv_scale, mom, bad); break;
      case kBF16: stats_chunk<kBF16, false>(td, base, sc.inv_scale, mom, bad); break;
      default: stats_chunk<kFP16, false>(td, base, sc.inv_scale, mom, bad); break;
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mom = merge(mom, shfl_down(mom, o));
  bad = wave_or(bad);
  __shared__ Moments s_m[kThreads / kWave];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  if (lane == 0) {
    s_m[wave] = mom;
    if (bad) {
      atomicExch(&layers[cr.tensor].found_epoch, sc.step_id);
      atomicExch(&glob->skip_epoch, sc.step_id);
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    Moments t = s_m[0];
#pragma unroll
    for (int w = 1; w < kThreads / kWave; ++w) t = merge(t, s_m[w]);
    partials[blockIdx.x].mean = t.mean;
    partials[blockIdx.x].m2 = t.m2;
  }
}

// ---------------------------------------------------------------------------------------------
// Histogram window helpers (radix select on 31-bit magnitude keys).
// ---------------------------------------------------------------------------------------------
struct Window {
  uint32_t lo, shift, bins;
};

// Flush a workgroup's LDS histogram and per-lane accumulators to the tensor's global ones.
__device__ __forceinline__ void flush_hist(uint32_t* s_hist, uint32_t bins, uint32_t* g_hist) {
  __syncthreads();
  for (uint32_t b = threadIdx.x; b < bins; b += kThreads) {
    const uint32_t v = s_hist[b];
    if (v) {
      atomicAdd(&g_hist[b], v);
      s_hist[b] = 0;
    }
  }
  __syncthreads();
}

// ---------------------------------------------------------------------------------------------
// Stage 2: curvature EMA (diagonal Hutchinson signal of Sec. 3.2) fused with the first
// histogram pass of the threshold selection.  Persistent workgroups, each owning a contiguous
// range of chunks so that the LDS histogram is flushed once per (workgroup, tensor).
// Per element, fp32:  u = (z * hz) * inv_scale;  h = u on the tensor's first probe, else
// h = fma(beta_h, h, (1 - beta_h) * u);  a non-finite u leaves h unchanged.
// ---------------------------------------------------------------------------------------------
template <bool FULL>
__device__ __forceinline__ void ema_chunk(const TensorDesc& td, int64_t base, float inv_scale, float beta_h,
                                          float omb_h, bool first, const Window& w, uint32_t* s_hist,
                                          uint32_t& above, uint32_t& zeros, uint32_t& maxkey, uint32_t& nonfin) {
  const int tid = threadIdx.x;
  float z[kRows][4], hz[kRows][4], h[kRows][4];
#pragma unroll
  for (int r = 0; r < kRows; ++r) {
    const int64_t idx = base + r * kRowElems + tid * kVec;
    if (FULL) {
      load4<kFP32>(td.z, idx, z[r]);
      load4<kFP32>(td.hz, idx, hz[r]);
      load4<kFP32>(td.curv, idx, h[r]);
    } else {
      load4_guard<kFP32>(td.z, idx, td.numel, 0.0f, z[r]);
      load4_guard<kFP32>(td.hz, idx, td.numel, 0.0f, hz[r]);
      load4_guard<kFP32>(td.curv, idx, td.numel, 0.0f, h[r]);
    }
  }
#pragma unroll
  for (int r = 0; r < kRows; ++r) {
    const int64_t idx = base + r * kRowElems + tid * kVec;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float u = z[r][i] * hz[r][i];
      u = u * inv_scale;
      float hn = h[r][i];
      if ((f2u(u) & 0x7f800000u) == 0x7f800000u) {
        if (FULL || idx + i < td.numel) nonfin = 1u;
      } else if (first) {
        hn = u;
      } else {
        const float p = omb_h * u;
        hn = fmaf(beta_h, hn, p);
      }
      h[r][i] = hn;
      if (FULL || idx + i < td.numel) {
        const uint32_t key = f2u(hn) & 0x7fffffffu;
        maxkey = max(maxkey, key);
        if (key == 0u) {
          ++zeros;
        } else if (key >= w.lo) {
          const uint32_t bin = (key - w.lo) >> w.shift;
          if (bin < w.bins) atomicAdd(&s_hist[bin], 1u);
          else ++above;
        }
      }
    }
    if (FULL) store4<kFP32>(td.curv, idx, h[r]);
    else store4_guard<kFP32>(td.curv, idx, td.numel, h[r]);
  }
}

__global__ __launch_bounds__(kThreads) void k_curv_ema_hist(const TensorDesc* __restrict__ tds,
                                                            const ChunkRef* __restrict__ chunks,
                                                            uint32_t total_chunks, LayerDev* layers,
                                                            const GlobalDev* glob, uint32_t* hist, StepScalars sc,
                                                            float beta_h, float omb_h) {
  if (step_skipped(glob, sc.step_id)) return;
  __shared__ uint32_t s_hist[kHistBins];
  for (int b = threadIdx.x; b < kHistBins; b += kThreads) s_hist[b] = 0;
  __syncthreads();
  const uint32_t per = (total_chunks + gridDim.x - 1) / gridDim.x;
  const uint32_t c0 = blockIdx.x * per;
  const uint32_t c1 = min(c0 + per, total_chunks);
  int cur = -1;
  bool active = false, first = false;
  Window w{0, 0, 0};
  TensorDesc td;
  uint32_t above = 0, zeros = 0, maxkey = 0, nonfin = 0;
  for (uint32_t c = c0; c <= c1; ++c) {
    const bool end = (c == c1);
    const int t = end ? -2 : (int)chunks[c].tensor;
    if (t != cur) {
      if (cur >= 0 && active) {
        flush_hist(s_hist, w.bins, hist + (size_t)cur * kHistBins);
        above = wave_sum(above);
        zeros = wave_sum(zeros);
        maxkey = wave_max(maxkey);
        nonfin = wave_or(nonfin);
        if ((threadIdx.x & (kWave - 1)) == 0) {
          LayerDev& ls = layers[cur];
          if (above) atomicAdd(&ls.acc_above, above);
          if (zeros) atomicAdd(&ls.acc_zeros, zeros);
          if (maxkey) atomicMax(&ls.acc_maxkey, maxkey);
          if (nonfin) atomicOr(&ls.acc_nonfinite, 1u);
        }
      }
      if (end) break;
      cur = t;
      td = tds[t];
      active = td.has_probe != 0;
      const LayerDev& ls = layers[t];
      w = Window{ls.win_lo, ls.win_shift, ls.win_bins};
      first = ls.probes_seen == 0;
      above = zeros = maxkey = nonfin = 0;
    }
    if (!active) continue;
    const int64_t base = (int64_t)chunks[c].index * kChunk;
    if (base + kChunk <= td.numel)
      ema_chunk<true>(td, base, sc.inv_scale, beta_h, omb_h, first, w, s_hist, above, zeros, maxkey, nonfin);
    else
      ema_chunk<false>(td, base, sc.inv_scale, beta_h, omb_h, first, w, s_hist, above, zeros, maxkey, nonfin);
  }
}

// ---------------------------------------------------------------------------------------------
// Stage 3a: one more histogram pass over |h| for tensors whose window still holds too many keys
// to list (mode kSelHist after a scan).  Same chunk ownership as stage 2; reads h only.
// ---------------------------------------------------------------------------------------------
template <bool FULL>
__device__ __forceinline__ void hist_chunk(const TensorDesc& td, int64_t base, const Window& w, uint32_t* s_hist) {
  const int tid = threadIdx.x;
  float h[kRows][4];
#pragma unroll
  for (int r = 0; r < kRows; ++r) {
    const int64_t idx = base + r * kRowElems + tid * kVec;
    if (FULL) load4<kFP32>(td.curv, idx, h[r]);
    else load4_guard<kFP32>(td.curv, idx, td.numel, 0.0f, h[r]);
  }
#pragma unroll
  for (int r = 0; r < kRows; ++r) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t key = f2u(h[r][i]) & 0x7fffffffu;  // guarded fill 0 is never counted
      if (key != 0u && key >= w.lo) {
        const uint32_t bin = (key - w.lo) >> w.shift;
        if (bin < w.bins) atomicAdd(&s_hist[bin], 1u);
      }
    }
  }
}

__global__ __launch_bounds__(kThreads) void k_hist_pass(const TensorDesc* __restrict__ tds,
                                                        const ChunkRef* __restrict__ chunks, uint32_t total_chunks,
                                                        const LayerDev* layers, const GlobalDev* glob,
                                                        uint32_t* hist, StepScalars sc) {
  if (step_skipped(glob, sc.step_id)) return;
  __shared__ uint32_t s_hist[kHistBins];
  for (int b = threadIdx.x; b < kHistBins; b += kThreads) s_hist[b] = 0;
  __syncthreads();
  const uint32_t per = (total_chunks + gridDim.x - 1) / gridDim.x;
  const uint32_t c0 = blockIdx.x * per;
  const uint32_t c1 = min(c0 + per, total_chunks);
  int cur = -1;
  bool active = false;
  Window w{0, 0, 0};
  TensorDesc td;
  uint32_t c = c0;
  while (c <= c1) {
    const bool end = (c == c1);
    const int t = end ? -2 : (int)chunks[c].tensor;
    if (t != cur) {
      if (cur >= 0 && active) flush_hist(s_hist, w.bins, hist + (size_t)cur * kHistBins);
      if (end) break;
      cur = t;
      td = tds[t];
      const LayerDev& ls = layers[t];
      active = td.has_probe != 0 && ls.mode == kSelHist && ls.passes > 0;
      w = Window{ls.win_lo, ls.win_shift, ls.win_bins};
      if (!active) {
        // jump over the rest of this tensor's chunks owned by this workgroup
        const uint32_t next = td.first_chunk + td.n_chunks;
        c = min(next, c1);
        continue;
      }
    }
    const int64_t base = (int64_t)chunks[c].index * kChunk;
    if (base + kChunk <= td.numel) hist_chunk<true>(td, base, w, s_hist);
    else hist_chunk<false>(td, base, w, s_hist);
    ++c;
  }
}

// ---------------------------------------------------------------------------------------------
// Rank search in an LDS histogram: find the bin, counted from the top, that holds the r-th
// largest key (1 <= r <= total).  All kThreads threads call it; results are broadcast.
// ---------------------------------------------------------------------------------------------
struct BinHit {
  uint32_t bin;     // bin holding the r-th largest key
  uint32_t higher;  // number of keys in bins above it
  uint32_t count;   // keys in that bin
};
__device__ BinHit find_rank_from_top(const uint32_t* s_hist, uint32_t bins, uint32_t r, uint32_t* s_part,
                                     uint32_t* s_out) {
  const uint32_t per = (bins + kThreads - 1) / kThreads;
  const uint32_t b0 = threadIdx.x * per;
  uint32_t sum = 0;
  for (uint32_t b = b0; b < min(b0 + per, bins); ++b) sum += s_hist[b];
  s_part[threadIdx.x] = sum;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t acc = 0;
    int t = kThreads - 1;
    for (; t > 0; --t) {
      if (acc + s_part[t] >= r) break;
      acc += s_part[t];
    }
    s_out[0] = (uint32_t)t;
    s_out[1] = acc;
  }
  __syncthreads();
  if (threadIdx.x == s_out[0]) {
    uint32_t acc = s_out[1];
    uint32_t b = min(b0 + per, bins);
    uint32_t found = b0, cnt = 0;
    while (b > b0) {
      --b;
      const uint32_t v = s_hist[b];
      if (acc + v >= r) {
        found = b;
        cnt = v;
        break;
      }
      acc += v;
    }
    s_out[2] = found;
    s_out[3] = acc;
    s_out[4] = cnt;
  }
  __syncthreads();
  BinHit hit{s_out[2], s_out[3], s_out[4]};
  __syncthreads();
  return hit;
}

__device__ __forceinline__ uint32_t topk_count(int64_t n, uint32_t s_ppm) {
  // k = n - floor(n * s / 1e6), clamped to [1, n]; n < 2^31 so the product fits 64 bits
  int64_t k = n - (int64_t)(((uint64_t)n * (uint64_t)s_ppm) / 1000000ull);
  if (k < 1) k = 1;
  if (k > n) k = n;
  return (uint32_t)k;
}

// ---------------------------------------------------------------------------------------------
// Stage 3 scan: one workgroup per tensor reads the tensor's histogram, clears it, and decides
// whether theta is now exact, lies in a range small enough to list, or needs a finer pass.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void k_select_scan(const TensorDesc* __restrict__ tds, LayerDev* layers,
                                                          const GlobalDev* glob, uint32_t* hist, StepScalars sc,
                                                          uint32_t sparsity_ppm) {
  if (step_skipped(glob, sc.step_id)) return;
  const uint32_t l = blockIdx.x;
  const TensorDesc td = tds[l];
  if (!td.has_probe) return;
  LayerDev& ls = layers[l];
  if (ls.mode != kSelHist) return;
  __shared__ uint32_t s_hist[kHistBins];
  __shared__ uint32_t s_part[kThreads];
  __shared__ uint32_t s_out[8];
  const uint32_t bins = ls.win_bins, lo = ls.win_lo, shift = ls.win_shift;
  uint32_t* gh = hist + (size_t)l * kHistBins;
  uint32_t local = 0;
  for (uint32_t b = threadIdx.x; b < kHistBins; b += kThreads) {
    const uint32_t v = (b < bins) ? gh[b] : 0u;
    s_hist[b] = v;
    local += v;
    if (v) gh[b] = 0;
  }
  local = wave_sum(local);
  if ((threadIdx.x & (kWave - 1)) == 0) s_part[threadIdx.x / kWave] = local;
  __syncthreads();
  const uint32_t in_window = s_part[0] + s_part[1] + s_part[2] + s_part[3];
  __syncthreads();

  uint32_t k, above;
  const bool first_scan = ls.passes == 0;
  if (first_scan) {
    const uint32_t nonzero = (uint32_t)td.numel - ls.acc_zeros;
    k = topk_count(td.numel, sparsity_ppm);
    above = ls.acc_above;
    if (k > nonzero) {  // fewer non-zero magnitudes than k: theta = 0, every non-zero entry is kept
      if (threadIdx.x == 0) {
        ls.nonzero = nonzero;
        ls.mode = kSelExact;
        ls.theta_key = 0;
        ls.above = nonzero;
        ls.sel_count = 0;
        ls.k_rem = k;
        ls.passes = 1;
      }
      return;
    }
    if (threadIdx.x == 0) ls.nonzero = nonzero;
  } else {
    k = ls.k_rem;
    above = ls.above;
  }
  // miss of a predicted window: theta lies above or below it -> restart with the full key range
  if (above >= k || above + in_window < k) {
    if (threadIdx.x == 0) {
      ls.mode = kSelHist;
      ls.win_lo = 0;
      ls.win_shift = kFullShift;
      ls.win_bins = kHistBins;
      ls.predicted = 0;
      ls.above = 0;
      ls.k_rem = k;
      ls.passes = 1;
    }
    return;
  }
  const BinHit hit = find_rank_from_top(s_hist, bins, k - above, s_part, s_out);
  if (threadIdx.x == 0) {
    const uint32_t new_above = above + hit.higher;
    const uint32_t new_lo = lo + (hit.bin << shift);
    ls.above = new_above;
    ls.k_rem = k;
    ls.sel_count = hit.count;
    ls.passes = ls.passes + 1;
    if (shift == 0) {
      ls.mode = kSelExact;
      ls.theta_key = new_lo;
    } else if (hit.count <= td.cand_cap) {
      ls.mode = kSelCand;
      ls.rng_lo = new_lo;
      ls.rng_hi = new_lo + (1u << shift);
    } else {
      const uint32_t ns = shift > (uint32_t)kHistBits ? shift - kHistBits : 0u;
      ls.mode = kSelHist;
      ls.win_lo = new_lo;
      ls.win_shift = ns;
      ls.win_bins = 1u << (shift - ns);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Stage 3 mask: one workgroup per chunk re-reads |h| and writes the bit mask.  Keys above the
// candidate range are kept, keys below dropped; keys inside it are appended to the tensor's
// candidate list and their bits are set afterwards by k_select_finish.
// ---------------------------------------------------------------------------------------------
template <bool FULL>
__device__ __forceinline__ void mask_chunk(const TensorDesc& td, int64_t base, uint32_t mode, uint32_t theta,
                                           uint32_t rng_lo, uint32_t rng_hi, LayerDev& ls, Candidate* cands) {
  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  float h[kRows][4];
#pragma unroll
  for (int r = 0; r < kRows; ++r) {
    const int64_t idx = base + r * kRowElems + tid * kVec;
    if (FULL) load4<kFP32>(td.curv, idx, h[r]);
    else load4_guard<kFP32>(td.curv, idx, td.numel, 0.0f, h[r]);
  }
  uint32_t word[kRows];
#pragma unroll
  for (int r = 0; r < kRows; ++r) {
    const int64_t idx = base + r * kRowElems + tid * kVec;
    uint32_t nib = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t key = f2u(h[r][i]) & 0x7fffffffu;  // guarded fill 0: never kept, never listed
      bool keep;
      if (mode == kSelExact) {
        keep = key >= theta && key != 0u;
      } else {
        keep = key >= rng_hi;
        if (key != 0u && key >= rng_lo && key < rng_hi) {
          const uint32_t slot = atomicAdd(&ls.cand_count, 1u);
          if (slot < td.cand_cap) cands[td.cand_offset + slot] = Candidate{(uint32_t)(idx + i), key};
        }
      }
      nib |= keep ? (1u << i) : 0u;
    }
    // eight consecutive lanes hold the 32 elements of one mask word
    uint32_t v = nib << (4 * (lane & 7));
    v |= (uint32_t)__shfl_xor(v, 1);
    v |= (uint32_t)__shfl_xor(v, 2);
    v |= (uint32_t)__shfl_xor(v, 4);
    word[r] = v;
  }
  const int64_t n_words = (td.numel + 31) >> 5;
  const int sub = lane & 7;
  if (sub < kRows) {
    uint32_t v = word[0];
#pragma unroll
    for (int r = 1; r < kRows; ++r) v = (sub == r) ? word[r] : v;
    const int64_t widx = ((base + (int64_t)sub * kRowElems) >> 5) + (tid >> 3);
    if (FULL || widx < n_words) td.mask[widx] = v;
  }
}

__global__ __launch_bounds__(kThreads) void k_mask(const TensorDesc* __restrict__ tds,
                                                   const ChunkRef* __restrict__ chunks, LayerDev* layers,
                                                   const GlobalDev* glob, Candidate* cands, StepScalars sc) {
  if (step_skipped(glob, sc.step_id)) return;
  const ChunkRef cr = chunks[blockIdx.x];
  const TensorDesc td = tds[cr.tensor];
  if (!td.has_probe) return;
  LayerDev& ls = layers[cr.tensor];
  const uint32_t mode = ls.mode;
  if (mode == kSelHist) return;  // cannot happen after the last scan; never write a mask from a stale range
  const uint32_t theta = ls.theta_key, lo = ls.rng_lo, hi = ls.rng_hi;
  const int64_t base = (int64_t)cr.index * kChunk;
  if (base + kChunk <= td.numel) mask_chunk<true>(td, base, mode, theta, lo, hi, ls, cands);
  else mask_chunk<false>(td, base, mode, theta, lo, hi, ls, cands);
}

// ---------------------------------------------------------------------------------------------
// Stage 3 finish: one workgroup per tensor resolves theta among the listed candidates (radix
// select in LDS), sets their mask bits, publishes theta / nnz / lambda and prepares the
// histogram window of the next probed step (centred on this theta).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void k_select_finish(const TensorDesc* __restrict__ tds, LayerDev* layers,
                                                            const GlobalDev* glob, const Candidate* cands,
                                                            StepScalars sc) {
  if (step_skipped(glob, sc.step_id)) return;
  const uint32_t l = blockIdx.x;
  const TensorDesc td = tds[l];
  if (!td.has_probe) return;
  LayerDev& ls = layers[l];
  __shared__ uint32_t s_hist[kHistBins];
  __shared__ uint32_t s_part[kThreads];
  __shared__ uint32_t s_out[8];
  const uint32_t mode = ls.mode;
  uint32_t theta = ls.theta_key;
  uint32_t nnz = ls.above + ls.sel_count;
  if (mode == kSelExact && theta == 0u) nnz = ls.nonzero;
  if (mode == kSelCand) {
    const Candidate* cl = cands + td.cand_offset;
    const uint32_t count = min(ls.cand_count, td.cand_cap);
    uint32_t lo = ls.rng_lo;
    uint32_t width_shift = 31u - (uint32_t)__clz(ls.rng_hi - ls.rng_lo);  // range width is a power of two
    uint32_t r = ls.k_rem - ls.above;
    while (width_shift > 0) {
      const uint32_t ns = width_shift > (uint32_t)kHistBits ? width_shift - kHistBits : 0u;
      const uint32_t bins = 1u << (width_shift - ns);
      for (uint32_t b = threadIdx.x; b < bins; b += kThreads) s_hist[b] = 0;
      __syncthreads();
      for (uint32_t i = threadIdx.x; i < count; i += kThreads) {
        const uint32_t key = cl[i].key;
        if (key >= lo && ((key - lo) >> width_shift) == 0u) atomicAdd(&s_hist[(key - lo) >> ns], 1u);
      }
      __syncthreads();
      const BinHit hit = find_rank_from_top(s_hist, bins, r, s_part, s_out);
      r -= hit.higher;
      lo += hit.bin << ns;
      width_shift = ns;
    }
    theta = lo;
    // set the bits of the candidates at or above theta
    uint32_t kept = 0;
    for (uint32_t i = threadIdx.x; i < count; i += kThreads) {
      const Candidate c = cl[i];
      if (c.key >= theta) {
        atomicOr(&td.mask[c.idx >> 5], 1u << (c.idx & 31u));
        ++kept;
      }
    }
    kept = wave_sum(kept);
    __syncthreads();
    if ((threadIdx.x & (kWave - 1)) == 0) s_part[threadIdx.x / kWave] = kept;
    __syncthreads();
    nnz = ls.above + s_part[0] + s_part[1] + s_part[2] + s_part[3];
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    ls.theta_key = theta;
    ls.theta = u2f(theta);
    ls.nnz = nnz;
    ls.lambda = u2f(ls.acc_maxkey);
    ls.curv_nonfinite = ls.acc_nonfinite;
    ls.probes_seen = ls.probes_seen + 1;
    // window of the next probed step: 2048 bins of 512 keys centred on this theta
    const uint32_t p = theta >> kPredShift;
    const uint32_t lo_bin = p > (uint32_t)(kHistBins / 2) ? p - kHistBins / 2 : 0u;
    ls.mode = kSelHist;
    ls.win_lo = lo_bin << kPredShift;
    ls.win_shift = kPredShift;
    ls.win_bins = kHistBins;
    ls.predicted = 1;
    ls.passes = 0;
    ls.above = 0;
    ls.k_rem = 0;
    ls.sel_count = 0;
    ls.acc_above = 0;
    ls.acc_zeros = 0;
    ls.acc_maxkey = 0;
    ls.acc_nonfinite = 0;
    ls.cand_count = 0;
  }
}

// ---------------------------------------------------------------------------------------------
// Stage 4: per-layer assignment (one workgroup per tensor): merge the chunk moments, variance
// EMA (Sec. 3.1 first equation), precision rule (second equation) with curvature promotion
// (Sec. 3.2), step size eta_l (Sec. 3.2), overflow decision and loss-scale schedule.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void k_assign(const TensorDesc* __restrict__ tds,
                                                     const StatPartial* __restrict__ partials, LayerDev* layers,
                                                     GlobalDev* glob, uint32_t* trans_list, uint32_t n_tensors,
                                                     StepScalars sc, Hyper hp) {
  const uint32_t l = blockIdx.x;
  const TensorDesc td = tds[l];
  LayerDev& ls = layers[l];
  const bool skip = step_skipped(glob, sc.step_id);
  __shared__ Moments s_m[kThreads / kWave];
  Moments mom{0.0, 0.0, 0.0};
  if (!skip) {
    // fixed merge order: each thread folds a contiguous run of chunk partials, then a tree
    const uint32_t per = (td.n_chunks + kThreads - 1) / kThreads;
    const uint32_t c0 = threadIdx.x * per, c1 = min(c0 + per, td.n_chunks);
    for (uint32_t c = c0; c < c1; ++c) {
      const StatPartial p = partials[td.first_chunk + c];
      const int64_t left = td.numel - (int64_t)c * kChunk;
      Moments m{(double)(left < kChunk ? left : kChunk), p.mean, p.m2};
      mom = merge(mom, m);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mom = merge(mom, shfl_down(mom, o));
    if ((threadIdx.x & (kWave - 1)) == 0) s_m[threadIdx.x / kWave] = mom;
  }
  __syncthreads();
  if (threadIdx.x != 0) return;
  ls.found_inf = (ls.found_epoch == sc.step_id) ? 1u : 0u;
  if (!skip) {
    Moments t = s_m[0];
    for (int w = 1; w < kThreads / kWave; ++w) t = merge(t, s_m[w]);
    const double var = t.m2 / t.n;
    const uint32_t applied = ls.applied_steps + 1;
    ls.applied_steps = applied;
    ls.mean = (float)t.mean;
    ls.var = (float)var;
    if (applied == 1) ls.v = (float)var;
    else ls.v = (float)((double)hp.beta_var * (double)ls.v + (1.0 - (double)hp.beta_var) * var);
    if (!td.has_probe) ls.curv_nonfinite = 0;
    const int prev = ls.code;
    ls.prev_code = prev;
    int code = prev;
    if (applied % (uint32_t)hp.ctrl_interval == 0) {
      ls.lambda_ctrl = ls.lambda;
      const float v = ls.v;
      code = (v < hp.tau_low) ? kFP16 : (v < hp.tau_high) ? kBF16 : kFP32;
      if (ls.lambda_ctrl > hp.tau_curv && code < kFP32) code += 1;
      ls.code = code;
    }
    const float den = fmaf(hp.alpha, ls.lambda_ctrl, 1.0f);
    ls.eta = sc.lr / den;
    if (elem_size(code) != elem_size(prev)) {
      const uint32_t slot = atomicAdd(&glob->trans_count[sc.step_id & 1u], 1u);
      trans_list[(sc.step_id & 1u) * n_tensors + slot] = l;
    }
  }
  if (l == 0) {
    glob->trans_count[(sc.step_id + 1u) & 1u] = 0;
    float next = sc.loss_scale;
    if (skip) {
      glob->good_steps = 0;
      next = sc.loss_scale * hp.scale_backoff;
    } else {
      const int32_t good = glob->good_steps + 1;
      if (good >= hp.growth_interval) {
        glob->good_steps = 0;
        next = sc.loss_scale * hp.scale_growth;
      } else {
        glob->good_steps = good;
      }
    }
    glob->res_skipped = skip ? 1 : 0;
    glob->res_next_scale = next;
    glob->res_step_id = sc.step_id;
  }
}

// ---------------------------------------------------------------------------------------------
// Stage 5: fused update + cast.  Per element, fp32:
//   theta = widen(param);  gt = widen(g) * inv_scale;  d = fma(wd, theta, gt);
//   m = fma(mu, m, d) (m = d without a buffer);  theta' = fma(-eta, m, theta);
//   store theta' in the layer's new precision, round to nearest even.
// All loads of a chunk complete before its first store (needed when the storage size changes
// in place, harmless otherwise).
// ---------------------------------------------------------------------------------------------
template <int GD, int PD, int ND, bool FULL, bool MOM>
__device__ __forceinline__ void update_chunk(const TensorDesc& td, int64_t base, float inv_scale, float wd, float mu,
                                             float neg_eta, bool barrier) {
  const int tid = threadIdx.x;
  float g[kRows][4], th[kRows][4], m[kRows][4];
#pragma unroll
  for (int r = 0; r < kRows; ++r) {
    const int64_t idx = base + r * kRowElems + tid * kVec;
    if (FULL) {
      load4<GD>(td.grad, idx, g[r]);
      load4<PD>(td.param, idx, th[r]);
      if (MOM) load4<kFP32>(td.mom, idx, m[r]);
    } else {
      load4_guard<GD>(td.grad, idx, td.numel, 0.0f, g[r]);
      load4_guard<PD>(td.param, idx, td.numel, 0.0f, th[r]);
      if (MOM) load4_guard<kFP32>(td.mom, idx, td.numel, 0.0f, m[r]);
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

// Any combination of gradient / old / new precision, decided at run time (uniform per workgroup).
template <bool MOM>
__device__ __noinline__ void update_chunk_rt(const TensorDesc& td, int gd, int pd, int nd, int64_t base,
                                             float inv_scale, float wd, float mu, float neg_eta, bool barrier) {
  const int tid = threadIdx.x;
  const bool full = base + kChunk <= td.numel;
  float g[kRows][4], th[kRows][4], m[kRows][4];
#pragma unroll
  for (int r = 0; r < kRows; ++r) {
    const int64_t idx = base + r * kRowElems + tid * kVec;
    load4_rt(gd, td.grad, idx, td.numel, full, g[r]);
    load4_rt(pd, td.param, idx, td.numel, full, th[r]);
    if (MOM) load4_rt(kFP32, td.mom, idx, td.numel, full, m[r]);
  }
#pragma unroll
  for (int r = 0; r < kRows; ++r) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float gt = g[r][i] * inv_scale;
      const float d = fmaf(wd, th[r][i], gt);
      const float mm = MOM ? fmaf(mu, m[r][i], d) : d;
      m[r][i] = mm;
      th[r][i] = fmaf(neg_eta, mm, th[r][i]);
    }
  }
  if (barrier) __syncthreads();
#pragma unroll
  for (int r = 0; r < kRows; ++r) {
    const int64_t idx = base + r * kRowElems + tid * kVec;
    store4_rt(nd, td.param, idx, td.numel, full, th[r]);
    if (MOM) store4_rt(kFP32, td.mom, idx, td.numel, full, m[r]);
  }
}

__device__ __forceinline__ void update_any(const TensorDesc& td, int pd, int nd, int64_t base, float inv_scale,
                                           float wd, float mu, float neg_eta, bool barrier) {
  const bool full = base + kChunk <= td.numel;
  const bool mom = td.mom != nullptr;
  // the streaming case gets a fully specialised body: fp32 gradients, fp32 parameters, whole chunk
  if (full && mom && td.grad_dtype == kFP32 && pd == kFP32 && nd == kFP32) {
    update_chunk<kFP32, kFP32, kFP32, true, true>(td, base, inv_scale, wd, mu, neg_eta, barrier);
  } else if (full && mom && td.grad_dtype == kFP32 && pd == kBF16 && nd == kBF16) {
    update_chunk<kFP32, kBF16, kBF16, true, true>(td, base, inv_scale, wd, mu, neg_eta, barrier);
  } else if (mom) {
    update_chunk_rt<true>(td, td.grad_dtype, pd, nd, base, inv_scale, wd, mu, neg_eta, barrier);
  } else {
    update_chunk_rt<false>(td, td.grad_dtype, pd, nd, base, inv_scale, wd, mu, neg_eta, barrier);
  }
}

// Tensors whose storage size does not change: element i is read and written at the same address
// by the same lane, so the update is in place.  One workgroup per chunk.
__global__ __launch_bounds__(kThreads) void k_update(const TensorDesc* __restrict__ tds,
                                                     const ChunkRef* __restrict__ chunks, const LayerDev* layers,
                                                     const GlobalDev* glob, StepScalars sc, float wd, float mu) {
  if (step_skipped(glob, sc.step_id)) return;
  const ChunkRef cr = chunks[blockIdx.x];
  const LayerDev& ls = layers[cr.tensor];
  const int pd = ls.prev_code, nd = ls.code;
  if (elem_size(pd) != elem_size(nd)) return;
  const TensorDesc td = tds[cr.tensor];
  update_any(td, pd, nd, (int64_t)cr.index * kChunk, sc.inv_scale, wd, mu, -ls.eta, false);
}

// Tensors whose storage size changes (2 <-> 4 bytes per element) are rewritten in place in
// phases: phase 0 is chunk 0, phase p >= 1 the chunks [2^(p-1), 2^p).  Inside a phase the bytes
// written (element range [lo, hi) at the new size) never overlap the bytes read (same range at
// the old size) because hi <= 2 lo.  Narrowing runs the phases in ascending order, so every
// write lands on bytes whose old contents were consumed by an earlier phase; widening runs them
// in descending order for the same reason.  Launch `launch` of `n_launch` handles, for each
// listed tensor, phase `launch` (narrowing) or `last_phase - launch` (widening).
__global__ __launch_bounds__(kThreads) void k_update_resize(const TensorDesc* __restrict__ tds,
                                                            const LayerDev* layers, const GlobalDev* glob,
                                                            const uint32_t* trans_list, uint32_t n_tensors,
                                                            uint32_t launch, StepScalars sc, float wd, float mu) {
  if (step_skipped(glob, sc.step_id)) return;
  const uint32_t count = glob->trans_count[sc.step_id & 1u];
  const uint32_t* list = trans_list + (sc.step_id & 1u) * n_tensors;
  for (uint32_t i = 0; i < count; ++i) {
    const uint32_t l = list[i];
    const TensorDesc td = tds[l];
    const LayerDev& ls = layers[l];
    const int pd = ls.prev_code, nd = ls.code;
    // number of phases: 1 + ceil(log2(n_chunks))
    const uint32_t last_phase = td.n_chunks <= 1 ? 0u : 32u - (uint32_t)__clz(td.n_chunks - 1u);
    if (launch > last_phase) continue;
    const bool narrowing = elem_size(nd) < elem_size(pd);
    const uint32_t phase = narrowing ? launch : last_phase - launch;
    const uint32_t c_lo = phase == 0 ? 0u : (1u << (phase - 1u));
    const uint32_t c_hi = phase == 0 ? 1u : min(1u << phase, td.n_chunks);
    for (uint32_t c = c_lo + blockIdx.x; c < c_hi; c += gridDim.x)
      update_any(td, pd, nd, (int64_t)c * kChunk, sc.inv_scale, wd, mu, -ls.eta, true);
  }
}

// ---------------------------------------------------------------------------------------------
// Utility: fp32 -> {fp16, bf16, fp32} array conversion with the store path of the update kernel.
// ---------------------------------------------------------------------------------------------
template <int ND>
__global__ __launch_bounds__(kThreads) void k_cast(const float* __restrict__ src, void* dst, int64_t n) {
  const int64_t stride = (int64_t)gridDim.x * kThreads * kVec;
  for (int64_t idx = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * kVec; idx < n; idx += stride) {
    float v[4];
    load4_guard<kFP32>(src, idx, n, 0.0f, v);
    store4_guard<ND>(dst, idx, n, v);
  }
}

// ---------------------------------------------------------------------------------------------
// Host-side launchers
// ---------------------------------------------------------------------------------------------
#define TA_LAUNCH_CHECK()                      \
  do {                                         \
    hipError_t e_ = hipGetLastError();         \
    if (e_ != hipSuccess) return e_;           \
  } while (0)

hipError_t launch_grad_stats(const DeviceTables& t, const StepScalars& sc, hipStream_t s) {
  hipLaunchKernelGGL(k_grad_stats, dim3(t.total_chunks), dim3(kThreads), 0, s, t.tensors, t.chunks, t.partials,
                     t.layers, t.glob, sc);
  TA_LAUNCH_CHECK();
  return hipSuccess;
}

hipError_t launch_curv_ema_hist(const DeviceTables& t, const StepScalars& sc, float beta_h, float omb_h,
                                hipStream_t s) {
  const uint32_t grid = t.total_chunks < t.persistent_grid ? t.total_chunks : t.persistent_grid;
  hipLaunchKernelGGL(k_curv_ema_hist, dim3(grid), dim3(kThreads), 0, s, t.tensors, t.chunks, t.total_chunks,
                     t.layers, t.glob, t.hist, sc, beta_h, omb_h);
  TA_LAUNCH_CHECK();
  return hipSuccess;
}

hipError_t launch_hist_pass(const DeviceTables& t, const StepScalars& sc, hipStream_t s) {
  const uint32_t grid = t.total_chunks < t.fallback_grid ? t.total_chunks : t.fallback_grid;
  hipLaunchKernelGGL(k_hist_pass, dim3(grid), dim3(kThreads), 0, s, t.tensors, t.chunks, t.total_chunks, t.layers,
                     t.glob, t.hist, sc);
  TA_LAUNCH_CHECK();
  return hipSuccess;
}

hipError_t launch_select_scan(const DeviceTables& t, const StepScalars& sc, uint32_t sparsity_ppm, hipStream_t s) {
  hipLaunchKernelGGL(k_select_scan, dim3(t.n_tensors), dim3(kThreads), 0, s, t.tensors, t.layers, t.glob, t.hist, sc,
                     sparsity_ppm);
  TA_LAUNCH_CHECK();
  return hipSuccess;
}

hipError_t launch_mask(const DeviceTables& t, const StepScalars& sc, hipStream_t s) {
  hipLaunchKernelGGL(k_mask, dim3(t.total_chunks), dim3(kThreads), 0, s, t.tensors, t.chunks, t.layers, t.glob,
                     t.cands, sc);
  TA_LAUNCH_CHECK();
  return hipSuccess;
}

hipError_t launch_select_finish(const DeviceTables& t, const StepScalars& sc, hipStream_t s) {
  hipLaunchKernelGGL(k_select_finish, dim3(t.n_tensors), dim3(kThreads), 0, s, t.tensors, t.layers, t.glob, t.cands,
                     sc);
  TA_LAUNCH_CHECK();
  return hipSuccess;
}

hipError_t launch_assign(const DeviceTables& t, const StepScalars& sc, const Hyper& hp, hipStream_t s) {
  hipLaunchKernelGGL(k_assign, dim3(t.n_tensors), dim3(kThreads), 0, s, t.tensors, t.partials, t.layers, t.glob,
                     t.trans_list, t.n_tensors, sc, hp);
  TA_LAUNCH_CHECK();
  return hipSuccess;
}

hipError_t launch_update(const DeviceTables& t, const StepScalars& sc, float wd, float mu, hipStream_t s) {
  hipLaunchKernelGGL(k_update, dim3(t.total_chunks), dim3(kThreads), 0, s, t.tensors, t.chunks, t.layers, t.glob, sc,
                     wd, mu);
  TA_LAUNCH_CHECK();
  return hipSuccess;
}

hipError_t launch_update_resize(const DeviceTables& t, const StepScalars& sc, float wd, float mu, hipStream_t s) {
  // phases 0 .. ceil(log2(max chunks per tensor)); a phase holds at most half the chunks of a tensor
  uint32_t last_phase = 0;
  while ((1u << last_phase) < t.max_chunks_per_tensor) ++last_phase;
  uint32_t grid = (t.max_chunks_per_tensor + 1) / 2;
  if (grid < 1) grid = 1;
  if (grid > t.fallback_grid) grid = t.fallback_grid;
  for (uint32_t launch = 0; launch <= last_phase; ++launch) {
    hipLaunchKernelGGL(k_update_resize, dim3(grid), dim3(kThreads), 0, s, t.tensors, t.layers, t.glob, t.trans_list,
                       t.n_tensors, launch, sc, wd, mu);
    TA_LAUNCH_CHECK();
  }
  return hipSuccess;
}

hipError_t launch_cast(const float* src, void* dst, int64_t n, int dtype, hipStream_t s) {
  int64_t blocks = (n + kThreads * kVec - 1) / (kThreads * kVec);
  if (blocks > 65536) blocks = 65536;
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

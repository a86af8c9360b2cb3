// gfx950 kernels of the Tri-Accel optimizer step.
//
// Every kernel streams tensors in chunks of kChunk = 4096 elements: four rows of 256 lanes, each
// lane holding 4 consecutive elements (one 128-bit access per lane, row and fp32 array).  All
// arithmetic that decides a stored value is fp32 with an explicit operation order (fmaf where a
// fused multiply-add is meant; the file is compiled with -ffp-contract=off); reductions are fp64.
#include "device_util.h"

namespace triaccel {

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
// One workgroup per chunk.  Each lane accumulates, in fp64, the sums of (x - K) and (x - K)^2 of
// its 16 unscaled values x = fp32(g) * inv_scale, where the shift K is the chunk's first value
// (a sample of the data, so the sums stay small against their cancellation).  Lanes and
// wavefronts are added in a fixed order; one (mean, M2) partial per chunk.
// ---------------------------------------------------------------------------------------------
template <int GD, bool FULL>
__device__ __forceinline__ void stats_chunk(const TensorDesc& td, int64_t base, float inv_scale, double& shift,
                                            double& s1, double& s2, uint32_t& bad) {
  const int tid = threadIdx.x;
  float g[kRows][4];
  // the shift is read in the same batch of loads as the data: one memory latency per chunk, not two
  const float first = load1<GD>(td.grad, base);
#pragma unroll
  for (int r = 0; r < kRows; ++r) {
    const int64_t idx = base + r * kRowElems + tid * kVec;
    if (FULL) load4<GD>(td.grad, idx, g[r]);
    else load4_guard<GD>(td.grad, idx, td.numel, 0.0f, g[r]);
  }
  shift = (double)(first * inv_scale);
#pragma unroll
  for (int r = 0; r < kRows; ++r) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int64_t idx = base + r * kRowElems + tid * kVec + i;
      if (FULL || idx < td.numel) {
        const float raw = g[r][i];
        bad |= ((f2u(raw) & 0x7f800000u) == 0x7f800000u) ? 1u : 0u;
        const double d = (double)(raw * inv_scale) - shift;
        s1 += d;
        s2 = fma(d, d, s2);
      }
    }
  }
}

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

__global__ __launch_bounds__(kThreads) void k_grad_stats(const TensorDesc* __restrict__ tds,
                                                         const ChunkRef* __restrict__ chunks,
                                                         StatPartial* __restrict__ partials, LayerDev* layers,
                                                         GlobalDev* glob, StepArg sa) {
  const StepScalars sc = step_scalars(sa);
  const ChunkRef cr = chunks[blockIdx.x];
  const TensorDesc td = tds[cr.tensor];
  const int64_t base = (int64_t)cr.index * kChunk;
  const bool full = base + kChunk <= td.numel;
  double s1 = 0.0, s2 = 0.0;
  uint32_t bad = 0;
  double shift = 0.0;
  if (full) {
    switch (td.grad_dtype) {
      case kFP32: stats_chunk<kFP32, true>(td, base, sc.inv_scale, shift, s1, s2, bad); break;
      case kBF16: stats_chunk<kBF16, true>(td, base, sc.inv_scale, shift, s1, s2, bad); break;
      default: stats_chunk<kFP16, true>(td, base, sc.inv_scale, shift, s1, s2, bad); break;
    }
  } else {
    switch (td.grad_dtype) {
      case kFP32: stats_chunk<kFP32, false>(td, base, sc.inv_scale, shift, s1, s2, bad); break;
      case kBF16: stats_chunk<kBF16, false>(td, base, sc.inv_scale, shift, s1, s2, bad); break;
      default: stats_chunk<kFP16, false>(td, base, sc.inv_scale, shift, s1, s2, bad); break;
    }
  }
  s1 = wave_sum_f64(s1);
  s2 = wave_sum_f64(s2);
  bad = wave_or(bad);
  __shared__ double s_sum[2][kThreads / kWave];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  if (lane == 0) {
    s_sum[0][wave] = s1;
    s_sum[1][wave] = s2;
    if (bad) {
      atomicExch(reinterpret_cast<unsigned long long*>(&layers[cr.tensor].found_epoch), (unsigned long long)sc.step_id);
      atomicExch(reinterpret_cast<unsigned long long*>(&glob->skip_epoch), (unsigned long long)sc.step_id);
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    double t1 = s_sum[0][0], t2 = s_sum[1][0];
#pragma unroll
    for (int w = 1; w < kThreads / kWave; ++w) {
      t1 += s_sum[0][w];
      t2 += s_sum[1][w];
    }
    const int64_t left = td.numel - base;
    const double n = (double)(left < kChunk ? left : kChunk);
    const double m2 = t2 - t1 * t1 / n;
    partials[blockIdx.x].mean = shift + t1 / n;
    partials[blockIdx.x].m2 = m2 > 0.0 ? m2 : 0.0;
  }
}

// ---------------------------------------------------------------------------------------------
// Threshold selection (exact k-th largest |h_i| per tensor) on the 31-bit magnitude keys,
// organised so that a probed step normally needs NO pass over h beyond the one that creates it:
//
//   * From the thresholds of the last probed steps (up to three) the library predicts this
//     step's threshold and a BAND around it (a few times the error the last predictions made).
//   * The EMA kernel writes a provisional mask (bit = key at or above the band), lists the keys
//     inside the band, and counts the keys above it.
//   * If the k-th largest key falls inside the band (count above < k <= count above + listed),
//     the listed keys resolve theta exactly and only their mask bits are patched.
//   * Otherwise (no prediction yet, prediction off, too many keys to list) the tensor falls
//     back to a radix select by histogram passes over h and a separate mask pass.
//   * Tensors with at most kListAllMax elements list all their non-zero keys and select from the list.
// ---------------------------------------------------------------------------------------------
struct Window {
  uint32_t lo, shift, bins;
  uint32_t hi;  // keys in [lo, hi) are counted; hi <= lo + (bins << shift)
};

// Flush a workgroup's LDS histogram to the tensor's global one and clear it.
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
// Stage 2: curvature EMA (diagonal Hutchinson signal of Sec. 3.2), one workgroup per chunk.
// Per element, fp32:  u = (z * hz) * inv_scale;  h = u on the tensor's first probe, else
// h = fma(beta_h, h, (1 - beta_h) * u);  a non-finite u leaves h unchanged.
// The same pass writes the provisional mask, lists the keys of the band and leaves one small
// record per chunk (keys above the band, zero keys, largest key, non-finite flag); no atomics
// except the candidate appends.
// ---------------------------------------------------------------------------------------------
// SRC selects the sample: -1 = Hutchinson pair z * Hz / S; a precision code = squared unscaled
// gradient (g / S)^2 read from the gradient buffer of that precision (empirical Fisher).
template <bool FULL, int SRC>
__device__ __forceinline__ void ema_chunk(const TensorDesc& td, int64_t base, float inv_scale, float beta_h,
                                          float omb_h, bool first, bool band, bool list_all, uint32_t band_lo,
                                          uint32_t band_hi, uint32_t chunk_index, uint32_t tensor, Candidate* cands,
                                          uint32_t* counters, uint32_t& above_zeros, uint32_t& maxkey,
                                          uint32_t& nonfin) {
  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  float z[kRows][4], hz[SRC < 0 ? kRows : 1][4], h[kRows][4];
#pragma unroll
  for (int r = 0; r < kRows; ++r) {
    const int64_t idx = base + r * kRowElems + tid * kVec;
    if constexpr (SRC < 0) {
      if (FULL) {
        load4<kFP32>(td.z, idx, z[r]);
        load4<kFP32>(td.hz, idx, hz[r]);
      } else {
        load4_guard<kFP32>(td.z, idx, td.numel, 0.0f, z[r]);
        load4_guard<kFP32>(td.hz, idx, td.numel, 0.0f, hz[r]);
      }
    } else {
      // x = g / S in both factors: u = x * x
      if (FULL) load4<SRC>(td.grad, idx, z[r]);
      else load4_guard<SRC>(td.grad, idx, td.numel, 0.0f, z[r]);
#pragma unroll
      for (int i = 0; i < 4; ++i) z[r][i] = z[r][i] * inv_scale;
    }
    if (FULL) load4<kFP32>(td.curv, idx, h[r]);
    else load4_guard<kFP32>(td.curv, idx, td.numel, 0.0f, h[r]);
  }
  uint32_t word[kRows];
  uint32_t cflags = 0;
#pragma unroll
  for (int r = 0; r < kRows; ++r) {
    const int64_t idx = base + r * kRowElems + tid * kVec;
    uint32_t nib = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float u;
      if constexpr (SRC < 0) {
        u = z[r][i] * hz[r][i];
        u = u * inv_scale;
      } else {
        u = z[r][i] * z[r][i];
      }
      float hn = h[r][i];
      const bool valid = FULL || idx + i < td.numel;
      if ((f2u(u) & 0x7f800000u) == 0x7f800000u) {
        if (valid) nonfin = 1u;
      } else if (first) {
        hn = u;
      } else {
        const float p = omb_h * u;
        hn = fmaf(beta_h, hn, p);
      }
      h[r][i] = hn;
      if (valid) {
        const uint32_t key = f2u(hn) & 0x7fffffffu;
        maxkey = max(maxkey, key);
        if (key == 0u) {
          above_zeros += 1u << 16;  // zero keys in the high half, keys above the band in the low half
        } else if (list_all) {
          cflags |= 1u << (r * 4 + i);
        } else if (band) {
          if (key >= band_hi) {
            nib |= 1u << i;
            above_zeros += 1u;
          } else if (key >= band_lo) {
            cflags |= 1u << (r * 4 + i);
          }
        }
      }
    }
    if (FULL) store4<kFP32>(td.curv, idx, h[r]);
    else store4_guard<kFP32>(td.curv, idx, td.numel, h[r]);
    if (band || list_all) word[r] = gather_mask_word(nib, lane);
  }
  if (band || list_all) {
    store_mask_words<FULL>(td, base, word);
    append_candidates(cflags, h, base, chunk_index, tensor, td, cands, counters);
  }
}

template <bool FISHER>
__global__ __launch_bounds__(kThreads) void k_curv_ema(const TensorDesc* __restrict__ tds,
                                                       const ChunkRef* __restrict__ chunks, const LayerDev* layers,
                                                       const GlobalDev* glob, EmaPartial* __restrict__ ema_partials,
                                                       Candidate* cands, uint32_t* counters, StepArg sa,
                                                       float beta_h, float omb_h) {
  const StepScalars sc = step_scalars(sa);
  if (step_skipped(glob, sc.step_id)) return;
  const ChunkRef cr = chunks[blockIdx.x];
  const TensorDesc td = tds[cr.tensor];
  if (!td.has_probe) return;
  const LayerDev& ls = layers[cr.tensor];
  const bool first = ls.probes_seen == 0;
  const bool list_all = td.list_all != 0;
  const bool band = !list_all && ls.use_band != 0;
  const uint32_t band_lo = ls.band_lo, band_hi = ls.band_hi;
  const int64_t base = (int64_t)cr.index * kChunk;
  uint32_t above_zeros = 0, maxkey = 0, nonfin = 0;
#define TA_EMA(FULL_, SRC_)                                                                                   \
  ema_chunk<FULL_, SRC_>(td, base, sc.inv_scale, beta_h, omb_h, first, band, list_all, band_lo, band_hi, cr.index, \
                         cr.tensor, cands, counters, above_zeros, maxkey, nonfin)
  const bool full = base + kChunk <= td.numel;
  if constexpr (!FISHER) {
    if (full) TA_EMA(true, -1);
    else TA_EMA(false, -1);
  } else {
    switch (td.grad_dtype) {
      case kFP32:
        if (full) TA_EMA(true, kFP32);
        else TA_EMA(false, kFP32);
        break;
      case kBF16:
        if (full) TA_EMA(true, kBF16);
        else TA_EMA(false, kBF16);
        break;
      default:
        if (full) TA_EMA(true, kFP16);
        else TA_EMA(false, kFP16);
        break;
    }
  }
#undef TA_EMA
  // per-chunk record: fixed-order reduction over lanes and wavefronts, one plain store
  above_zeros = wave_sum(above_zeros);  // at most 4096 in either half: no carry between the halves
  maxkey = wave_max(maxkey);
  const uint32_t anynf = __any(nonfin != 0u) ? 1u : 0u;
  __shared__ uint32_t s_red[3][kThreads / kWave];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  if (lane == 0) {
    s_red[0][wave] = above_zeros;
    s_red[1][wave] = maxkey;
    s_red[2][wave] = anynf;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t az = 0, mk = 0, nf = 0;
#pragma unroll
    for (int w = 0; w < kThreads / kWave; ++w) {
      az += s_red[0][w];
      mk = max(mk, s_red[1][w]);
      nf |= s_red[2][w];
    }
    ema_partials[blockIdx.x] = EmaPartial{az & 0xffffu, az >> 16, mk, nf};
  }
}

// ---------------------------------------------------------------------------------------------
// Fallback: histogram pass over |h| for tensors whose threshold is not yet confined to a range
// whose keys can be listed (mode kSelHist).  Workgroups own contiguous ranges of chunks so that
// the LDS histogram is flushed once per (workgroup, tensor); reads h only.
// ---------------------------------------------------------------------------------------------
template <bool FULL>
__device__ __forceinline__ void hist_chunk(const TensorDesc& td, int64_t base, const Window& w, uint32_t* s_hist,
                                           bool count_above, uint32_t& above) {
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
        if (key < w.hi) atomicAdd(&s_hist[(key - w.lo) >> w.shift], 1u);
        else if (count_above) ++above;
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Rank search in an LDS histogram: find the bin, counted from the top, that holds the r-th
// largest key (1 <= r <= total).  All NT threads of the workgroup call it; results are broadcast.
// ---------------------------------------------------------------------------------------------
struct BinHit {
  uint32_t bin;     // bin holding the r-th largest key
  uint32_t higher;  // number of keys in bins above it
  uint32_t count;   // keys in that bin
};
template <int NT>
__device__ BinHit find_rank_from_top(const uint32_t* s_hist, uint32_t bins, uint32_t r, uint32_t* s_part,
                                     uint32_t* s_out) {
  // level 0: every thread sums its run of bins; level 1: every lane of wavefront 0 sums a run of
  // thread sums; a suffix scan over the 64 lanes locates the lane, then the thread, then the bin.
  constexpr int G = NT / kWave;  // thread sums per lane of wavefront 0
  const uint32_t per = (bins + NT - 1) / NT;
  const uint32_t b0 = threadIdx.x * per;
  uint32_t sum = 0;
  for (uint32_t b = b0; b < min(b0 + per, bins); ++b) sum += s_hist[b];
  s_part[threadIdx.x] = sum;
  __syncthreads();
  if (threadIdx.x < kWave) {
    const int lane = threadIdx.x;
    uint32_t mine = 0;
#pragma unroll
    for (int i = 0; i < G; ++i) mine += s_part[lane * G + i];
    uint32_t suffix = mine;  // sum over lanes >= this one
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
      const uint32_t t = __shfl_down(suffix, o);
      if (lane + o < kWave) suffix += t;
    }
    const unsigned long long reach = __ballot(suffix >= r);  // lanes from which the top reaches rank r
    const int pick = reach ? 63 - __clzll(reach) : 0;         // the highest such lane holds the rank
    if (lane == pick) {
      uint32_t acc = suffix - mine;  // keys in lanes above
      int t = pick * G + G - 1;
      for (; t > pick * G; --t) {
        if (acc + s_part[t] >= r) break;
        acc += s_part[t];
      }
      s_out[0] = (uint32_t)t;
      s_out[1] = acc;
    }
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

__device__ __forceinline__ uint32_t topk_count(int64_t n, uint32_t s_ppm, uint32_t k_abs) {
  // a fixed k if given, else k = n - floor(n * s / 1e6); clamped to [1, n]; n < 2^31 so the
  // product fits 64 bits
  int64_t k = k_abs ? (int64_t)k_abs : n - (int64_t)(((uint64_t)n * (uint64_t)s_ppm) / 1000000ull);
  if (k < 1) k = 1;
  if (k > n) k = n;
  return (uint32_t)k;
}

// ---------------------------------------------------------------------------------------------
// First decision after the EMA pass (called by the per-layer kernel, one workgroup per tensor):
// add up the per-chunk records and decide whether the listed keys settle the threshold (band
// hit, or small tensor) or the tensor must fall back to histogram passes.
// ---------------------------------------------------------------------------------------------
__device__ void select_begin(uint32_t l, const TensorDesc& td, LayerDev& ls, GlobalDev* glob,
                             const EmaPartial* __restrict__ ema_partials, uint32_t* counters, uint64_t step_id,
                             uint32_t sparsity_ppm, uint32_t topk_abs, uint32_t (*s_red)[kThreads / kWave]) {
  uint32_t above = 0, zeros = 0, maxkey = 0, nonfin = 0, listed = 0;
  for (uint32_t c = threadIdx.x; c < td.n_chunks; c += kThreads) {
    const EmaPartial p = ema_partials[td.first_chunk + c];
    above += p.above;
    zeros += p.zeros;
    maxkey = max(maxkey, p.maxkey);
    nonfin |= p.nonfinite;
  }
  if (threadIdx.x < kCandLists) listed = *cand_counter(counters, l, threadIdx.x);
  above = wave_sum(above);
  zeros = wave_sum(zeros);
  maxkey = wave_max(maxkey);
  nonfin = wave_or(nonfin);
  listed = wave_sum(listed);
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  if (lane == 0) {
    s_red[0][wave] = above;
    s_red[1][wave] = zeros;
    s_red[2][wave] = maxkey;
    s_red[3][wave] = nonfin;
    s_red[4][wave] = listed;
  }
  __syncthreads();
  above = zeros = maxkey = nonfin = listed = 0;
#pragma unroll
  for (int w = 0; w < kThreads / kWave; ++w) {
    above += s_red[0][w];
    zeros += s_red[1][w];
    maxkey = max(maxkey, s_red[2][w]);
    nonfin |= s_red[3][w];
    listed += s_red[4][w];
  }
  const uint32_t nonzero = (uint32_t)td.numel - zeros;
  const uint32_t k = topk_count(td.numel, sparsity_ppm, topk_abs);
  // 0: the lists settle it; 1: theta = 0 (fewer non-zero keys than k); 2: histogram passes
  int outcome;
  if (td.list_all) outcome = 0;
  else if (k > nonzero) outcome = 1;
  else if (ls.use_band && above < k && k <= above + listed && listed <= td.cand_cap) outcome = 0;
  else outcome = 2;
  if (outcome != 0) reset_cand_counters(counters, l);  // drop whatever the EMA kernel listed
  if (threadIdx.x == 0) {
    // diagnostic: 0 small tensor, 1 band held, 2 no band this step, 3 threshold above the band,
    // 4 threshold below the band, 5 too many keys listed, 6 fewer non-zero keys than k
    ls.sel_listed = listed;
    ls.sel_outcome = td.list_all ? 0u
                     : k > nonzero ? 6u
                     : !ls.use_band ? 2u
                     : above >= k ? 3u
                     : k > above + listed ? 4u
                     : listed > td.cand_cap ? 5u : 1u;
    ls.acc_maxkey = maxkey;
    ls.acc_nonfinite = nonfin;
    ls.nonzero = nonzero;
    ls.k_rem = k;
    ls.passes = 1;
    ls.acc_above = 0;
    if (outcome != 0) atomicAdd(&glob->mask_pending[step_id & 1u], 1u);
    if (outcome == 0) {
      ls.mode = kSelCand;
      ls.mask_done = 1;
      if (td.list_all) {
        ls.above = 0;
        ls.rng_lo = 0;
        ls.rng_hi = 0x80000000u;
      } else {
        ls.above = above;
        ls.rng_lo = ls.band_lo;
        ls.rng_hi = ls.band_hi;
        ls.dens_count = listed;
        ls.dens_width = ls.band_hi - ls.band_lo;
      }
    } else if (outcome == 1) {
      ls.mode = kSelExact;
      ls.mask_done = 0;
      ls.theta_key = 0;
      ls.above = nonzero;
      ls.sel_count = 0;
    } else {
      // histogram over the predicted window if there is one; else over the kFirstOctaves octaves
      // below the largest key, where the threshold of a top-k selection normally lies (nothing is
      // above that window, so the count above it is known)
      ls.mode = kSelHist;
      ls.mask_done = 0;
      ls.above = 0;
      ls.count_above = ls.predicted;
      if (!ls.predicted) {
        const uint32_t span = (uint32_t)kHistBins << kFirstShift;
        const uint32_t hi = maxkey + 1u;
        ls.win_lo = hi > span ? hi - span : 0u;
        ls.win_hi = hi;
        ls.win_shift = kFirstShift;
        ls.win_bins = kHistBins;
      }
      atomicAdd(&glob->hist_pending[step_id & 1u], 1u);
    }
  }
  __syncthreads();
}

// ---------------------------------------------------------------------------------------------
// Scan after a histogram pass, by one workgroup for one tensor in mode kSelHist: read the
// tensor's histogram (from memory, clearing it, or already complete in LDS), and decide whether
// theta is now exact, lies in a range whose keys can be listed by the mask pass, or needs a finer
// histogram.  Uniform over the workgroup.
// ---------------------------------------------------------------------------------------------
__device__ void select_scan(uint32_t l, const TensorDesc& td, LayerDev& ls, GlobalDev* glob, uint32_t* hist,
                            uint64_t step_id, uint32_t* s_hist, uint32_t* s_part, uint32_t* s_out, bool from_global) {
  const uint32_t bins = ls.win_bins, lo = ls.win_lo, shift = ls.win_shift;
  uint32_t* gh = hist + (size_t)l * kHistBins;
  uint32_t local = 0;
  for (uint32_t b = threadIdx.x; b < kHistBins; b += kThreads) {
    uint32_t v;
    if (from_global) {
      // counted by other workgroups of the running kernel: read at device scope
      v = (b < bins) ? __hip_atomic_load(&gh[b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
      s_hist[b] = v;
      if (v) gh[b] = 0;
    } else {
      v = (b < bins) ? s_hist[b] : 0u;
    }
    local += v;
  }
  local = wave_sum(local);
  if ((threadIdx.x & (kWave - 1)) == 0) s_part[threadIdx.x / kWave] = local;
  __syncthreads();
  const uint32_t in_window = s_part[0] + s_part[1] + s_part[2] + s_part[3];
  __syncthreads();
  const uint32_t k = ls.k_rem;
  // counted by this pass (same remark), or known
  const uint32_t above = ls.count_above ? __hip_atomic_load(&ls.acc_above, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : ls.above;
  const bool missed = above >= k || above + in_window < k;
  BinHit hit{0, 0, 0};
  if (!missed) hit = find_rank_from_top<kThreads>(s_hist, bins, k - above, s_part, s_out);
  __syncthreads();
  if (threadIdx.x == 0) {
    ls.acc_above = 0;
    ls.count_above = 0;
    ls.hist_arrived = 0;
    ls.passes = ls.passes + 1;
    if (missed) {
      // The window does not contain theta.  Continue with what lies on the side where it must be:
      // between the window and the largest key (nothing is above that), or below the window (then
      // every key counted so far is above the new window).
      const uint32_t old_hi = ls.win_hi;
      uint32_t new_lo, new_hi;
      if (above >= k) {
        new_lo = old_hi;
        new_hi = ls.acc_maxkey + 1u;  // acc_maxkey >= old_hi: some key lies above the window
        ls.above = 0;
      } else {
        new_lo = 0;
        new_hi = lo;
        ls.above = above + in_window;
      }
      uint32_t ns = 0;
      while (ns < kFullShift && ((uint32_t)kHistBins << ns) < new_hi - new_lo) ++ns;
      ls.win_lo = new_lo;
      ls.win_hi = new_hi;
      ls.win_shift = ns;
      ls.win_bins = kHistBins;
      ls.window_missed = 1;
    } else {
      const uint32_t new_lo = lo + (hit.bin << shift);
      // the bin ends where the window ends (its last bin may be cut short)
      const uint32_t new_hi = min(new_lo + (1u << shift), ls.win_hi);
      ls.above = above + hit.higher;
      ls.sel_count = hit.count;
      ls.dens_count = hit.count;
      ls.dens_width = 1u << shift;
      if (shift == 0) {
        ls.mode = kSelExact;
        ls.theta_key = new_lo;
        atomicSub(&glob->hist_pending[step_id & 1u], 1u);
      } else if (hit.count <= td.cand_cap) {
        ls.mode = kSelCand;
        ls.rng_lo = new_lo;
        ls.rng_hi = new_hi;
        atomicSub(&glob->hist_pending[step_id & 1u], 1u);
      } else {
        const uint32_t ns = shift > (uint32_t)kHistBits ? shift - kHistBits : 0u;
        ls.win_lo = new_lo;
        ls.win_hi = new_hi;
        ls.win_shift = ns;
        ls.win_bins = 1u << (shift - ns);
      }
    }
  }
  __syncthreads();
}

// ---------------------------------------------------------------------------------------------
// Fallback radix select: histogram pass over the tensors in histogram mode, each workgroup over
// its share of the chunk list.  The workgroup that is the last to deliver its part of a tensor's
// histogram also scans it (select_scan), so no workgroup ever waits for another.  One round is
// what a tensor normally needs, and the step launches two (a window that missed, or more keys in
// the pivot bin than can be listed, needs the second).  Beyond that (a miss followed by
// refinements, heavy ties: at most four rounds in all) the workgroup that scans makes up to
// `serial_rounds` further passes over the whole tensor on its own -- slow for a large tensor, but
// rare, and it bounds the fallback to two launches.
// Leaves at once when no tensor is in histogram mode: a workgroup that sees the pending count at
// zero owns no chunk of a tensor still being counted, because a tensor's scan, which alone
// lowers the count, needs every workgroup owning one of its chunks to have arrived.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void k_hist_pass(const TensorDesc* __restrict__ tds,
                                                        const ChunkRef* __restrict__ chunks, uint32_t total_chunks,
                                                        LayerDev* layers, GlobalDev* glob, uint32_t* hist,
                                                        StepArg sa, int serial_rounds) {
  const StepScalars sc = step_scalars(sa);
  if (step_skipped(glob, sc.step_id)) return;
  if (__hip_atomic_load(&glob->hist_pending[sc.step_id & 1u], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0) return;
  __shared__ uint32_t s_hist[kHistBins];
  __shared__ uint32_t s_part[kThreads];
  __shared__ uint32_t s_out[8];
  __shared__ uint32_t s_last;
  for (int b = threadIdx.x; b < kHistBins; b += kThreads) s_hist[b] = 0;
  __syncthreads();
  const uint32_t per = (total_chunks + gridDim.x - 1) / gridDim.x;
  const uint32_t c0 = min(blockIdx.x * per, total_chunks);
  const uint32_t c1 = min(c0 + per, total_chunks);
  int cur = -1;
  bool active = false;
  Window w{0, 0, 0, 0};
  TensorDesc td;
  bool count_above = false;  // the number of keys above the window is not known yet (predicted window)
  uint32_t above = 0;
  uint32_t mine = 0;         // chunks of the current tensor counted by this workgroup
  uint32_t c = c0;
  while (c <= c1) {
    const bool end = (c == c1);
    const int t = end ? -2 : (int)chunks[c].tensor;
    if (t != cur) {
      if (cur >= 0 && active) {
        flush_hist(s_hist, w.bins, hist + (size_t)cur * kHistBins);
        above = wave_sum(above);
        if ((threadIdx.x & (kWave - 1)) == 0 && above) atomicAdd(&layers[cur].acc_above, above);
        // release: this workgroup's atomics are complete before its arrival is counted
        __threadfence();
        __syncthreads();
        if (threadIdx.x == 0) {
          const uint32_t before = atomicAdd(&layers[cur].hist_arrived, mine);
          s_last = (before + mine == td.n_chunks) ? 1u : 0u;
        }
        __syncthreads();
        if (s_last) {
          __threadfence();  // acquire: the scan below reads what the other workgroups added
          select_scan((uint32_t)cur, td, layers[cur], glob, hist, sc.step_id, s_hist, s_part, s_out, true);
          for (int extra = 0; extra < serial_rounds; ++extra) {
            if (layers[cur].mode != kSelHist) break;  // written before the barrier that ends the scan
            for (int b = threadIdx.x; b < kHistBins; b += kThreads) s_hist[b] = 0;
            __syncthreads();
            // after a scan the number of keys above the window is known
            const Window w2{layers[cur].win_lo, layers[cur].win_shift, layers[cur].win_bins, layers[cur].win_hi};
            uint32_t unused = 0;
            for (uint32_t q = 0; q < td.n_chunks; ++q) {
              const int64_t b2 = (int64_t)q * kChunk;
              if (b2 + kChunk <= td.numel) hist_chunk<true>(td, b2, w2, s_hist, false, unused);
              else hist_chunk<false>(td, b2, w2, s_hist, false, unused);
            }
            __syncthreads();
            select_scan((uint32_t)cur, td, layers[cur], glob, hist, sc.step_id, s_hist, s_part, s_out, false);
          }
          for (int b = threadIdx.x; b < kHistBins; b += kThreads) s_hist[b] = 0;
          __syncthreads();
        }
      }
      if (end) break;
      cur = t;
      td = tds[t];
      const LayerDev& ls = layers[t];
      active = td.has_probe != 0 && ls.mode == kSelHist && ls.passes > 0;
      w = Window{ls.win_lo, ls.win_shift, ls.win_bins, ls.win_hi};
      count_above = ls.count_above != 0;
      above = 0;
      mine = 0;
      if (!active) {
        // jump over the rest of this tensor's chunks owned by this workgroup
        c = min(td.first_chunk + td.n_chunks, c1);
        continue;
      }
    }
    const int64_t base = (int64_t)chunks[c].index * kChunk;
    if (base + kChunk <= td.numel) hist_chunk<true>(td, base, w, s_hist, count_above, above);
    else hist_chunk<false>(td, base, w, s_hist, count_above, above);
    ++mine;
    ++c;
  }
}

// ---------------------------------------------------------------------------------------------
// Finish: one workgroup per tensor resolves theta among the listed keys (radix select in LDS),
// sets their mask bits, publishes theta / nnz and plans the next probed step: the band and the
// fallback window are centred on the predicted threshold; their widths follow the error the
// recent predictions made.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t abs_diff(uint32_t a, uint32_t b) { return a > b ? a - b : b - a; }

// Sum of a per-thread count over the workgroup (kFinishThreads threads); s_red holds one word per wavefront.
__device__ __forceinline__ uint32_t finish_block_sum(uint32_t v, uint32_t* s_red) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & (kWave - 1)) == 0) s_red[threadIdx.x / kWave] = v;
  __syncthreads();
  uint32_t t = 0;
#pragma unroll
  for (int w = 0; w < kFinishThreads / kWave; ++w) t += s_red[w];
  return t;
}

__global__ __launch_bounds__(kFinishThreads) void k_select_finish(const TensorDesc* __restrict__ tds,
                                                                  LayerDev* layers, const GlobalDev* glob,
                                                                  const Candidate* cands, uint32_t* counters,
                                                                  StepArg sa, float beta_h) {
  const StepScalars sc = step_scalars(sa);
  if (step_skipped(glob, sc.step_id)) return;
  const uint32_t l = blockIdx.x;
  const TensorDesc td = tds[l];
  if (!td.has_probe) return;
  LayerDev& ls = layers[l];
  __shared__ uint32_t s_hist[kHistBins];
  __shared__ uint32_t s_part[kFinishThreads];
  __shared__ uint32_t s_red[kFinishThreads / kWave];
  __shared__ uint32_t s_out[8];
  __shared__ uint32_t s_counts[kCandLists + 1];
  __shared__ uint32_t s_prefix[kCandLists + 2];
  if (threadIdx.x <= kCandLists) {
    const uint32_t c = *cand_counter(counters, l, threadIdx.x);
    s_counts[threadIdx.x] = min(c, threadIdx.x < kCandLists ? td.sub_cap : td.cand_cap);
  }
  __syncthreads();
  const uint32_t mode = ls.mode;
  const uint32_t above = ls.above;
  const uint32_t rng_lo = ls.rng_lo, rng_hi = ls.rng_hi;
  uint32_t theta = ls.theta_key;
  uint32_t nnz = above + ls.sel_count;
  if (mode == kSelExact && theta == 0u) nnz = ls.nonzero;
  if (mode == kSelCand) {
    // all listed keys lie in [rng_lo, rng_hi); select inside the enclosing power-of-two range
    uint32_t lo = rng_lo;
    const uint32_t width = rng_hi - rng_lo;
    uint32_t width_shift = 32u - (uint32_t)__clz(width - 1u);  // ceil(log2(width)), width >= 2
    if (width <= 1u) width_shift = 0;
    uint32_t r = ls.k_rem - above;
    // exclusive prefix sums of the list lengths (flat numbering of the listed keys)
    if (threadIdx.x == 0) {
      uint32_t acc = 0;
      for (uint32_t i = 0; i <= kCandLists; ++i) {
        s_prefix[i] = acc;
        acc += s_counts[i];
      }
      s_prefix[kCandLists + 1] = acc;
    }
    __syncthreads();
    const uint32_t inside = s_prefix[kCandLists + 1];
    // up to kFinishRegs keys per thread are held in registers for the passes below; longer lists
    // are re-read from memory in every pass
    const bool in_regs = inside <= (uint32_t)(kFinishThreads * kFinishRegs);
    Candidate reg[kFinishRegs];
    uint32_t have = 0;
    if (in_regs) {
#pragma unroll
      for (int i = 0; i < kFinishRegs; ++i) {
        const uint32_t f = (uint32_t)i * kFinishThreads + threadIdx.x;
        reg[i] = Candidate{0u, 0u};
        if (f < inside) {
          uint32_t a = 0, b = kCandLists + 1;  // s_prefix[a] <= f < s_prefix[b]
          while (b - a > 1) {
            const uint32_t m = (a + b) >> 1;
            if (s_prefix[m] <= f) a = m;
            else b = m;
          }
          reg[i] = cands[td.cand_offset + (size_t)a * td.sub_cap + (f - s_prefix[a])];
          have |= 1u << i;
        }
      }
    }
    auto visit = [&](auto f) {
      if (in_regs) {
#pragma unroll
        for (int i = 0; i < kFinishRegs; ++i)
          if (have & (1u << i)) f(reg[i]);
      } else {
        for_each_candidate<kFinishThreads>(td, cands, s_counts, f);
      }
    };
    if (r > inside) {
      theta = 0;  // fewer non-zero keys than k (small tensors only): keep every non-zero entry
    } else {
      while (width_shift > 0) {
        const uint32_t ns = width_shift > (uint32_t)kHistBits ? width_shift - kHistBits : 0u;
        const uint32_t bins = 1u << (width_shift - ns);
        for (uint32_t b = threadIdx.x; b < bins; b += kFinishThreads) s_hist[b] = 0;
        __syncthreads();
        visit([&](const Candidate& c) {
          if (c.key >= lo && ((uint64_t)(c.key - lo) >> width_shift) == 0u) atomicAdd(&s_hist[(c.key - lo) >> ns], 1u);
        });
        __syncthreads();
        const BinHit hit = find_rank_from_top<kFinishThreads>(s_hist, bins, r, s_part, s_out);
        r -= hit.higher;
        lo += hit.bin << ns;
        width_shift = ns;
      }
      theta = lo;
    }
    // listed keys had their bits left clear: set those at or above theta
    uint32_t kept = 0;
    visit([&](const Candidate& c) {
      if (c.key >= theta) {
        atomicOr(&td.mask[c.idx >> 5], 1u << (c.idx & 31u));
        ++kept;
      }
    });
    kept = finish_block_sum(kept, s_red);
    nnz = above + kept;
  }
  __syncthreads();
  reset_cand_counters(counters, l);
  if (threadIdx.x != 0) return;
  // ---- publish ----
  const uint32_t prev = ls.theta_key_last;
  const uint32_t have = ls.n_theta;
  ls.theta_key = theta;
  ls.theta = u2f(theta);
  ls.nnz = nnz;
  ls.sel_passes = ls.passes - 1 + (ls.mask_done ? 0u : 1u);  // passes over h beyond the EMA pass
  ls.probes_seen = ls.probes_seen + 1;
  // ---- plan the next probed step ----
  // Two predictors of the next threshold are tracked by the error each made for this step:
  // "hold" (the last threshold; best when the threshold only jitters) and a damped extrapolation
  // in the value domain, theta + r (theta - prev), best while the curvature EMA still settles:
  // the distance of the threshold from its limit then shrinks by a nearly constant factor per
  // probe, so r is the ratio of the last two differences, kept within [0, 1] (between "hold" and
  // a straight line), and beta_h, the factor by which the EMA forgets, while only two thresholds
  // are known.  Each predictor keeps a running mean of its squared error in keys (an error three
  // times the running deviation replaces the mean at once); the one with the smaller mean is
  // used, and the band is a multiple of its deviation.
  const uint32_t prev2 = ls.theta_key_last2;
  const float unknown2 = (float)kUnknownPredErr * (float)kUnknownPredErr;
  auto track = [](float var, float err, bool first) {
    const float e2 = err * err;
    if (first || e2 > 9.0f * var) return e2;
    return 0.75f * var + 0.25f * e2;
  };
  float v_hold = unknown2, v_ext = ls.pred_ext_key ? ls.var_ext : 3.0e38f;
  if (have >= 1) v_hold = track(ls.var_hold, (float)abs_diff(theta, prev), have < 2);
  if (ls.pred_ext_key) v_ext = track(v_ext, (float)abs_diff(theta, ls.pred_ext_key), !(v_ext < 3.0e38f));
  if (ls.window_missed) {
    v_hold = fmaxf(v_hold, unknown2);
    if (v_ext < 3.0e38f) v_ext = fmaxf(v_ext, unknown2);
  }
  uint32_t ext = 0;
  if (have >= 1) {
    const double v0 = (double)u2f(theta), v1 = (double)u2f(prev);
    const double d1 = v0 - v1;
    double r = (double)beta_h;
    if (have >= 2) {
      const double d0 = v1 - (double)u2f(prev2);
      r = d0 != 0.0 ? d1 / d0 : 1.0;
    }
    r = fmin(fmax(r, 0.0), 1.0);
    const float p = (float)(v0 + r * d1);
    ext = p > 0.0f ? min(max(f2u(p), 1u), 0x7f7fffffu) : 1u;
  }
  ls.var_hold = v_hold;
  ls.var_ext = v_ext;
  ls.pred_ext_key = ext;
  ls.theta_key_last2 = prev;
  ls.theta_key_last = theta;
  ls.n_theta = have < 2 ? have + 1 : 2;
  const bool extrapolate = ext != 0u && v_ext < v_hold;
  // e: 1.5 deviations of the chosen predictor (band = 3 e = 4.5 deviations, window half = 32 e)
  const float dev = 1.5f * sqrtf(extrapolate ? v_ext : v_hold);
  const uint32_t e = dev < 16.0f ? 16u : (dev > 1.0e9f ? 1000000000u : (uint32_t)dev);
  int64_t centre = extrapolate ? (int64_t)ext : (int64_t)theta;
  if (centre < 1) centre = 1;
  if (centre > 0x7f7fffff) centre = 0x7f7fffff;
  // fallback window: 2048 bins whose half (1024 bins) spans 32 e
  uint32_t s = kMinPredShift;
  while (s < kFullShift && ((uint64_t)1024 << s) < (uint64_t)32 * e) ++s;
  const uint32_t cbin = (uint32_t)centre >> s;
  const uint32_t lo_bin = cbin > (uint32_t)(kHistBins / 2) ? cbin - kHistBins / 2 : 0u;
  // band: 3 e on either side of the centre
  const uint64_t half = (uint64_t)3 * e;
  const uint32_t band_lo = (uint64_t)centre > half ? (uint32_t)((uint64_t)centre - half) : 1u;
  const uint64_t hi64 = (uint64_t)centre + half + 1;
  const uint32_t band_hi = hi64 < 0x7f800000ull ? (uint32_t)hi64 : 0x7f800000u;
  // expected number of keys inside the band, from the key density around this step's threshold;
  // listing them only pays when they fit the lists with room to spare
  const uint64_t expect = ls.dens_width ? ((uint64_t)(band_hi - band_lo) * ls.dens_count) / ls.dens_width : 0u;
  ls.mode = kSelHist;
  ls.win_lo = lo_bin << s;
  ls.win_hi = ls.win_lo + ((uint32_t)kHistBins << s);
  ls.win_shift = s;
  ls.win_bins = kHistBins;
  ls.band_lo = band_lo;
  ls.band_hi = band_hi;
  ls.use_band = expect <= (uint64_t)(td.cand_cap - td.cand_cap / 4) ? 1u : 0u;
  ls.predicted = 1;
  ls.window_missed = 0;
  ls.mask_done = 0;
  ls.passes = 0;
  ls.above = 0;
  ls.k_rem = 0;
  ls.sel_count = 0;
  ls.dens_count = 0;
  ls.dens_width = 0;
  ls.acc_above = 0;
}

// ---------------------------------------------------------------------------------------------
// Stage 4: per-layer kernel (one workgroup per tensor): band check of the threshold selection
// (select_begin above), then the per-layer assignment: merge the chunk moments, variance
// EMA (Sec. 3.1 first equation), precision rule (second equation) with curvature promotion
// (Sec. 3.2), step size eta_l (Sec. 3.2), overflow decision and loss-scale schedule.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void k_layer(const TensorDesc* __restrict__ tds,
                                                    const StatPartial* __restrict__ partials,
                                                    const EmaPartial* __restrict__ ema_partials, uint32_t* counters,
                                                    LayerDev* layers, GlobalDev* glob, GlobalDev* host_result,
                                                    uint32_t* trans_list, uint32_t n_tensors, StepArg sa, Hyper hp) {
  const StepScalars sc = step_scalars(sa);
  const uint32_t l = blockIdx.x;
  const TensorDesc td = tds[l];
  LayerDev& ls = layers[l];
  const bool skip = step_skipped(glob, sc.step_id);
  __shared__ Moments s_m[kThreads / kWave];
  __shared__ uint32_t s_red[5][kThreads / kWave];
  if (!skip && td.has_probe) select_begin(l, td, ls, glob, ema_partials, counters, sc.step_id, hp.sparsity_ppm, hp.topk_abs, s_red);
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
    // lambda_l = largest |h_i| (always inside the mask); accumulated by the EMA kernel of this step
    if (td.has_probe) {
      ls.lambda = u2f(ls.acc_maxkey);
      ls.curv_nonfinite = ls.acc_nonfinite;
    } else {
      ls.curv_nonfinite = 0;
    }
    if (hp.lambda_source == 1) ls.lambda = ls.lambda_power;
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
    glob->hist_pending[(sc.step_id + 1u) & 1u] = 0;
    glob->mask_pending[(sc.step_id + 1u) & 1u] = 0;
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
    // the host's copy, written straight into pinned host memory (read after the stream has been
    // waited for): no separate device-to-host copy in the stream
    host_result->res_skipped = skip ? 1 : 0;
    host_result->res_next_scale = next;
    host_result->res_step_id = sc.step_id;
  }
}

// ---------------------------------------------------------------------------------------------
// Host-side launchers
// ---------------------------------------------------------------------------------------------
hipError_t launch_grad_stats(const DeviceTables& t, const StepArg& sa, hipStream_t s) {
  hipLaunchKernelGGL(k_grad_stats, dim3(t.total_chunks), dim3(kThreads), 0, s, t.tensors, t.chunks, t.partials,
                     t.layers, t.glob, sa);
  TA_LAUNCH_CHECK();
  return hipSuccess;
}

hipError_t launch_curv_ema(const DeviceTables& t, const StepArg& sa, float beta_h, float omb_h, int fisher,
                           hipStream_t s) {
  if (fisher)
    hipLaunchKernelGGL(k_curv_ema<true>, dim3(t.total_chunks), dim3(kThreads), 0, s, t.tensors, t.chunks, t.layers,
                       t.glob, t.ema_partials, t.cands, t.cand_counters, sa, beta_h, omb_h);
  else
    hipLaunchKernelGGL(k_curv_ema<false>, dim3(t.total_chunks), dim3(kThreads), 0, s, t.tensors, t.chunks, t.layers,
                       t.glob, t.ema_partials, t.cands, t.cand_counters, sa, beta_h, omb_h);
  TA_LAUNCH_CHECK();
  return hipSuccess;
}

hipError_t launch_hist_pass(const DeviceTables& t, const StepArg& sa, int serial_rounds, hipStream_t s) {
  const uint32_t grid = t.total_chunks < t.persistent_grid ? t.total_chunks : t.persistent_grid;
  hipLaunchKernelGGL(k_hist_pass, dim3(grid), dim3(kThreads), 0, s, t.tensors, t.chunks, t.total_chunks, t.layers,
                     t.glob, t.hist, sa, serial_rounds);
  TA_LAUNCH_CHECK();
  return hipSuccess;
}

hipError_t launch_select_finish(const DeviceTables& t, const StepArg& sa, float beta_h, hipStream_t s) {
  hipLaunchKernelGGL(k_select_finish, dim3(t.n_tensors), dim3(kFinishThreads), 0, s, t.tensors, t.layers, t.glob,
                     t.cands, t.cand_counters, sa, beta_h);
  TA_LAUNCH_CHECK();
  return hipSuccess;
}

hipError_t launch_layer(const DeviceTables& t, const StepArg& sa, const Hyper& hp, hipStream_t s) {
  hipLaunchKernelGGL(k_layer, dim3(t.n_tensors), dim3(kThreads), 0, s, t.tensors, t.partials, t.ema_partials,
                     t.cand_counters, t.layers, t.glob, t.host_result, t.trans_list, t.n_tensors, sa, hp);
  TA_LAUNCH_CHECK();
  return hipSuccess;
}

}  // namespace triaccel

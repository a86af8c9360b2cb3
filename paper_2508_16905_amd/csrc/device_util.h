// Device helpers shared by the translation units of the optimizer-step kernels: wavefront
// reductions, the mask-word gather, the candidate lists and the fallback mask pass of a chunk.
#pragma once
#include <hip/hip_runtime.h>

#include "kernels.h"
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

__device__ __forceinline__ bool step_skipped(const GlobalDev* glob, uint64_t step_id) {
  return *reinterpret_cast<const volatile uint64_t*>(&glob->skip_epoch) == step_id;
}

__device__ __forceinline__ StepScalars step_scalars(const StepArg& sa) { return sa.dev ? *sa.dev : sa.value; }

__device__ __forceinline__ uint32_t elem_size(int code) { return code == kFP32 ? 4u : 2u; }

// Data-parallel-primitive moves inside the wavefront (no LDS traffic): swap neighbours in a quad,
// swap the quad's halves, then mirror the 8-lane half row (lane i reads lane 7 - i; after the first
// two steps all four lanes of a quad agree, so the mirror brings in the other quad's value).
#define TA_DPP_OR(v, ctrl) ((v) | (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(v), (ctrl), 0xF, 0xF, true))
// Eight consecutive lanes hold the 32 elements of one mask word: combine their 4-bit nibbles.
__device__ __forceinline__ uint32_t gather_mask_word(uint32_t nib, int lane) {
  uint32_t v = nib << (4 * (lane & 7));
  v = TA_DPP_OR(v, 0xB1);   // quad_perm [1, 0, 3, 2]
  v = TA_DPP_OR(v, 0x4E);   // quad_perm [2, 3, 0, 1]
  v = TA_DPP_OR(v, 0x141);  // row_half_mirror
  return v;
}

// Store the kRows mask words of a chunk: lane (8j + r) of a wavefront writes row r's word j.
template <bool FULL>
__device__ __forceinline__ void store_mask_words(const TensorDesc& td, int64_t base, const uint32_t word[kRows]) {
  const int tid = threadIdx.x;
  const int sub = tid & 7;
  if (sub < kRows) {
    uint32_t v = word[0];
#pragma unroll
    for (int r = 1; r < kRows; ++r) v = (sub == r) ? word[r] : v;
    const int64_t widx = ((base + (int64_t)sub * kRowElems) >> 5) + (tid >> 3);
    if (FULL || widx < ((td.numel + 31) >> 5)) as_global<uint32_t>(td.mask)[widx] = v;
  }
}

// Candidate storage.  Each tensor owns kCandLists sub-lists of sub_cap entries plus one overflow
// list of cand_cap entries, each with its own counter in its own 128-byte line: appends from
// different chunks and wavefronts go to different counters, because atomics on one hot address
// serialise.  A batch that does not fit its sub-list spills into the overflow list, so nothing
// is lost as long as the tensor lists at most cand_cap keys in total.
__device__ __forceinline__ uint32_t* cand_counter(uint32_t* counters, uint32_t tensor, uint32_t list) {
  return counters + ((size_t)tensor * (kCandLists + 1) + list) * kCandCounterStride;
}

__device__ __forceinline__ void reset_cand_counters(uint32_t* counters, uint32_t tensor) {
  if (threadIdx.x <= kCandLists) *cand_counter(counters, tensor, threadIdx.x) = 0;
}

// Append a wavefront's candidates of one chunk (flag bit e of `flags` = element e of the lane's
// 16) with one atomic per wavefront: lanes take consecutive slots by a prefix sum.  The sub-list
// is chosen by (chunk, wavefront), so wavefronts running at the same time use different counters.
__device__ __forceinline__ void append_candidates(uint32_t flags, const float (&h)[kRows][4], int64_t base,
                                                  uint32_t chunk_index, uint32_t tensor, const TensorDesc& td,
                                                  Candidate* cands, uint32_t* counters) {
  if (!__any(flags != 0u)) return;  // uniform over the wavefront
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const uint32_t mine = __popc(flags);
  uint32_t incl = mine;
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const uint32_t t = __shfl_up(incl, o);
    if (lane >= o) incl += t;
  }
  const uint32_t total = __shfl(incl, kWave - 1);
  const uint32_t list = (chunk_index * (kThreads / kWave) + wave) % kCandLists;
  uint32_t start = 0, fit = 0, ostart = 0;
  if (lane == 0) {
    start = atomicAdd(cand_counter(counters, tensor, list), total);
    fit = start < td.sub_cap ? min(total, td.sub_cap - start) : 0u;
    if (fit < total) ostart = atomicAdd(cand_counter(counters, tensor, kCandLists), total - fit);
  }
  start = __shfl(start, 0);
  fit = __shfl(fit, 0);
  ostart = __shfl(ostart, 0);
  uint32_t rank = incl - mine;
  Candidate* lists = cands + td.cand_offset;
#pragma unroll
  for (int r = 0; r < kRows; ++r) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (flags & (1u << (r * 4 + i))) {
        const int64_t idx = base + r * kRowElems + threadIdx.x * kVec + i;
        const Candidate c{(uint32_t)idx, f2u(h[r][i]) & 0x7fffffffu};
        if (rank < fit) {
          lists[(size_t)list * td.sub_cap + start + rank] = c;
        } else {
          const uint32_t o = ostart + (rank - fit);
          if (o < td.cand_cap) lists[(size_t)kCandLists * td.sub_cap + o] = c;
        }
        ++rank;
      }
    }
  }
}

// Visit every listed candidate of a tensor.  s_counts holds the kCandLists + 1 clamped counts.
template <int NT, typename F>
__device__ __forceinline__ void for_each_candidate(const TensorDesc& td, const Candidate* cands,
                                                   const uint32_t* s_counts, F f) {
  const uint32_t lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  for (uint32_t list = wave; list <= kCandLists; list += NT / kWave) {
    const uint32_t cnt = s_counts[list];
    const Candidate* p = cands + td.cand_offset + (size_t)list * td.sub_cap;
    for (uint32_t j = lane; j < cnt; j += kWave) f(p[j]);
  }
}

// ---------------------------------------------------------------------------------------------
// Fallback mask pass for tensors whose mask was not settled by the EMA kernel: re-reads |h| and
// writes the bit mask.  Keys above the range are kept, keys below dropped; keys inside it are
// listed and their bits are set afterwards by k_select_finish.  Called from k_update.
// ---------------------------------------------------------------------------------------------
template <bool FULL>
__device__ __forceinline__ void mask_chunk(const TensorDesc& td, int64_t base, uint32_t mode, uint32_t theta,
                                           uint32_t rng_lo, uint32_t rng_hi, uint32_t chunk_index,
                                           uint32_t tensor, Candidate* cands, uint32_t* counters) {
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
  uint32_t cflags = 0;
#pragma unroll
  for (int r = 0; r < kRows; ++r) {
    uint32_t nib = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t key = f2u(h[r][i]) & 0x7fffffffu;  // guarded fill 0: never kept, never listed
      if (mode == kSelExact) {
        if (key >= theta && key != 0u) nib |= 1u << i;
      } else if (key >= rng_hi) {
        nib |= 1u << i;
      } else if (key != 0u && key >= rng_lo) {
        cflags |= 1u << (r * 4 + i);
      }
    }
    word[r] = gather_mask_word(nib, lane);
  }
  store_mask_words<FULL>(td, base, word);
  append_candidates(cflags, h, base, chunk_index, tensor, td, cands, counters);
}

// ---------------------------------------------------------------------------------------------
// Host-side launchers
// ---------------------------------------------------------------------------------------------
#define TA_LAUNCH_CHECK()                      \
  do {                                         \
    hipError_t e_ = hipGetLastError();         \
    if (e_ != hipSuccess) return e_;           \
  } while (0)

}  // namespace triaccel

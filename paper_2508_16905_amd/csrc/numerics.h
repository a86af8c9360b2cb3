// Device-side number-format conversions and 4-element vector accessors (gfx950).
//
// IEEE round-to-nearest-even, overflow to infinity, subnormals produced exactly, NaN kept NaN.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace triaccel {

enum : int { kFP16 = 0, kBF16 = 1, kFP32 = 2 };

__device__ __forceinline__ uint32_t f2u(float f) { return __float_as_uint(f); }
__device__ __forceinline__ float u2f(uint32_t u) { return __uint_as_float(u); }

// Conversions use the gfx950 conversion instructions through the language casts: v_cvt_f16_f32 /
// v_cvt_pk_bf16_f32 round to nearest even (the mode HIP kernels run in), overflow to infinity
// and produce subnormals exactly; v_cvt_f32_f16 and the 16-bit shift of bfloat16 are exact.
// The result is checked against the CPU oracle for all 2^32 inputs by the GPU test suite.
//
// The fp32 value is pinned in a register before it is narrowed: otherwise the compiler may merge
// the producing fused multiply-add with the conversion into one mixed-precision instruction that
// rounds the exact product-sum once, straight to 16 bits, instead of first to fp32 and then to 16
// bits as the update is defined.
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float x) {
  asm volatile("" : "+v"(x));
  const __bf16 b = (__bf16)x;
  return (uint32_t)__builtin_bit_cast(unsigned short, b);
}

__device__ __forceinline__ uint32_t f32_to_f16_bits(float x) {
  asm volatile("" : "+v"(x));
  const _Float16 h = (_Float16)x;
  return (uint32_t)__builtin_bit_cast(unsigned short, h);
}

__device__ __forceinline__ float f16_bits_to_f32(uint32_t h) {
  return (float)__builtin_bit_cast(_Float16, (unsigned short)h);
}

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return u2f(b << 16); }

// ---- 4 consecutive elements, index multiple of 4, base 16-byte aligned ------------------------
// Every tensor is streamed exactly once per kernel, so the vector accesses carry the
// non-temporal hint (measured on MI355X: read-only streaming 6.5 -> 7.3 TB/s, read-modify-write
// 5.3 -> 5.7 TB/s).
typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t v2u __attribute__((ext_vector_type(2)));

// Tensor pointers reach the kernels through tables in memory, so the compiler cannot tell that they
// point to global memory and would emit FLAT accesses.  A wavefront cannot count flat loads back
// one by one (they may be served by another memory), so it waits for ALL its outstanding loads
// before it uses the first result -- in the middle of a batch of loads that serialises their
// latencies.  Every tensor is device (global) memory by the library's contract: say so.
#define TA_GLOBAL __attribute__((address_space(1)))

template <typename T>
__device__ __forceinline__ const TA_GLOBAL T* as_global(const void* p) {
  return (const TA_GLOBAL T*)(p);
}
template <typename T>
__device__ __forceinline__ TA_GLOBAL T* as_global(void* p) {
  return (TA_GLOBAL T*)(p);
}

template <int DT>
__device__ __forceinline__ void load4(const void* base, int64_t idx, float out[4]) {
  if constexpr (DT == kFP32) {
    const v4f v = __builtin_nontemporal_load(as_global<v4f>(static_cast<const float*>(base) + idx));
    out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
  } else {
    const v2u v = __builtin_nontemporal_load(as_global<v2u>(static_cast<const uint16_t*>(base) + idx));
    const uint32_t h0 = v.x & 0xffffu, h1 = v.x >> 16, h2 = v.y & 0xffffu, h3 = v.y >> 16;
    if constexpr (DT == kBF16) {
      out[0] = bf16_bits_to_f32(h0); out[1] = bf16_bits_to_f32(h1);
      out[2] = bf16_bits_to_f32(h2); out[3] = bf16_bits_to_f32(h3);
    } else {
      out[0] = f16_bits_to_f32(h0); out[1] = f16_bits_to_f32(h1);
      out[2] = f16_bits_to_f32(h2); out[3] = f16_bits_to_f32(h3);
    }
  }
}

template <int DT>
__device__ __forceinline__ float load1(const void* base, int64_t idx) {
  if constexpr (DT == kFP32) return as_global<float>(base)[idx];
  const uint32_t h = as_global<uint16_t>(base)[idx];
  if constexpr (DT == kBF16) return bf16_bits_to_f32(h);
  return f16_bits_to_f32(h);
}

template <int DT>
__device__ __forceinline__ void store4(void* base, int64_t idx, const float v[4]) {
  if constexpr (DT == kFP32) {
    v4f o;
    o.x = v[0]; o.y = v[1]; o.z = v[2]; o.w = v[3];
    __builtin_nontemporal_store(o, as_global<v4f>(static_cast<float*>(base) + idx));
  } else {
    uint32_t h[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) h[i] = (DT == kBF16) ? f32_to_bf16_bits(v[i]) : f32_to_f16_bits(v[i]);
    v2u o;
    o.x = h[0] | (h[1] << 16);
    o.y = h[2] | (h[3] << 16);
    __builtin_nontemporal_store(o, as_global<v2u>(static_cast<uint16_t*>(base) + idx));
  }
}

template <int DT>
__device__ __forceinline__ void store1(void* base, int64_t idx, float v) {
  if constexpr (DT == kFP32) as_global<float>(base)[idx] = v;
  else if constexpr (DT == kBF16) as_global<uint16_t>(base)[idx] = static_cast<uint16_t>(f32_to_bf16_bits(v));
  else as_global<uint16_t>(base)[idx] = static_cast<uint16_t>(f32_to_f16_bits(v));
}

// Guarded variants for the ragged end of a tensor: elements at or beyond `n` read as `fill`
// and are not written.
template <int DT>
__device__ __forceinline__ void load4_guard(const void* base, int64_t idx, int64_t n, float fill, float out[4]) {
  if (idx + 4 <= n) { load4<DT>(base, idx, out); return; }
#pragma unroll
  for (int i = 0; i < 4; ++i) out[i] = (idx + i < n) ? load1<DT>(base, idx + i) : fill;
}

template <int DT>
__device__ __forceinline__ void store4_guard(void* base, int64_t idx, int64_t n, const float v[4]) {
  if (idx + 4 <= n) { store4<DT>(base, idx, v); return; }
#pragma unroll
  for (int i = 0; i < 4; ++i)
    if (idx + i < n) store1<DT>(base, idx + i, v[i]);
}

}  // namespace triaccel

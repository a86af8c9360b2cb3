// Device-side number-format conversions and 4-element vector accessors (gfx950).
//
// Conversions are integer bit manipulation so that their result does not depend on the
// wavefront's floating-point mode: IEEE round-to-nearest-even, overflow to infinity,
// subnormals produced exactly, NaN kept quiet.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace triaccel {

enum : int { kFP16 = 0, kBF16 = 1, kFP32 = 2 };

__device__ __forceinline__ uint32_t f2u(float f) { return __float_as_uint(f); }
__device__ __forceinline__ float u2f(uint32_t u) { return __uint_as_float(u); }

__device__ __forceinline__ uint32_t f32_to_bf16_bits(float x) {
  uint32_t u = f2u(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return ((u >> 16) & 0x8000u) | 0x7fc0u;  // NaN
  u += 0x7fffu + ((u >> 16) & 1u);  // ties to even; carries into the exponent, up to infinity
  return u >> 16;
}

__device__ __forceinline__ uint32_t f32_to_f16_bits(float x) {
  const uint32_t u = f2u(x);
  const uint32_t sign = (u >> 16) & 0x8000u;
  const uint32_t a = u & 0x7fffffffu;
  if (a > 0x7f800000u) return sign | 0x7e00u;   // NaN
  if (a >= 0x477ff000u) return sign | 0x7c00u;  // |x| >= 65520 rounds to infinity
  if (a < 0x38800000u) {                        // |x| < 2^-14: subnormal result, quantum 2^-24
    if (a < 0x33000000u) return sign;           // |x| < 2^-25 rounds to zero
    const uint32_t e = a >> 23;                 // 102 .. 112
    const uint32_t m = (a & 0x007fffffu) | 0x00800000u;
    const uint32_t shift = 126u - e;            // 14 .. 24
    uint32_t q = m >> shift;
    const uint32_t rem = m & ((1u << shift) - 1u);
    const uint32_t half = 1u << (shift - 1u);
    if (rem > half || (rem == half && (q & 1u))) ++q;
    return sign | q;                            // q == 1024 is the smallest normal number
  }
  uint32_t h = (((a >> 23) - 112u) << 10) | ((a >> 13) & 0x3ffu);
  const uint32_t rem = a & 0x1fffu;
  if (rem > 0x1000u || (rem == 0x1000u && (h & 1u))) ++h;  // may carry into the exponent
  return sign | h;
}

__device__ __forceinline__ float f16_bits_to_f32(uint32_t h) {
  const uint32_t sign = (h & 0x8000u) << 16;
  const uint32_t e = (h >> 10) & 31u;
  const uint32_t m = h & 0x3ffu;
  if (e == 0u) {
    if (m == 0u) return u2f(sign);
    // subnormal m * 2^-24: normalise with integer shifts
    const uint32_t lz = __clz(m) - 21u;  // m has at most 10 bits; lz = shifts to reach bit 10
    const uint32_t mm = (m << lz) & 0x3ffu;
    return u2f(sign | ((113u - lz) << 23) | (mm << 13));
  }
  if (e == 31u) return u2f(sign | 0x7f800000u | (m << 13));
  return u2f(sign | ((e + 112u) << 23) | (m << 13));
}

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return u2f(b << 16); }

// ---- 4 consecutive elements, index multiple of 4, base 16-byte aligned ------------------------
// Every tensor is streamed exactly once per kernel, so the vector accesses carry the
// non-temporal hint (measured on MI355X: read-only streaming 6.5 -> 7.3 TB/s, read-modify-write
// 5.3 -> 5.7 TB/s).
typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t v2u __attribute__((ext_vector_type(2)));

template <int DT>
__device__ __forceinline__ void load4(const void* base, int64_t idx, float out[4]) {
  if constexpr (DT == kFP32) {
    const v4f v = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(static_cast<const float*>(base) + idx));
    out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
  } else {
    const v2u v = __builtin_nontemporal_load(reinterpret_cast<const v2u*>(static_cast<const uint16_t*>(base) + idx));
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
  if constexpr (DT == kFP32) return static_cast<const float*>(base)[idx];
  const uint32_t h = static_cast<const uint16_t*>(base)[idx];
  if constexpr (DT == kBF16) return bf16_bits_to_f32(h);
  return f16_bits_to_f32(h);
}

template <int DT>
__device__ __forceinline__ void store4(void* base, int64_t idx, const float v[4]) {
  if constexpr (DT == kFP32) {
    v4f o;
    o.x = v[0]; o.y = v[1]; o.z = v[2]; o.w = v[3];
    __builtin_nontemporal_store(o, reinterpret_cast<v4f*>(static_cast<float*>(base) + idx));
  } else {
    uint32_t h[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) h[i] = (DT == kBF16) ? f32_to_bf16_bits(v[i]) : f32_to_f16_bits(v[i]);
    v2u o;
    o.x = h[0] | (h[1] << 16);
    o.y = h[2] | (h[3] << 16);
    __builtin_nontemporal_store(o, reinterpret_cast<v2u*>(static_cast<uint16_t*>(base) + idx));
  }
}

template <int DT>
__device__ __forceinline__ void store1(void* base, int64_t idx, float v) {
  if constexpr (DT == kFP32) static_cast<float*>(base)[idx] = v;
  else if constexpr (DT == kBF16) static_cast<uint16_t*>(base)[idx] = static_cast<uint16_t>(f32_to_bf16_bits(v));
  else static_cast<uint16_t*>(base)[idx] = static_cast<uint16_t>(f32_to_f16_bits(v));
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

// Runtime-dtype variants (the dtype is uniform over a workgroup, so the branch does not diverge).
__device__ __forceinline__ void load4_rt(int dt, const void* base, int64_t idx, int64_t n, bool full, float out[4]) {
  if (dt == kFP32) { if (full) load4<kFP32>(base, idx, out); else load4_guard<kFP32>(base, idx, n, 0.0f, out); }
  else if (dt == kBF16) { if (full) load4<kBF16>(base, idx, out); else load4_guard<kBF16>(base, idx, n, 0.0f, out); }
  else { if (full) load4<kFP16>(base, idx, out); else load4_guard<kFP16>(base, idx, n, 0.0f, out); }
}

__device__ __forceinline__ void store4_rt(int dt, void* base, int64_t idx, int64_t n, bool full, const float v[4]) {
  if (dt == kFP32) { if (full) store4<kFP32>(base, idx, v); else store4_guard<kFP32>(base, idx, n, v); }
  else if (dt == kBF16) { if (full) store4<kBF16>(base, idx, v); else store4_guard<kBF16>(base, idx, n, v); }
  else { if (full) store4<kFP16>(base, idx, v); else store4_guard<kFP16>(base, idx, n, v); }
}

}  // namespace triaccel

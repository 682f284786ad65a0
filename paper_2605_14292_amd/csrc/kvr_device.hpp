// Device-side helpers shared by the kvr kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kvr {

constexpr int kD = 128;          // head dimension every kernel is written for
constexpr int kWave = 64;

enum : int { DT_F32 = 0, DT_BF16 = 1 };

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// Eight consecutive elements of a row, widened to fp32.  `p` points at the
// first of them and is 16-byte aligned.
template <int DT>
__device__ __forceinline__ void load8(const void* p, float (&x)[8]) {
  if constexpr (DT == DT_BF16) {
    const uint4 w = *reinterpret_cast<const uint4*>(p);
    x[0] = bf16_lo(w.x); x[1] = bf16_hi(w.x);
    x[2] = bf16_lo(w.y); x[3] = bf16_hi(w.y);
    x[4] = bf16_lo(w.z); x[5] = bf16_hi(w.z);
    x[6] = bf16_lo(w.w); x[7] = bf16_hi(w.w);
  } else {
    const float4 a = reinterpret_cast<const float4*>(p)[0];
    const float4 b = reinterpret_cast<const float4*>(p)[1];
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
    x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
  }
}

template <int DT> __device__ __forceinline__ constexpr int elem_bytes() { return DT == DT_BF16 ? 2 : 4; }

// Monotone map float -> uint32 (larger float <=> larger key; -inf and NaNs
// still give a key, so a comparison never sees an "empty" candidate).
__device__ __forceinline__ uint32_t ordered_key(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key_to_float(uint32_t k) {
  const uint32_t u = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
  return __uint_as_float(u);
}
// 64-bit argmax key: gain in the high word, ~index in the low word, so that a
// plain unsigned max picks the larger gain and, among equal gains, the lower
// token index.  Key 0 is reserved for "already selected".
__device__ __forceinline__ unsigned long long pack_key(float gain, int idx) {
  return (static_cast<unsigned long long>(ordered_key(gain)) << 32) |
         static_cast<unsigned long long>(0xffffffffu - static_cast<uint32_t>(idx));
}
__device__ __forceinline__ int key_index(unsigned long long k) {
  return static_cast<int>(0xffffffffu - static_cast<uint32_t>(k & 0xffffffffull));
}
__device__ __forceinline__ float key_gain(unsigned long long k) {
  return key_to_float(static_cast<uint32_t>(k >> 32));
}

__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long k) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const unsigned long long o = __shfl_xor(k, off, kWave);
    k = o > k ? o : k;
  }
  return k;
}

// Sum over each aligned group of 16 lanes; every lane of the group gets it.
__device__ __forceinline__ float group16_sum(float v) {
#pragma unroll
  for (int off = 8; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

}  // namespace kvr

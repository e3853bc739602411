// Device-side helpers shared by the gfx950 kernels: bf16 conversion, wave64
// reductions, Philox4x32-10 and the uniform -> Gumbel mapping.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace copris {

constexpr int kWave = 64;

// ---- bf16 <-> fp32 (bit patterns; round to nearest even on the way down) ----
__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
  return __uint_as_float(static_cast<uint32_t>(b) << 16);
}
__device__ __forceinline__ float bf16lo_to_f32(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16hi_to_f32(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0;           // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<uint16_t>(u >> 16);
}

// ---- wave64 reductions (all lanes end with the result) ----
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ int wave_sum_i(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

// ---- Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11) ----
struct Philox4 { uint32_t x, y, z, w; };

__device__ __forceinline__ Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                 uint32_t k0, uint32_t k1) {
  constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
  constexpr uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    // one 32x32->64 multiply per product (v_mad_u64_u32) instead of a hi/lo pair
    const uint64_t p0 = static_cast<uint64_t>(M0) * c0;
    const uint64_t p1 = static_cast<uint64_t>(M1) * c2;
    const uint32_t hi0 = static_cast<uint32_t>(p0 >> 32), lo0 = static_cast<uint32_t>(p0);
    const uint32_t hi1 = static_cast<uint32_t>(p1 >> 32), lo1 = static_cast<uint32_t>(p1);
    c0 = hi1 ^ c1 ^ k0;
    c1 = lo1;
    c2 = hi0 ^ c3 ^ k1;
    c3 = lo0;
    k0 += W0;
    k1 += W1;
  }
  return Philox4{c0, c1, c2, c3};
}

// A 32-bit word -> the midpoint of one of 2^23 equal cells of (0,1): exact in
// fp32, never 0 or 1.
__device__ __forceinline__ float word_to_uniform(uint32_t x) {
  return (static_cast<float>(x >> 9) + 0.5f) * 0x1.0p-23f;
}

// Standard Gumbel variate -ln(-ln u).  The inner logarithm must keep RELATIVE
// accuracy where u is close to 1 (its result is then close to 0), so it is the
// full-precision logf, not the hardware approximation.
__device__ __forceinline__ float gumbel_from_uniform(float u) {
  const float w = -logf(u);        // in [6e-8, 16.7]
  return -logf(w);
}

}  // namespace copris

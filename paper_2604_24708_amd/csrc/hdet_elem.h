// Element access for activation tensors that are fp32 in full precision and bfloat16 (stored
// as uint16_t, round to nearest even) in mixed precision.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

__device__ __forceinline__ float hdet_ld(const float* p) { return *p; }
__device__ __forceinline__ float hdet_ld(const uint16_t* p) { return __uint_as_float((unsigned)(*p) << 16); }
__device__ __forceinline__ void hdet_st(float* p, float x) { *p = x; }
__device__ __forceinline__ void hdet_st(uint16_t* p, float x) {
  unsigned u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) { *p = (uint16_t)((u >> 16) | 0x0040u); return; }
  u += 0x7fffu + ((u >> 16) & 1u);
  *p = (uint16_t)(u >> 16);
}

__device__ __forceinline__ float hdet_wave_sum(float x) {
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
  return x;
}
__device__ __forceinline__ float hdet_wave_max(float x) {
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
  return x;
}

// Philox-4x32 with 10 rounds (Salmon et al., SC'11); used for dropout masks.
struct hdet_philox4 { uint32_t x[4]; };
__device__ __forceinline__ hdet_philox4 hdet_philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                           uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int rnd = 0; rnd < 10; ++rnd) {
    if (rnd > 0) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n1 = (uint32_t)p1;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    const uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
  }
  hdet_philox4 o = {{c0, c1, c2, c3}};
  return o;
}

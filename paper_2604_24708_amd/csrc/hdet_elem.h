// Element access for activation tensors that are fp32 in full precision and bfloat16 (stored
// as uint16_t, round to nearest even) in mixed precision.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

__device__ __forceinline__ float hdet_ld(const float* p) { return *p; }
__device__ __forceinline__ float hdet_ld(const uint16_t* p) { return __uint_as_float((unsigned)(*p) << 16); }
__device__ __forceinline__ void hdet_st(float* p, float x) { *p = x; }
__device__ __forceinline__ void hdet_st(uint16_t* p, float x) { *p = __builtin_bit_cast(unsigned short, (__bf16)x); }

// Eight consecutive elements (16-byte aligned for bf16, 32-byte for fp32) in one or two
// 128-bit accesses.
struct hdet_f8 { float v[8]; };
typedef float hdet_f4v __attribute__((ext_vector_type(4)));
typedef unsigned int hdet_u4v __attribute__((ext_vector_type(4)));
__device__ __forceinline__ hdet_f8 hdet_ld8(const float* p) {
  const hdet_f4v a = *reinterpret_cast<const hdet_f4v*>(p), b = *reinterpret_cast<const hdet_f4v*>(p + 4);
  hdet_f8 r = {{a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]}};
  return r;
}
__device__ __forceinline__ hdet_f8 hdet_ld8(const uint16_t* p) {
  const hdet_u4v u = *reinterpret_cast<const hdet_u4v*>(p);
  hdet_f8 r;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    r.v[2 * i] = __uint_as_float(u[i] << 16);
    r.v[2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u);
  }
  return r;
}
__device__ __forceinline__ unsigned hdet_bf16_bits(float x) {      // round to nearest even (the hardware conversion)
  return (unsigned)__builtin_bit_cast(unsigned short, (__bf16)x);
}
// two values rounded and packed, lo in the low half: one conversion instruction
typedef float hdet_f2v __attribute__((ext_vector_type(2)));
typedef __bf16 hdet_bf2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned hdet_bf16_pack(float lo, float hi) {
  return __builtin_bit_cast(unsigned, __builtin_convertvector((hdet_f2v){lo, hi}, hdet_bf2v));
}
__device__ __forceinline__ void hdet_st8(float* p, const hdet_f8& x) {
  *reinterpret_cast<hdet_f4v*>(p) = (hdet_f4v){x.v[0], x.v[1], x.v[2], x.v[3]};
  *reinterpret_cast<hdet_f4v*>(p + 4) = (hdet_f4v){x.v[4], x.v[5], x.v[6], x.v[7]};
}
__device__ __forceinline__ void hdet_st8(uint16_t* p, const hdet_f8& x) {
  hdet_u4v u;
#pragma unroll
  for (int i = 0; i < 4; ++i) u[i] = hdet_bf16_pack(x.v[2 * i], x.v[2 * i + 1]);
  *reinterpret_cast<hdet_u4v*>(p) = u;
}

// Four consecutive elements in one access (16 B fp32, 8 B bf16).
struct hdet_f4 { float v[4]; };
typedef unsigned int hdet_u2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ hdet_f4 hdet_ld4(const float* p) {
  const hdet_f4v a = *reinterpret_cast<const hdet_f4v*>(p);
  hdet_f4 r = {{a[0], a[1], a[2], a[3]}};
  return r;
}
__device__ __forceinline__ hdet_f4 hdet_ld4(const uint16_t* p) {
  const hdet_u2v u = *reinterpret_cast<const hdet_u2v*>(p);
  hdet_f4 r = {{__uint_as_float(u[0] << 16), __uint_as_float(u[0] & 0xffff0000u),
                __uint_as_float(u[1] << 16), __uint_as_float(u[1] & 0xffff0000u)}};
  return r;
}
__device__ __forceinline__ void hdet_st4(float* p, const hdet_f4& x) {
  *reinterpret_cast<hdet_f4v*>(p) = (hdet_f4v){x.v[0], x.v[1], x.v[2], x.v[3]};
}
__device__ __forceinline__ void hdet_st4(uint16_t* p, const hdet_f4& x) {
  hdet_u2v u = {hdet_bf16_pack(x.v[0], x.v[1]), hdet_bf16_pack(x.v[2], x.v[3])};
  *reinterpret_cast<hdet_u2v*>(p) = u;
}

// the same accesses marked non-temporal: data that is touched once and is larger than the caches
__device__ __forceinline__ hdet_f4 hdet_ld4_stream(const float* p) {
  const hdet_f4v a = __builtin_nontemporal_load(reinterpret_cast<const hdet_f4v*>(p));
  hdet_f4 r = {{a[0], a[1], a[2], a[3]}};
  return r;
}
__device__ __forceinline__ void hdet_st4_stream(float* p, const hdet_f4& x) {
  __builtin_nontemporal_store((hdet_f4v){x.v[0], x.v[1], x.v[2], x.v[3]}, reinterpret_cast<hdet_f4v*>(p));
}
__device__ __forceinline__ void hdet_st4_stream(uint16_t* p, const hdet_f4& x) {
  const hdet_u2v u = {hdet_bf16_pack(x.v[0], x.v[1]), hdet_bf16_pack(x.v[2], x.v[3])};
  __builtin_nontemporal_store(u, reinterpret_cast<hdet_u2v*>(p));
}

// x of another lane of the same row of 16 lanes, by a data-parallel primitive: CTRL 0xB1 / 0x4E = quad
// permutations [1,0,3,2] / [2,3,0,1], 0x141 / 0x140 = mirror within 8 / 16 lanes
template <int CTRL>
__device__ __forceinline__ float hdet_dpp(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, false));
}
// Reductions over the wavefront, the same value in every lane: four steps inside each row of 16 lanes
// (pairs, quads, 8, 16), then two exchanges between rows.  The order is fixed.
__device__ __forceinline__ float hdet_wave_sum(float x) {
  x += hdet_dpp<0xB1>(x);
  x += hdet_dpp<0x4E>(x);
  x += hdet_dpp<0x141>(x);
  x += hdet_dpp<0x140>(x);
  x += __shfl_xor(x, 16);
  x += __shfl_xor(x, 32);
  return x;
}
__device__ __forceinline__ float hdet_wave_max(float x) {
  x = fmaxf(x, hdet_dpp<0xB1>(x));
  x = fmaxf(x, hdet_dpp<0x4E>(x));
  x = fmaxf(x, hdet_dpp<0x141>(x));
  x = fmaxf(x, hdet_dpp<0x140>(x));
  x = fmaxf(x, __shfl_xor(x, 16));
  x = fmaxf(x, __shfl_xor(x, 32));
  return x;
}

// GELU in its tanh form and its derivative (the transformer's MLP activation)
__device__ __forceinline__ float hdet_gelu_tanh(float z) {
  const float c = 0.7978845608028654f;
  return 0.5f * z * (1.f + tanhf(c * (z + 0.044715f * z * z * z)));
}
__device__ __forceinline__ float hdet_gelu_tanh_grad(float z) {
  const float c = 0.7978845608028654f;
  const float t = tanhf(c * (z + 0.044715f * z * z * z));
  return 0.5f * (1.f + t) + 0.5f * z * (1.f - t * t) * c * (1.f + 3.f * 0.044715f * z * z);
}

// The same two functions for results that are rounded to bfloat16 anyway, on the hardware exp2 and reciprocal
// (absolute error of a few 1e-7).  With u = c (z + 0.044715 z^3):  0.5 (1 + tanh u) = sigma(2u) = 1 / (1 + exp(-2u)), so
//   gelu(z)  = z sigma(2u),        exp(-2u) = exp2(z (k1 + k2 z^2)),  k1 = -2 c log2(e),  k2 = 0.044715 k1
//   gelu'(z) = sigma + z sigma (1 - sigma) 2 u'(z) = sigma (1 + z (1 - sigma) (k3 + k4 z^2)),  k3 = 2 c,  k4 = 6 c 0.044715
// z -> -inf gives exp2 = inf, sigma = 0 and the limits 0 and 0; z -> +inf gives sigma = 1 and the limits z and 1.
__device__ __forceinline__ float hdet_gelu_sigma_fast(float z, float z2) {
  const float k1 = -2.302208198144325f, k2 = -0.1029432395800235f;
  return __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(z * __builtin_fmaf(k2, z2, k1)));
}
__device__ __forceinline__ float hdet_gelu_tanh_fast(float z) {
  return z * hdet_gelu_sigma_fast(z, z * z);
}
__device__ __forceinline__ float hdet_gelu_tanh_grad_fast(float z) {
  const float k3 = 1.5957691216057308f, k4 = 0.21406444881780076f;
  const float z2 = z * z;
  const float sg = hdet_gelu_sigma_fast(z, z2);
  return __builtin_fmaf(sg, (z * (1.f - sg)) * __builtin_fmaf(k4, z2, k3), sg);
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

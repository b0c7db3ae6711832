// Arithmetic of the fan-out update of one element (Sec. 3.2, Eq. 2 generalised to SGD-momentum and AdamW), shared by
// every kernel that applies it: the update kernels proper and the weight-gradient GEMM whose epilogue applies the
// update to the tile it has just formed.
//
// Fused multiply-adds are written out and automatic contraction is off inside these functions, so that every
// replica, every kernel and every launch shape rounds identically: replicas that start identical and see identical
// gradients stay bit-identical (alpha = 0 is plain data parallelism, Sec. 3.2).
#pragma once

#include "hdet_internal.h"

namespace hdet_um {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef unsigned short us4 __attribute__((ext_vector_type(4)));

template <typename T> __device__ __forceinline__ T splat(float x);
template <> __device__ __forceinline__ f4 splat<f4>(float x) { return (f4){x, x, x, x}; }
template <> __device__ __forceinline__ float splat<float>(float x) { return x; }

// fp32 -> bfloat16, round to nearest even; NaN stays NaN.
__device__ __forceinline__ unsigned short to_bf16(float x) {
  unsigned u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x0040u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (unsigned short)(u >> 16);
}

// Per-replica scalars of one update.
struct rep_scalars {
  float lr;
  float step;    // AdamW: lr / (1 - beta1^t)
  float decay;   // AdamW: 1 - lr * wd
  float wd;
};

__device__ __forceinline__ rep_scalars replica_scalars(const hdet_update_args& a, int r) {
#pragma clang fp contract(off)
  rep_scalars s;
  s.lr = (float)hdet_channel_value(a.ctrl, a.lr_channel, r, a.eta_sched);
  s.wd = a.wd_channel >= 0 ? (float)hdet_channel_value(a.ctrl, a.wd_channel, r, 0.0) : (float)a.wd_const;
  s.decay = (float)(1.0 - (double)s.lr * (double)s.wd);
  s.step = (float)((double)s.lr * a.inv_bc1);
  return s;
}

template <typename T> __device__ __forceinline__ T fma_(float a, T b, T c) {
  return __builtin_elementwise_fma(splat<T>(a), b, c);
}

template <int OPT, typename T>
__device__ __forceinline__ void update_one(T& th, T g, T& m, T& v, const hdet_update_args& a,
                                           const rep_scalars& s) {
#pragma clang fp contract(off)
  if (OPT == HDET_ADAMW) {
    // theta *= 1 - lr wd;  m = b1 m + (1-b1) g;  v = b2 v + (1-b2) g^2;
    // theta -= lr/(1-b1^t) * m / (sqrt(v)/sqrt(1-b2^t) + eps)
    th = th * s.decay;
    m = fma_<T>(a.beta1, m, a.one_m_beta1 * g);
    v = fma_<T>(a.beta2, v, a.one_m_beta2 * (g * g));
    const T denom = fma_<T>(a.inv_sqrt_bc2, __builtin_elementwise_sqrt(v), splat<T>(a.eps));
    th = fma_<T>(-s.step, m / denom, th);
  } else {
    // g' = g + wd theta;  buf = g' (first step) or mu buf + g';  theta -= lr buf
    const T gp = fma_<T>(s.wd, th, g);
    m = a.first_step ? gp : fma_<T>(a.momentum, m, gp);
    th = fma_<T>(-s.lr, m, th);
  }
}

// AdamW with the moments kept once for all replicas (they depend on the mean gradient only):
// the same operations as update_one, split into the part that is common to the replicas --
// returns m / (sqrt(v)/sqrt(1-b2^t) + eps) -- and the part that is a replica's own.
template <typename T>
__device__ __forceinline__ T adamw_moments(T g, T& m, T& v, const hdet_update_args& a) {
#pragma clang fp contract(off)
  m = fma_<T>(a.beta1, m, a.one_m_beta1 * g);
  v = fma_<T>(a.beta2, v, a.one_m_beta2 * (g * g));
  const T denom = fma_<T>(a.inv_sqrt_bc2, __builtin_elementwise_sqrt(v), splat<T>(a.eps));
  return m / denom;
}
template <typename T>
__device__ __forceinline__ void adamw_apply(T& th, T ratio, const rep_scalars& s) {
#pragma clang fp contract(off)
  th = th * s.decay;
  th = fma_<T>(-s.step, ratio, th);
}

}  // namespace hdet_um

// Fan-out update (Sec. 3.2, Eq. 2 generalised to SGD-momentum / AdamW), the gradient
// exchange of Algorithm 1 and the converge of Sec. 3.3 (Eq. 3) as single-pass HBM streams.
//
// Layout: every tensor is [N][stride] fp32, plane r = replica r.  A thread owns one 16-byte
// column (4 consecutive parameters) and walks the replica axis, so
//   * each of theta, g, m, v is read once and theta, m, v written once per step
//     (28 B per replica-element for AdamW, 20 B for SGD-momentum, +2 B with a bf16 copy);
//   * the replica mean of the gradients (shared mode) and the replica mean of the updated
//     parameters (fused converge) are formed in registers and cost no extra traffic.
// Loads and stores are 128-bit, coalesced along the parameter axis and non-temporal (every
// byte is touched exactly once per step, far beyond any cache).

#include "hdet_internal.h"

#pragma clang fp contract(off)

namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef unsigned short us4 __attribute__((ext_vector_type(4)));
typedef double d4 __attribute__((ext_vector_type(4)));

// fp64 companions of the column types, for the replica mean of the gradients
__device__ __forceinline__ d4 widen(f4 x) { return __builtin_convertvector(x, d4); }
__device__ __forceinline__ double widen(float x) { return (double)x; }
__device__ __forceinline__ f4 narrow(d4 x) { return __builtin_convertvector(x, f4); }
__device__ __forceinline__ float narrow(double x) { return (float)x; }

constexpr int kThreads = 256;

template <typename T> __device__ __forceinline__ T ld(const float* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const T*>(p));
}
template <typename T> __device__ __forceinline__ void st(float* p, T x) {
  __builtin_nontemporal_store(x, reinterpret_cast<T*>(p));
}

// fp32 -> bfloat16, round to nearest even; NaN stays NaN.
__device__ __forceinline__ unsigned short to_bf16(float x) {
  unsigned u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x0040u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (unsigned short)(u >> 16);
}
__device__ __forceinline__ void st_bf16(uint16_t* p, f4 x) {
  us4 o = {to_bf16(x[0]), to_bf16(x[1]), to_bf16(x[2]), to_bf16(x[3])};
  __builtin_nontemporal_store(o, reinterpret_cast<us4*>(p));
}
__device__ __forceinline__ void st_bf16(uint16_t* p, float x) { *p = to_bf16(x); }

template <typename T> __device__ __forceinline__ T splat(float x);
template <> __device__ __forceinline__ f4 splat<f4>(float x) { return (f4){x, x, x, x}; }
template <> __device__ __forceinline__ float splat<float>(float x) { return x; }

// Per-replica scalars, prepared once per block.
struct rep_scalars {
  float lr[HDET_MAX_REPLICAS];
  float step[HDET_MAX_REPLICAS];    // AdamW: lr / (1 - beta1^t)
  float decay[HDET_MAX_REPLICAS];   // AdamW: 1 - lr * wd
  float wd[HDET_MAX_REPLICAS];
};

// The arithmetic of one element.  Fused multiply-adds are written out and automatic
// contraction is off (see the pragma above), so that every replica, every unrolled copy of
// the loop and every launch shape rounds identically: replicas that start identical and see
// identical gradients stay bit-identical (alpha = 0 is plain data parallelism, Sec. 3.2).
template <typename T> __device__ __forceinline__ T fma_(float a, T b, T c) {
  return __builtin_elementwise_fma(splat<T>(a), b, c);
}

template <int OPT, typename T>
__device__ __forceinline__ void update_one(T& th, T g, T& m, T& v, const hdet_update_args& a,
                                           const rep_scalars& s, int r) {
  if (OPT == HDET_ADAMW) {
    // theta *= 1 - lr wd;  m = b1 m + (1-b1) g;  v = b2 v + (1-b2) g^2;
    // theta -= lr/(1-b1^t) * m / (sqrt(v)/sqrt(1-b2^t) + eps)
    th = th * s.decay[r];
    m = fma_<T>(a.beta1, m, a.one_m_beta1 * g);
    v = fma_<T>(a.beta2, v, a.one_m_beta2 * (g * g));
    const T denom = fma_<T>(a.inv_sqrt_bc2, __builtin_elementwise_sqrt(v), splat<T>(a.eps));
    th = fma_<T>(-s.step[r], m / denom, th);
  } else {
    // g' = g + wd theta;  buf = g' (first step) or mu buf + g';  theta -= lr buf
    const T gp = fma_<T>(s.wd[r], th, g);
    m = a.first_step ? gp : fma_<T>(a.momentum, m, gp);
    th = fma_<T>(-s.lr[r], m, th);
  }
}

// One column of width `T` at element offset `col` for the replicas r0 .. r0+rg-1.
template <int OPT, int NT, bool SHARED, bool CONV, typename T>
__device__ __forceinline__ void update_column(const hdet_update_args& a, const rep_scalars& s,
                                              int64_t col, int r0, int rg) {
  const int n = a.n_replicas;
  T gbar = splat<T>(0.f);
  if (SHARED) {
    // The paper's gradient AllReduce: mean over the replica axis, r ascending.  Summed in
    // fp64 and rounded to fp32 once: Adam's first steps move by lr * g/(|g| + eps), which
    // magnifies a last-place difference in a near-zero mean gradient ten-thousandfold.
    auto sum = widen(splat<T>(0.f));
#pragma unroll
    for (int q = 0; q < (NT ? NT : n); ++q) sum = sum + widen(ld<T>(a.grad + (int64_t)q * a.stride + col));
    gbar = narrow(sum * (1.0 / (double)n));
  }
  // Eq. 3 accumulator, fp64: the sum of N fp32 values is then exact up to 2^-53, the mean is
  // rounded to fp32 once, and averaging identical replicas returns them bit for bit.
  auto acc = widen(splat<T>(0.f));
#pragma unroll
  for (int q = 0; q < (NT ? NT : rg); ++q) {
    const int r = r0 + q;
    const int64_t off = (int64_t)r * a.stride + col;
    T th = ld<T>(a.theta + off);
    T g = SHARED ? gbar : ld<T>(a.grad + off);
    T m = ld<T>(a.m + off);
    T v = splat<T>(0.f);
    if (OPT == HDET_ADAMW) v = ld<T>(a.v + off);
    update_one<OPT, T>(th, g, m, v, a, s, r);
    st<T>(a.m + off, m);
    if (OPT == HDET_ADAMW) st<T>(a.v + off, v);
    if (CONV) {
      acc = acc + widen(th);          // Eq. 3: sum in the order r = 0..N-1
    } else {
      st<T>(a.theta + off, th);
      if (a.shadow) st_bf16(a.shadow + off, th);
    }
  }
  if (CONV) {
    const T mean = narrow(acc * (1.0 / (double)n));
#pragma unroll
    for (int q = 0; q < (NT ? NT : n); ++q) {
      const int64_t off = (int64_t)q * a.stride + col;
      st<T>(a.theta + off, mean);
      if (a.shadow) st_bf16(a.shadow + off, mean);
    }
  }
}

// NT = replicas per thread fixed at compile time (0: taken from the arguments).  SHARED and
// CONV need the whole replica axis in one thread, i.e. rg == N and gridDim.y == 1.
template <int OPT, int NT, bool SHARED, bool CONV>
__global__ __launch_bounds__(kThreads) void hdet_update_kernel(const hdet_update_args a) {
  __shared__ rep_scalars s;
  const int n = a.n_replicas;
  if ((int)threadIdx.x < n) {
    const int r = threadIdx.x;
    const float lr = (float)hdet_channel_value(a.ctrl, 0, r, a.eta_sched);
    const float wd = a.wd_channel >= 0 ? (float)hdet_channel_value(a.ctrl, a.wd_channel, r, 0.0)
                                       : (float)a.wd_const;
    s.lr[r] = lr;
    s.wd[r] = wd;
    s.decay[r] = (float)(1.0 - (double)lr * (double)wd);
    s.step[r] = (float)((double)lr * a.inv_bc1);
    if (blockIdx.x == 0 && blockIdx.y == 0) a.ctrl_out->lr_used[r] = lr;
  }
  __syncthreads();

  const int rg = NT ? NT : a.rg;
  const int r0 = blockIdx.y * rg;
  const int64_t nvec = a.n_params >> 2;
  const int64_t gstride = (int64_t)gridDim.x * kThreads;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < nvec; i += gstride)
    update_column<OPT, NT, SHARED, CONV, f4>(a, s, i << 2, r0, rg);

  // ragged tail: P mod 4 trailing parameters, one per thread of the last block
  if (blockIdx.x == gridDim.x - 1) {
    const int64_t col = (nvec << 2) + threadIdx.x;
    if (col < a.n_params) update_column<OPT, NT, SHARED, CONV, float>(a, s, col, r0, rg);
  }
}

// Standalone converge (Eq. 3): 4 B read + 4 B written per replica-element.
template <int NT, typename T>
__device__ __forceinline__ void converge_column(const hdet_converge_args& a, int64_t col) {
  const int n = a.n_replicas;
  auto acc = widen(splat<T>(0.f));     // fp64 sum, one rounding to fp32 (see update_column)
#pragma unroll
  for (int q = 0; q < (NT ? NT : n); ++q) acc = acc + widen(ld<T>(a.theta + (int64_t)q * a.stride + col));
  const T mean = narrow(acc * (1.0 / (double)n));
#pragma unroll
  for (int q = 0; q < (NT ? NT : n); ++q) {
    const int64_t off = (int64_t)q * a.stride + col;
    st<T>(a.theta + off, mean);
    if (a.shadow) st_bf16(a.shadow + off, mean);
  }
}

template <int NT>
__global__ __launch_bounds__(kThreads) void hdet_converge_kernel(const hdet_converge_args a) {
  const int64_t nvec = a.n_params >> 2;
  const int64_t gstride = (int64_t)gridDim.x * kThreads;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < nvec; i += gstride)
    converge_column<NT, f4>(a, i << 2);
  if (blockIdx.x == gridDim.x - 1) {
    const int64_t col = (nvec << 2) + threadIdx.x;
    if (col < a.n_params) converge_column<NT, float>(a, col);
  }
}

// bf16 copy of the parameters (creation / resume).
__global__ __launch_bounds__(kThreads) void hdet_shadow_kernel(const float* theta, uint16_t* shadow,
                                                               int64_t n_params, int64_t stride) {
  const int64_t base = (int64_t)blockIdx.y * stride;
  const int64_t nvec = n_params >> 2;
  const int64_t gstride = (int64_t)gridDim.x * kThreads;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < nvec; i += gstride)
    st_bf16(shadow + base + (i << 2), *reinterpret_cast<const f4*>(theta + base + (i << 2)));
  if (blockIdx.x == gridDim.x - 1) {
    const int64_t col = (nvec << 2) + threadIdx.x;
    if (col < n_params) st_bf16(shadow + base + col, theta[base + col]);
  }
}

int clamp_blocks(int64_t n_params, int blocks) {
  int64_t need = ((n_params >> 2) + kThreads - 1) / kThreads;
  if (need < 1) need = 1;
  return (int)(need < blocks ? need : blocks);
}

template <int OPT, bool SHARED, bool CONV>
void launch_update_nt(const hdet_update_args& a, dim3 grid, hipStream_t stream) {
  switch (a.rg) {
    case 1: hipLaunchKernelGGL((hdet_update_kernel<OPT, 1, SHARED, CONV>), grid, dim3(kThreads), 0, stream, a); break;
    case 2: hipLaunchKernelGGL((hdet_update_kernel<OPT, 2, SHARED, CONV>), grid, dim3(kThreads), 0, stream, a); break;
    case 4: hipLaunchKernelGGL((hdet_update_kernel<OPT, 4, SHARED, CONV>), grid, dim3(kThreads), 0, stream, a); break;
    case 8: hipLaunchKernelGGL((hdet_update_kernel<OPT, 8, SHARED, CONV>), grid, dim3(kThreads), 0, stream, a); break;
    default: hipLaunchKernelGGL((hdet_update_kernel<OPT, 0, SHARED, CONV>), grid, dim3(kThreads), 0, stream, a); break;
  }
}

template <int OPT>
void launch_update_opt(const hdet_update_args& a, bool shared, bool conv, dim3 grid, hipStream_t stream) {
  if (shared && conv) launch_update_nt<OPT, true, true>(a, grid, stream);
  else if (shared) launch_update_nt<OPT, true, false>(a, grid, stream);
  else if (conv) launch_update_nt<OPT, false, true>(a, grid, stream);
  else launch_update_nt<OPT, false, false>(a, grid, stream);
}

}  // namespace

hipError_t hdet_launch_update(const hdet_update_args& a_in, int optimizer, bool shared, bool fuse_converge,
                              int blocks, hipStream_t stream) {
  hdet_update_args a = a_in;
  if (shared || fuse_converge) a.rg = a.n_replicas;   // whole replica axis in one thread
  if (a.rg < 1 || a.n_replicas % a.rg != 0) a.rg = a.n_replicas;
  dim3 grid(clamp_blocks(a.n_params, blocks), a.n_replicas / a.rg);
  if (optimizer == HDET_ADAMW) launch_update_opt<HDET_ADAMW>(a, shared, fuse_converge, grid, stream);
  else launch_update_opt<HDET_SGDM>(a, shared, fuse_converge, grid, stream);
  return hipGetLastError();
}

hipError_t hdet_launch_converge(const hdet_converge_args& a, int blocks, hipStream_t stream) {
  dim3 grid(clamp_blocks(a.n_params, blocks));
  switch (a.n_replicas) {
    case 2: hipLaunchKernelGGL(hdet_converge_kernel<2>, grid, dim3(kThreads), 0, stream, a); break;
    case 4: hipLaunchKernelGGL(hdet_converge_kernel<4>, grid, dim3(kThreads), 0, stream, a); break;
    case 8: hipLaunchKernelGGL(hdet_converge_kernel<8>, grid, dim3(kThreads), 0, stream, a); break;
    default: hipLaunchKernelGGL(hdet_converge_kernel<0>, grid, dim3(kThreads), 0, stream, a); break;
  }
  return hipGetLastError();
}

hipError_t hdet_launch_shadow(const float* theta, uint16_t* shadow, int64_t n_params, int64_t stride,
                              int n_replicas, int blocks, hipStream_t stream) {
  dim3 grid(clamp_blocks(n_params, blocks), n_replicas);
  hipLaunchKernelGGL(hdet_shadow_kernel, grid, dim3(kThreads), 0, stream, theta, shadow, n_params, stride);
  return hipGetLastError();
}

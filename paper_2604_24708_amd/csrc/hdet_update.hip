// Fan-out update (Sec. 3.2, Eq. 2 generalised to SGD-momentum / AdamW), the gradient
// exchange of Algorithm 1 and the converge of Sec. 3.3 (Eq. 3) as single-pass HBM streams.
//
// Layout: every tensor is [N][stride] fp32, plane r = replica r.  The unit of work is one
// 16-byte column (4 consecutive parameters) of one replica:
//   * each of theta, g, m, v is read once and theta, m, v written once per step
//     (28 B per replica-element for AdamW, 20 B for SGD-momentum, +2 B with a bf16 copy);
//   * the replica mean of the gradients (shared mode) and the replica mean of the updated
//     parameters (fused converge) are formed on chip and cost no extra traffic.
// Loads and stores are 128-bit, coalesced along the parameter axis and non-temporal (every
// byte is touched exactly once per step, far beyond any cache).
//
// Three kernels:
//   plane  -- one thread per (replica, column), replica on blockIdx.y; steps that need no
//             exchange along the replica axis.  One column per thread and a grid that covers
//             the plane exactly streamed fastest on MI355X (about 6.4 TB/s, against 5.9 for
//             persistent blocks with a grid-stride loop).
//   wave   -- N <= 16: the wavefronts of a block are the replicas of one 64-column group;
//             gradients (shared mode) and updated parameters (fused converge) cross the
//             replica axis through LDS, each wavefront then writes its own plane.  Keeps
//             the register footprint of the plane kernel instead of N columns per thread.
//   loop   -- one thread walks the replica axis of a column; any N; also used for the
//             P mod 4 trailing parameters.
// With AdamW on the mean gradient the moments are the same for every replica; they can be kept
// once (one plane each), which takes a step from 28 N to 12 N + 16 bytes per element.

#include "hdet_internal.h"
#include "hdet_update_math.h"

#pragma clang fp contract(off)

namespace {

using namespace hdet_um;
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

__device__ __forceinline__ void st_bf16(uint16_t* p, f4 x) {
  us4 o = {to_bf16(x[0]), to_bf16(x[1]), to_bf16(x[2]), to_bf16(x[3])};
  __builtin_nontemporal_store(o, reinterpret_cast<us4*>(p));
}
__device__ __forceinline__ void st_bf16(uint16_t* p, float x) { *p = to_bf16(x); }

// ---------------------------------------------------------------------------------------
// plane kernel: thread = (replica blockIdx.y, column blockIdx.x * 256 + threadIdx.x)
// ---------------------------------------------------------------------------------------
template <int OPT>
__global__ __launch_bounds__(kThreads) void hdet_update_plane_kernel(const hdet_update_args a) {
  const int r = blockIdx.y;
  const rep_scalars s = replica_scalars(a, r);
  if (blockIdx.x == 0 && threadIdx.x == 0 && a.lr_channel == 0) a.ctrl_out->lr_used[r] = s.lr;
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= (a.n_params >> 2)) return;
  const int64_t off = (int64_t)r * a.stride + (i << 2);
  f4 th = ld<f4>(a.theta + off);
  f4 g = ld<f4>(a.grad + (int64_t)r * a.grad_stride + (i << 2));
  if (a.grad_stride == 0) g = g * a.grad_scale;
  f4 m = ld<f4>(a.m + off);
  f4 v = splat<f4>(0.f);
  if (OPT == HDET_ADAMW) v = ld<f4>(a.v + off);
  update_one<OPT, f4>(th, g, m, v, a, s);
  st<f4>(a.m + off, m);
  if (OPT == HDET_ADAMW) st<f4>(a.v + off, v);
  st<f4>(a.theta + off, th);
  if (a.shadow) st_bf16(a.shadow + off, th);
}

// ---------------------------------------------------------------------------------------
// wave kernel: block = `groups` column groups x N wavefronts; wavefront (grp, r) owns the
// 64 columns of group grp in replica r.  ex[grp * N + r][lane] carries a column across the
// replica axis.
// ---------------------------------------------------------------------------------------
constexpr int kMaxWaves = 16;

// LDS staging for a mean along the replica axis, structure-of-arrays so that every access
// is free of bank conflicts.  val[w][c][lane]: component c of wavefront w's column.
struct exchange_buf {
  float val[kMaxWaves][4][64];
  float mean[kMaxWaves][4][64];      // indexed by group
};

// Every wavefront of group `grp` hands in its column x; all get back the group's replica
// mean.  The 256 scalars of a group are shared out over its threads, each summed once in
// fp64 in the order r = 0..N-1 and rounded to fp32 once (same bits as the loop kernel).
// Ends with every thread past both barriers, so the buffer can be reused at once.
__device__ __forceinline__ f4 exchange_mean(exchange_buf& e, f4 x, int w, int grp, int r, int n, int lane) {
#pragma unroll
  for (int c = 0; c < 4; ++c) e.val[w][c][lane] = x[c];
  __syncthreads();
  const double inv_n = 1.0 / (double)n;
  for (int sidx = r * 64 + lane; sidx < 256; sidx += n * 64) {
    const int c = sidx >> 6, l = sidx & 63;
    double sum = 0.0;
    for (int q = 0; q < n; ++q) sum += (double)e.val[grp * n + q][c][l];
    e.mean[grp][c][l] = (float)(sum * inv_n);
  }
  __syncthreads();
  return (f4){e.mean[grp][0][lane], e.mean[grp][1][lane], e.mean[grp][2][lane], e.mean[grp][3][lane]};
}

// SSTATE (AdamW on the mean gradient): m and v are single planes; the wavefront of replica 0
// reads, advances and writes them, and hands m / (sqrt(v)/sqrt(1-b2^t) + eps) to the other
// wavefronts of its group through LDS.
template <int OPT, bool SHARED, bool CONV, bool SSTATE>
__global__ __launch_bounds__(kMaxWaves * 64) void hdet_update_wave_kernel(const hdet_update_args a,
                                                                          const int groups) {
  static_assert(!SSTATE || (SHARED && OPT == HDET_ADAMW), "one set of moments needs AdamW on the mean gradient");
  __shared__ exchange_buf ex;
  const int n = a.n_replicas;
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int grp = w / n, r = w - grp * n;
  const rep_scalars s = replica_scalars(a, r);
  if (blockIdx.x == 0 && grp == 0 && lane == 0 && a.lr_channel == 0) a.ctrl_out->lr_used[r] = s.lr;
  const int64_t i = ((int64_t)blockIdx.x * groups + grp) * 64 + lane;
  const bool ok = i < (a.n_params >> 2);
  const int64_t off = (int64_t)r * a.stride + (i << 2);
  const int64_t moff = SSTATE ? (i << 2) : off;
  const bool mine = ok && (!SSTATE || r == 0);        // this thread holds moments
  f4 th = splat<f4>(0.f), g = th, m = th, v = th;
  if (ok) {
    th = ld<f4>(a.theta + off);
    g = ld<f4>(a.grad + (int64_t)r * a.grad_stride + (i << 2));
    if (a.grad_stride == 0) g = g * a.grad_scale;
  }
  if (mine) {
    m = ld<f4>(a.m + moff);
    if (OPT == HDET_ADAMW) v = ld<f4>(a.v + moff);
  }
  // the paper's gradient AllReduce: every replica applies the replica mean
  if (SHARED) g = exchange_mean(ex, g, w, grp, r, n, lane);
  if (SSTATE) {
    if (r == 0) {
      const f4 ratio = adamw_moments<f4>(g, m, v, a);
#pragma unroll
      for (int c = 0; c < 4; ++c) ex.mean[grp][c][lane] = ratio[c];
    }
    __syncthreads();
    const f4 ratio = {ex.mean[grp][0][lane], ex.mean[grp][1][lane], ex.mean[grp][2][lane], ex.mean[grp][3][lane]};
    adamw_apply<f4>(th, ratio, s);
    if (CONV) __syncthreads();                        // ex.mean is written again below
  } else {
    update_one<OPT, f4>(th, g, m, v, a, s);
  }
  if (mine) {
    st<f4>(a.m + moff, m);
    if (OPT == HDET_ADAMW) st<f4>(a.v + moff, v);
  }
  // Eq. 3 on the freshly updated parameters
  if (CONV) th = exchange_mean(ex, th, w, grp, r, n, lane);
  if (ok) {
    st<f4>(a.theta + off, th);
    if (a.shadow) st_bf16(a.shadow + off, th);
  }
}

// Standalone converge (Eq. 3) in the same shape: 4 B read + 4 B written per replica-element.
__global__ __launch_bounds__(kMaxWaves * 64) void hdet_converge_wave_kernel(const hdet_converge_args a,
                                                                            const int groups) {
  __shared__ exchange_buf ex;
  const int n = a.n_replicas;
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int grp = w / n, r = w - grp * n;
  const int64_t i = ((int64_t)blockIdx.x * groups + grp) * 64 + lane;
  const bool ok = i < (a.n_params >> 2);
  const int64_t off = (int64_t)r * a.stride + (i << 2);
  f4 th = splat<f4>(0.f);
  if (ok) th = ld<f4>(a.theta + off);
  th = exchange_mean(ex, th, w, grp, r, n, lane);
  if (ok) {
    st<f4>(a.theta + off, th);
    if (a.shadow) st_bf16(a.shadow + off, th);
  }
}

// ---------------------------------------------------------------------------------------
// loop kernel: one thread walks the replica axis of a column of width T (f4 or float).
// ---------------------------------------------------------------------------------------
template <int OPT, bool SHARED, bool CONV, bool SSTATE, typename T>
__device__ __forceinline__ void update_column(const hdet_update_args& a, const rep_scalars* s,
                                              int64_t col) {
  const int n = a.n_replicas;
  T gbar = splat<T>(0.f);
  if (SHARED) {
    // The paper's gradient AllReduce: mean over the replica axis, r ascending.  Summed in
    // fp64 and rounded to fp32 once: Adam's first steps move by lr * g/(|g| + eps), which
    // magnifies a last-place difference in a near-zero mean gradient ten-thousandfold.
    auto sum = widen(splat<T>(0.f));
    if (a.grad_stride == 0) {
      gbar = ld<T>(a.grad + col) * a.grad_scale;
    } else {
      for (int q = 0; q < n; ++q) sum = sum + widen(ld<T>(a.grad + (int64_t)q * a.grad_stride + col));
      gbar = narrow(sum * (1.0 / (double)n));
    }
  }
  T ratio = splat<T>(0.f);
  if (SSTATE) {                        // one set of moments for all replicas
    T m = ld<T>(a.m + col), v = ld<T>(a.v + col);
    ratio = adamw_moments<T>(gbar, m, v, a);
    st<T>(a.m + col, m);
    st<T>(a.v + col, v);
  }
  // Eq. 3 accumulator, fp64: the sum of N fp32 values is then exact up to 2^-53, the mean is
  // rounded to fp32 once, and averaging identical replicas returns them bit for bit.
  auto acc = widen(splat<T>(0.f));
  for (int r = 0; r < n; ++r) {
    const int64_t off = (int64_t)r * a.stride + col;
    T th = ld<T>(a.theta + off);
    if (SSTATE) {
      adamw_apply<T>(th, ratio, s[r]);
    } else {
      T g = SHARED ? gbar : ld<T>(a.grad + (int64_t)r * a.grad_stride + col);
      if (!SHARED && a.grad_stride == 0) g = g * a.grad_scale;
      T m = ld<T>(a.m + off);
      T v = splat<T>(0.f);
      if (OPT == HDET_ADAMW) v = ld<T>(a.v + off);
      update_one<OPT, T>(th, g, m, v, a, s[r]);
      st<T>(a.m + off, m);
      if (OPT == HDET_ADAMW) st<T>(a.v + off, v);
    }
    if (CONV) {
      acc = acc + widen(th);          // Eq. 3: sum in the order r = 0..N-1
    } else {
      st<T>(a.theta + off, th);
      if (a.shadow) st_bf16(a.shadow + off, th);
    }
  }
  if (CONV) {
    const T mean = narrow(acc * (1.0 / (double)n));
    for (int r = 0; r < n; ++r) {
      const int64_t off = (int64_t)r * a.stride + col;
      st<T>(a.theta + off, mean);
      if (a.shadow) st_bf16(a.shadow + off, mean);
    }
  }
}

// tail_only: skip the 16-byte columns (another kernel has done them) and handle only the
// P mod 4 trailing parameters.
template <int OPT, bool SHARED, bool CONV, bool SSTATE>
__global__ __launch_bounds__(kThreads) void hdet_update_loop_kernel(const hdet_update_args a,
                                                                    const int tail_only) {
  __shared__ rep_scalars s[HDET_MAX_REPLICAS];
  if ((int)threadIdx.x < a.n_replicas) {
    s[threadIdx.x] = replica_scalars(a, threadIdx.x);
    if (blockIdx.x == 0 && a.lr_channel == 0) a.ctrl_out->lr_used[threadIdx.x] = s[threadIdx.x].lr;
  }
  __syncthreads();
  const int64_t nvec = a.n_params >> 2;
  if (!tail_only) {
    const int64_t gstride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < nvec; i += gstride)
      update_column<OPT, SHARED, CONV, SSTATE, f4>(a, s, i << 2);
  }
  if (blockIdx.x == gridDim.x - 1) {
    const int64_t col = (nvec << 2) + threadIdx.x;
    if (col < a.n_params) update_column<OPT, SHARED, CONV, SSTATE, float>(a, s, col);
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
  if (!a.tail_only)
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

template <int OPT, bool SHARED, bool CONV, bool SSTATE = false>
void launch_variant(const hdet_update_args& a, int variant, int blocks, hipStream_t stream) {
  const int64_t nvec = a.n_params >> 2;
  const bool tail = (a.n_params & 3) != 0;
  const int n = a.n_replicas;
  const bool exchange = SHARED || CONV;
  bool columns_done = false;
  if (variant == 0 && nvec > 0) {
    // with one gradient plane for all replicas the wave kernel is taken as well: the replicas of a column share a
    // block, so the plane comes from memory once
    if (!exchange && !(a.grad_stride == 0 && n > 1 && n <= kMaxWaves)) {
      const int64_t bx = (nvec + kThreads - 1) / kThreads;
      if (bx <= 0x7fffffff) {
        hipLaunchKernelGGL((hdet_update_plane_kernel<OPT>), dim3((unsigned)bx, n), dim3(kThreads), 0, stream, a);
        columns_done = true;
      }
    } else if (n <= kMaxWaves) {
      int groups = 8 / n;                    // aim at 512-thread blocks
      if (groups < 1) groups = 1;
      const int64_t bx = (nvec + 64 * (int64_t)groups - 1) / (64 * (int64_t)groups);
      if (bx <= 0x7fffffff) {
        hipLaunchKernelGGL((hdet_update_wave_kernel<OPT, SHARED, CONV, SSTATE>), dim3((unsigned)bx), dim3(64 * groups * n), 0,
                           stream, a, groups);
        columns_done = true;
      }
    }
  }
  if (!columns_done)
    hipLaunchKernelGGL((hdet_update_loop_kernel<OPT, SHARED, CONV, SSTATE>), dim3(clamp_blocks(a.n_params, blocks)),
                       dim3(kThreads), 0, stream, a, 0);
  else if (tail)
    hipLaunchKernelGGL((hdet_update_loop_kernel<OPT, SHARED, CONV, SSTATE>), dim3(1), dim3(kThreads), 0, stream, a, 1);
}

template <int OPT>
void launch_update_opt(const hdet_update_args& a, bool shared, bool conv, int variant, int blocks,
                       hipStream_t stream) {
  if (shared && conv) launch_variant<OPT, true, true>(a, variant, blocks, stream);
  else if (shared) launch_variant<OPT, true, false>(a, variant, blocks, stream);
  else if (conv) launch_variant<OPT, false, true>(a, variant, blocks, stream);
  else launch_variant<OPT, false, false>(a, variant, blocks, stream);
}

}  // namespace

hipError_t hdet_launch_update(const hdet_update_args& a, int optimizer, bool shared, bool fuse_converge,
                              int variant, int blocks, hipStream_t stream) {
  if (a.shared_state) {
    if (optimizer != HDET_ADAMW || !shared) return hipErrorInvalidValue;
    if (fuse_converge) launch_variant<HDET_ADAMW, true, true, true>(a, variant, blocks, stream);
    else launch_variant<HDET_ADAMW, true, false, true>(a, variant, blocks, stream);
    return hipGetLastError();
  }
  if (optimizer == HDET_ADAMW) launch_update_opt<HDET_ADAMW>(a, shared, fuse_converge, variant, blocks, stream);
  else launch_update_opt<HDET_SGDM>(a, shared, fuse_converge, variant, blocks, stream);
  return hipGetLastError();
}

hipError_t hdet_launch_converge(const hdet_converge_args& a, int variant, int blocks, hipStream_t stream) {
  const int64_t nvec = a.n_params >> 2;
  const int n = a.n_replicas;
  if (variant == 0 && nvec > 0 && n <= kMaxWaves) {
    int groups = 8 / n;
    if (groups < 1) groups = 1;
    const int64_t bx = (nvec + 64 * (int64_t)groups - 1) / (64 * (int64_t)groups);
    if (bx <= 0x7fffffff) {
      hipLaunchKernelGGL(hdet_converge_wave_kernel, dim3((unsigned)bx), dim3(64 * groups * n), 0, stream, a, groups);
      if (a.n_params & 3) {                     // P mod 4 trailing parameters
        hdet_converge_args t = a;
        t.tail_only = 1;
        hipLaunchKernelGGL(hdet_converge_kernel<0>, dim3(1), dim3(kThreads), 0, stream, t);
      }
      return hipGetLastError();
    }
  }
  hipLaunchKernelGGL(hdet_converge_kernel<0>, dim3(clamp_blocks(a.n_params, blocks)), dim3(kThreads), 0, stream, a);
  return hipGetLastError();
}

hipError_t hdet_launch_shadow(const float* theta, uint16_t* shadow, int64_t n_params, int64_t stride,
                              int n_replicas, int blocks, hipStream_t stream) {
  dim3 grid(clamp_blocks(n_params, blocks), n_replicas);
  hipLaunchKernelGGL(hdet_shadow_kernel, grid, dim3(kThreads), 0, stream, theta, shadow, n_params, stride);
  return hipGetLastError();
}

// Warm noisy initialisation (Sec. 3.5, Eq. 10): theta_r = theta0 + eps_r with
// eps_r ~ N(0, nu^2 ||theta0||^2 / d), independent per replica and element.
//
// Two passes over HBM: a deterministic fp64 sum of squares of the checkpoint (per-block
// partials added in block order), then one kernel that reads theta0 once per replica plane and
// writes the N perturbed planes.  The noise is a pure function of (seed, replica, index):
// elements 4b..4b+3 come from philox(counter = (b, replica, 0, "WARM"), key = seed) through
// two Box-Muller pairs, evaluated in fp64 (a one-off kernel; fp32 logs would lose the tail).

#include "hdet_elem.h"
#include "hdet_internal.h"

namespace {

constexpr uint32_t kWarmStream = 0x5741524Du;   // "WARM"

__global__ __launch_bounds__(256) void sumsq_partial_kernel(const float* theta0, int64_t n, double* partial) {
  __shared__ double red[4];
  double s = 0.0;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const double v = (double)theta0[i];
    s += v * v;
  }
  for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) partial[blockIdx.x] = ((red[0] + red[1]) + red[2]) + red[3];
}

__global__ void sumsq_final_kernel(const double* partial, int nblocks, double* out) {
  double s = 0.0;
  for (int i = 0; i < nblocks; ++i) s += partial[i];
  *out = s;
}

__global__ __launch_bounds__(256) void warm_noise_kernel(const float* theta0, float* theta, int64_t n, int64_t stride,
                                                         const double* sumsq, double nu, uint32_t seed_lo, uint32_t seed_hi) {
  const int r = blockIdx.y;
  const double sigma = nu * sqrt(*sumsq / (double)n);
  const int64_t nblk = (n + 3) >> 2;
  for (int64_t b = (int64_t)blockIdx.x * 256 + threadIdx.x; b < nblk; b += (int64_t)gridDim.x * 256) {
    const hdet_philox4 w = hdet_philox4x32_10((uint32_t)b, (uint32_t)r, 0u, kWarmStream, seed_lo, seed_hi);
    double z[4];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const double u = ((double)w.x[2 * h] + 1.0) * (1.0 / 4294967296.0);      // (0, 1]
      const double v = (double)w.x[2 * h + 1] * (1.0 / 4294967296.0);          // [0, 1)
      const double rad = sqrt(-2.0 * log(u));
      double sn, cs;
      sincos(6.283185307179586476925286766559 * v, &sn, &cs);
      z[2 * h] = rad * cs;
      z[2 * h + 1] = rad * sn;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int64_t i = (b << 2) + j;
      if (i < n) theta[(int64_t)r * stride + i] = (float)((double)theta0[i] + sigma * z[j]);
    }
  }
}

}  // namespace

hipError_t hdet_launch_warm_init(const float* theta0, float* theta, int64_t n_params, int64_t stride, int n_replicas,
                                 hdet_ctrl* ctrl, double nu, uint64_t seed, hipStream_t s) {
  int64_t nb = (n_params + 256 * 64 - 1) / (256 * 64);
  if (nb > HDET_WARM_PARTIALS) nb = HDET_WARM_PARTIALS;
  if (nb < 1) nb = 1;
  hipLaunchKernelGGL(sumsq_partial_kernel, dim3((unsigned)nb), dim3(256), 0, s, theta0, n_params, ctrl->warm_partial);
  hipLaunchKernelGGL(sumsq_final_kernel, dim3(1), dim3(1), 0, s, ctrl->warm_partial, (int)nb, &ctrl->warm_sumsq);
  int64_t gb = ((n_params + 3) / 4 + 255) / 256;
  if (gb > 65536) gb = 65536;
  if (gb < 1) gb = 1;
  hipLaunchKernelGGL(warm_noise_kernel, dim3((unsigned)gb, n_replicas), dim3(256), 0, s, theta0, theta, n_params, stride,
                     &ctrl->warm_sumsq, nu, (uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32));
  return hipGetLastError();
}

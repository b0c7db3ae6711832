// Warm noisy initialisation (Sec. 3.5, Eq. 10): theta_r = theta0 + eps_r with
// eps_r ~ N(0, nu^2 ||theta0||^2 / d), independent per replica and element.
//
// Two passes over HBM: a deterministic fp64 sum of squares of the checkpoint (per-block
// partials added in block order), then one kernel that reads theta0 once and writes the N
// perturbed planes.  The noise is a pure function of (seed, replica, index):
// elements 4b..4b+3 come from philox(counter = (b, replica, 0, "WARM"), key = seed) through
// two Box-Muller pairs (see box_muller_f32).

#include <mutex>
#include <string>

#include "hdet_elem.h"
#include "hdet_internal.h"

namespace {

constexpr uint32_t kWarmStream = 0x5741524Du;   // "WARM"

// Each thread walks 16-byte columns with a grid stride and keeps one fp64 sum per component (four independent
// chains); components, lanes, wavefronts and blocks are then added in a fixed order.
__global__ __launch_bounds__(256) void sumsq_partial_kernel(const float* theta0, int64_t n, double* partial) {
  typedef float f4 __attribute__((ext_vector_type(4)));
  __shared__ double red[4];
  double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
  const int64_t nvec = n >> 2;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += (int64_t)gridDim.x * 256) {
    const f4 v = __builtin_nontemporal_load(reinterpret_cast<const f4*>(theta0) + i);
    s0 += (double)v[0] * (double)v[0];
    s1 += (double)v[1] * (double)v[1];
    s2 += (double)v[2] * (double)v[2];
    s3 += (double)v[3] * (double)v[3];
  }
  double s = (s0 + s1) + (s2 + s3);
  if (blockIdx.x == 0 && threadIdx.x < (n & 3)) {          // the n mod 4 trailing elements
    const double v = (double)theta0[(nvec << 2) + threadIdx.x];
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

// Box-Muller in single precision, arranged so that nothing the result depends on is lost to fp32:
//   -ln u, u = (w0 + 1) / 2^32:  for u <= 1/2 the logarithm of u itself; for u > 1/2, where u is too close to 1 for
//      fp32 to hold, -log1p(-x) of the exactly known small x = (2^32 - 1 - w0) / 2^32;
//   the angle 2 pi v, v = w1 / 2^32, through sin/cos of pi * (2 v), whose range reduction is exact.
// The deviates agree with a double-precision evaluation to about 1e-6 absolute (the angle keeps 24 of w1's 32 bits),
// i.e. to 1e-8 of the parameter scale at nu = 0.01: far inside what an fp32 parameter resolves.
__device__ __forceinline__ void box_muller_f32(uint32_t w0, uint32_t w1, float* z0, float* z1) {
  float t;       // -ln u
  if (w0 < 0x80000000u) t = -logf((float)(w0 + 1u) * 2.3283064365386963e-10f);
  else t = -log1pf(-((float)(0xffffffffu - w0) * 2.3283064365386963e-10f));
  const float rad = sqrtf(2.f * t);
  float sn, cs;
  sincospif((float)w1 * 4.6566128730773926e-10f, &sn, &cs);       // pi * (2 v)
  *z0 = rad * cs;
  *z1 = rad * sn;
}

// thread = one block of four elements in every replica: theta_0 comes from memory once
__global__ __launch_bounds__(256) void warm_noise_kernel(const float* theta0, float* theta, int64_t n, int64_t stride, int n_replicas,
                                                         const double* sumsq, double nu, uint32_t seed_lo, uint32_t seed_hi) {
  typedef float f4 __attribute__((ext_vector_type(4)));
  const float sigma = (float)(nu * sqrt(*sumsq / (double)n));
  const int64_t nblk = (n + 3) >> 2;
  for (int64_t b = (int64_t)blockIdx.x * 256 + threadIdx.x; b < nblk; b += (int64_t)gridDim.x * 256) {
    const int64_t i = b << 2;
    const bool whole = i + 3 < n;     // 16-byte accesses (theta0 and the planes are 16-byte aligned)
    f4 t0 = {0.f, 0.f, 0.f, 0.f};
    if (whole) t0 = __builtin_nontemporal_load(reinterpret_cast<const f4*>(theta0 + i));
    else
      for (int j = 0; j < 4; ++j)
        if (i + j < n) t0[j] = theta0[i + j];
    for (int r = 0; r < n_replicas; ++r) {
      const hdet_philox4 w = hdet_philox4x32_10((uint32_t)b, (uint32_t)r, 0u, kWarmStream, seed_lo, seed_hi);
      float z[4];
      box_muller_f32(w.x[0], w.x[1], &z[0], &z[1]);
      box_muller_f32(w.x[2], w.x[3], &z[2], &z[3]);
      const f4 o = {__builtin_fmaf(sigma, z[0], t0[0]), __builtin_fmaf(sigma, z[1], t0[1]), __builtin_fmaf(sigma, z[2], t0[2]),
                    __builtin_fmaf(sigma, z[3], t0[3])};
      float* dst = theta + (int64_t)r * stride + i;
      if (whole) __builtin_nontemporal_store(o, reinterpret_cast<f4*>(dst));
      else
        for (int j = 0; j < 4; ++j)
          if (i + j < n) dst[j] = o[j];
    }
  }
}

}  // namespace

// partial: HDET_WARM_PARTIALS doubles, sumsq: one double, both device memory that the three kernels own
// for the duration of the call (every entry that is read is written first: nothing has to start at zero)
hipError_t hdet_launch_warm_init(const float* theta0, float* theta, int64_t n_params, int64_t stride, int n_replicas,
                                 double* partial, double* sumsq, double nu, uint64_t seed, hipStream_t s) {
  int64_t nb = (n_params + 256 * 64 - 1) / (256 * 64);
  if (nb > HDET_WARM_PARTIALS) nb = HDET_WARM_PARTIALS;
  if (nb < 1) nb = 1;
  hipLaunchKernelGGL(sumsq_partial_kernel, dim3((unsigned)nb), dim3(256), 0, s, theta0, n_params, partial);
  hipLaunchKernelGGL(sumsq_final_kernel, dim3(1), dim3(1), 0, s, partial, (int)nb, sumsq);
  int64_t gb = ((n_params + 3) / 4 + 255) / 256;
  if (gb > 262144) gb = 262144;
  if (gb < 1) gb = 1;
  hipLaunchKernelGGL(warm_noise_kernel, dim3((unsigned)gb), dim3(256), 0, s, theta0, theta, n_params, stride, n_replicas,
                     sumsq, nu, (uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32));
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// The same initialisation for callers that cannot allocate device memory: no handle (hdet_create
// allocates the control block that holds the partial sums above), the partial sums live in a
// file-scope device array instead.  Every GPU holds its own copy of the array for the life of
// the process; its address on a device is looked up once, with that device current.
// ---------------------------------------------------------------------------------------
namespace {

constexpr int kScratchDoubles = HDET_WARM_PARTIALS + 1;                   // partial sums, then their total
static __device__ __align__(256) double scratch[kScratchDoubles];        // 8200 bytes per GPU

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
double* g_scratch_ptr[kMaxDevices] = {nullptr};

// device address of `scratch` on the current device (host code must never pass the array's name itself)
int scratch_on_current_device(double** out, std::string* why) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) { *why = std::string("hipGetDevice: ") + hipGetErrorString(e); return HDET_EHIP; }
  if (dev < 0 || dev >= kMaxDevices) { *why = "device ordinal out of range"; return HDET_EHIP; }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    double* ptr = nullptr;
    e = hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) { *why = std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e); return HDET_EHIP; }
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return HDET_OK;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

extern "C" int hdet_warm_init_noalloc(const float* theta0_dev, float* params_dev, uint16_t* params_bf16_dev,
                                      int64_t n_params, int64_t plane_stride, int32_t n_replicas, double nu,
                                      uint64_t seed, void* stream) {
  auto bad = [](int code, const std::string& msg) { hdet_set_global_error(msg); return code; };
  if (!theta0_dev || !params_dev) return bad(HDET_EINVAL, "theta0_dev and params_dev are required");
  if (!aligned16(theta0_dev) || !aligned16(params_dev) || !aligned16(params_bf16_dev))
    return bad(HDET_EINVAL, "device pointers must be 16-byte aligned");
  if (n_replicas < 1 || n_replicas > HDET_MAX_REPLICAS) return bad(HDET_EINVAL, "n_replicas out of range");
  if (n_params < 1 || n_params > HDET_WARM_MAX_PARAMS)
    return bad(HDET_EINVAL, "n_params must be in 1 .. 2^34 (the noise generator numbers blocks of four parameters with 32 bits)");
  if (plane_stride < n_params || (plane_stride & 3)) return bad(HDET_EINVAL, "plane_stride must be >= n_params and a multiple of 4");
  if (!(nu >= 0.0)) return bad(HDET_EINVAL, "nu must be >= 0");
  const float* lo = params_dev;
  const float* hi = lo + (int64_t)n_replicas * plane_stride;
  if (theta0_dev + n_params > lo && theta0_dev < hi) return bad(HDET_EINVAL, "theta0_dev must not overlap params_dev");
  double* ptr = nullptr;
  std::string why;
  const int rc = scratch_on_current_device(&ptr, &why);
  if (rc != HDET_OK) return bad(rc, why);
  hipStream_t s = (hipStream_t)stream;
  hipError_t e = hdet_launch_warm_init(theta0_dev, params_dev, n_params, plane_stride, n_replicas, ptr, ptr + HDET_WARM_PARTIALS,
                                       nu, seed, s);
  if (e == hipSuccess && params_bf16_dev)
    e = hdet_launch_shadow(params_dev, params_bf16_dev, n_params, plane_stride, n_replicas, 4096, s);
  if (e != hipSuccess) return bad(HDET_EHIP, std::string("warm initialisation kernels: ") + hipGetErrorString(e));
  return HDET_OK;
}

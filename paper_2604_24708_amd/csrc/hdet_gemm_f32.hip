// Replica-batched fp32 GEMM, LDS-tiled, for the full-precision model path: element strides
// select which of forward / dgrad / wgrad it is, the batch index selects the replica (and,
// for attention, the sequence and head).  64x64 tile per 256-thread block, 4x4 per thread.

#include "hdet_internal.h"

namespace {

constexpr int BM = 64, BN = 64, BK = 16;


// C = A * B with fp32 accumulation; 64x64 tile per 256-thread block, 4x4 per thread.
template <int EPI>
__global__ __launch_bounds__(256) void sgemm_kernel(const hdet_sgemm_args g) {
  __shared__ float As[BK][BM + 4];
  __shared__ float Bs[BK][BN + 4];
  const hdet_batch_index bi = hdet_split_batch(blockIdx.z, g.n1, g.n2);
  const int z = bi.z0;            // replica: bias and mask are per replica
  const float* A = g.a + hdet_batch_offset(bi, g.a_s);
  const float* B = g.b + hdet_batch_offset(bi, g.b_s);
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;
  const bool a_kfast = g.a_cs == 1;      // consecutive threads walk the contiguous axis
  const bool b_nfast = g.b_cs == 1;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < g.k; k0 += BK) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = tid + i * 256;
      const int mm = a_kfast ? e / BK : e % BM;
      const int kk = a_kfast ? e % BK : e / BM;
      const int gm = m0 + mm, gk = k0 + kk;
      As[kk][mm] = (gm < g.m && gk < g.k) ? A[(int64_t)gm * g.a_rs + (int64_t)gk * g.a_cs] : 0.f;
      const int nn = b_nfast ? e % BN : e / BK;
      const int kb = b_nfast ? e / BN : e % BK;
      const int gn = n0 + nn, gkb = k0 + kb;
      Bs[kb][nn] = (gn < g.n && gkb < g.k) ? B[(int64_t)gkb * g.b_rs + (int64_t)gn * g.b_cs] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      float av[4], bv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { av[i] = As[kk][ty * 4 + i]; bv[i] = Bs[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
    }
    __syncthreads();
  }
  float* C = g.c + hdet_batch_offset(bi, g.c_s);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int gm = m0 + ty * 4 + i;
    if (gm >= g.m) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int gn = n0 + tx * 4 + j;
      if (gn >= g.n) continue;
      float v = acc[i][j];
      if (EPI == HDET_SEPI_BIAS || EPI == HDET_SEPI_BIAS_RELU) v += g.bias[(int64_t)z * g.bias_bs + gn];
      if (EPI == HDET_SEPI_BIAS_RELU) v = v > 0.f ? v : 0.f;
      if (EPI == HDET_SEPI_MASK) v = g.mask[(int64_t)z * g.mask_bs + (int64_t)gm * g.mask_rs + gn] > 0.f ? v : 0.f;
      C[(int64_t)gm * g.c_rs + gn] = v;
    }
  }
}


}  // namespace

hipError_t hdet_launch_sgemm(const hdet_sgemm_args& g_in, int epi, int batch, hipStream_t s) {
  hdet_sgemm_args g = g_in;
  if (g.n1 < 1) g.n1 = 1;
  if (g.n2 < 1) g.n2 = 1;
  dim3 grid((g.n + BN - 1) / BN, (g.m + BM - 1) / BM, batch);
  switch (epi) {
    case HDET_SEPI_BIAS: hipLaunchKernelGGL(sgemm_kernel<HDET_SEPI_BIAS>, grid, dim3(256), 0, s, g); break;
    case HDET_SEPI_BIAS_RELU: hipLaunchKernelGGL(sgemm_kernel<HDET_SEPI_BIAS_RELU>, grid, dim3(256), 0, s, g); break;
    case HDET_SEPI_MASK: hipLaunchKernelGGL(sgemm_kernel<HDET_SEPI_MASK>, grid, dim3(256), 0, s, g); break;
    default: hipLaunchKernelGGL(sgemm_kernel<HDET_SEPI_NONE>, grid, dim3(256), 0, s, g); break;
  }
  return hipGetLastError();
}

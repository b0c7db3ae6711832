// Replica-batched bf16 GEMM on the gfx950 matrix cores for the "Forward + backward" of
// Algorithm 1 in mixed precision: bf16 operands, fp32 accumulation, N independent weight
// sets with the replica on blockIdx.z.
//
//   C(m,n) = sum_k A(m,k) * B(k,n)          A, B bfloat16; C fp32 or bfloat16
//
// One kernel serves the three products of a Linear layer; which axis of an operand is
// contiguous in memory differs between them:
//   forward  Y  = X  W^T : A = X [b][k]  (k contiguous)   B(k,n) = W[n][k]  (k contiguous)
//   dgrad    dX = dY W   : A = dY[b][o]  (k=o contiguous) B(k,n) = W[k][n]  (n contiguous)
//   wgrad    dW = dY^T X : A(m,k) = dY[k][m] (m contiguous) B(k,n) = X[k][n] (n contiguous)
// Tiles are staged through LDS in one layout -- rows of the output dimension, the
// contraction index contiguous -- so that every MFMA operand is a single 128-bit LDS read;
// an operand whose memory is contiguous along the other axis is transposed on its way into
// LDS (128-bit coalesced global loads, 16-bit LDS stores).
//
// Tiling: 128x128 output tile per 256-thread block (4 wavefronts, 2x2, 64x64 each as 2x2
// v_mfma_f32_32x32x16_bf16), K step 32, next tile's global loads in flight during the MFMAs.

#include "hdet_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f16v __attribute__((ext_vector_type(16)));
typedef unsigned short us8 __attribute__((ext_vector_type(8)));

constexpr int TM = 128, TN = 128, TK = 32;
constexpr int LDK = TK + 8;           // LDS row pitch in elements: 80 B, keeps rows 16-byte aligned

__device__ __forceinline__ unsigned short f2bf(float x) {
  unsigned u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x0040u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (unsigned short)(u >> 16);
}
__device__ __forceinline__ float bf2f(unsigned short h) { return __uint_as_float((unsigned)h << 16); }

// 8 consecutive elements starting at src[idx], of which the first `valid` exist (others 0).
__device__ __forceinline__ us8 load8(const uint16_t* src, int64_t idx, int valid, bool vec_ok) {
  if (valid >= 8 && vec_ok) return *reinterpret_cast<const us8*>(src + idx);
  us8 r = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
  for (int j = 0; j < 8; ++j)
    if (j < valid) r[j] = src[idx + j];
  return r;
}

// Stages one operand tile (128 rows of the output dimension x 32 of the contraction).
// KMAJOR: element (row, k) at src[row * ld + k]; otherwise at src[k * ld + row].
template <bool KMAJOR>
struct stager {
  us8 reg[2];
  __device__ __forceinline__ void fetch(const uint16_t* src, int64_t ld, int row0, int rows, int k0, int kdim,
                                        bool vec_ok, int tid) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int c = tid + i * 256;
      if (KMAJOR) {
        const int row = row0 + (c >> 2), k = k0 + ((c & 3) << 3);
        const int valid = row < rows ? kdim - k : 0;
        reg[i] = load8(src, (int64_t)row * ld + k, valid, vec_ok);
      } else {
        const int k = k0 + (c >> 4), row = row0 + ((c & 15) << 3);
        const int valid = k < kdim ? rows - row : 0;
        reg[i] = load8(src, (int64_t)k * ld + row, valid, vec_ok);
      }
    }
  }
  __device__ __forceinline__ void commit(uint16_t (*tile)[LDK], int tid) const {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int c = tid + i * 256;
      if (KMAJOR) {
        *reinterpret_cast<us8*>(&tile[c >> 2][(c & 3) << 3]) = reg[i];
      } else {
        const int k = c >> 4, row = (c & 15) << 3;
#pragma unroll
        for (int j = 0; j < 8; ++j) tile[row + j][k] = reg[i][j];
      }
    }
  }
};

}  // namespace

template <bool A_KMAJOR, bool B_KMAJOR, int EPI>
__global__ __launch_bounds__(256) void hdet_bgemm_kernel(const hdet_bgemm_args g) {
  __shared__ __attribute__((aligned(16))) uint16_t As[TM][LDK];
  __shared__ __attribute__((aligned(16))) uint16_t Bs[TN][LDK];
  const int z = blockIdx.z;
  const uint16_t* A = g.a + (int64_t)z * g.a_bs;
  const uint16_t* B = g.b + (int64_t)z * g.b_bs;
  const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
  const bool a_vec = (g.lda & 7) == 0 && (reinterpret_cast<uintptr_t>(A) & 15) == 0;
  const bool b_vec = (g.ldb & 7) == 0 && (reinterpret_cast<uintptr_t>(B) & 15) == 0;

  f16v acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  stager<A_KMAJOR> sa;
  stager<B_KMAJOR> sb;
  sa.fetch(A, g.lda, m0, g.m, 0, g.k, a_vec, tid);
  sb.fetch(B, g.ldb, n0, g.n, 0, g.k, b_vec, tid);
  for (int k0 = 0; k0 < g.k; k0 += TK) {
    sa.commit(As, tid);
    sb.commit(Bs, tid);
    __syncthreads();
    if (k0 + TK < g.k) {
      sa.fetch(A, g.lda, m0, g.m, k0 + TK, g.k, a_vec, tid);
      sb.fetch(B, g.ldb, n0, g.n, k0 + TK, g.k, b_vec, tid);
    }
#pragma unroll
    for (int ks = 0; ks < TK; ks += 16) {
      bf16x8 af[2], bfr[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        af[i] = *reinterpret_cast<const bf16x8*>(&As[wm + i * 32 + (lane & 31)][ks + ((lane >> 5) << 3)]);
        bfr[i] = *reinterpret_cast<const bf16x8*>(&Bs[wn + i * 32 + (lane & 31)][ks + ((lane >> 5) << 3)]);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
  }

  // epilogue: accumulator element e of lane l is C(row, col) with
  //   row = (e / 4) * 8 + (l / 32) * 4 + e % 4,  col = l % 32   inside its 32x32 block
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int col = n0 + wn + j * 32 + (lane & 31);
      if (col >= g.n) continue;
      float bias = 0.f;
      if (EPI == HDET_EPI_BIAS_RELU_BF16 || EPI == HDET_EPI_BIAS_F32) bias = g.bias[(int64_t)z * g.bias_bs + col];
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int row = m0 + wm + i * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
        if (row >= g.m) continue;
        float v = acc[i][j][e];
        const int64_t off = (int64_t)z * g.c_bs + (int64_t)row * g.ldc + col;
        if (EPI == HDET_EPI_F32) {
          reinterpret_cast<float*>(g.c)[off] = v;
        } else if (EPI == HDET_EPI_BIAS_F32) {
          reinterpret_cast<float*>(g.c)[off] = v + bias;
        } else if (EPI == HDET_EPI_BIAS_RELU_BF16) {
          v += bias;
          reinterpret_cast<uint16_t*>(g.c)[off] = f2bf(v > 0.f ? v : 0.f);
        } else {   // HDET_EPI_MASK_BF16: gradient through the ReLU of the layer below
          const float act = bf2f(g.mask[(int64_t)z * g.mask_bs + (int64_t)row * g.mask_ld + col]);
          reinterpret_cast<uint16_t*>(g.c)[off] = f2bf(act > 0.f ? v : 0.f);
        }
      }
    }
}

hipError_t hdet_launch_bgemm(const hdet_bgemm_args& g, bool a_kmajor, bool b_kmajor, int epi, int batch,
                             hipStream_t s) {
  dim3 grid((g.n + TN - 1) / TN, (g.m + TM - 1) / TM, batch);
#define HDET_BGEMM(AK, BK, E) hipLaunchKernelGGL((hdet_bgemm_kernel<AK, BK, E>), grid, dim3(256), 0, s, g)
  if (a_kmajor && b_kmajor) {            // forward
    if (epi == HDET_EPI_BIAS_RELU_BF16) HDET_BGEMM(true, true, HDET_EPI_BIAS_RELU_BF16);
    else HDET_BGEMM(true, true, HDET_EPI_BIAS_F32);
  } else if (a_kmajor && !b_kmajor) {    // dgrad
    HDET_BGEMM(true, false, HDET_EPI_MASK_BF16);
  } else if (!a_kmajor && !b_kmajor) {   // wgrad
    HDET_BGEMM(false, false, HDET_EPI_F32);
  } else {
    return hipErrorInvalidValue;
  }
#undef HDET_BGEMM
  return hipGetLastError();
}

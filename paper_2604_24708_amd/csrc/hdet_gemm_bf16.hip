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
// Tiles are staged through LDS with 128-bit coalesced global loads and 128-bit LDS stores in
// the operand's own memory order, and read back as MFMA operands (8 consecutive contraction
// elements per lane):
//   * contraction-contiguous operand: LDS tile [128 rows][32 k], one ds_read_b128 per fragment;
//   * operand contiguous along the output axis: LDS tile [32 k][128 rows], read with the
//     transposing LDS load of gfx950 (ds_read_b64_tr_b16, two per fragment), so that no
//     transposed copy of weights or activations ever exists in HBM.
//
// Tiling: 128x128 output tile per 256-thread block (4 wavefronts, 2x2, 64x64 each as 2x2
// v_mfma_f32_32x32x16_bf16), K step 32, LDS double-buffered (one barrier per K step), global
// loads prefetched two K steps ahead through a ring of registers.

#include "hdet_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f16v __attribute__((ext_vector_type(16)));
typedef unsigned short us8 __attribute__((ext_vector_type(8)));
typedef short s4 __attribute__((ext_vector_type(4)));
typedef short s8 __attribute__((ext_vector_type(8)));

constexpr int TM = 128, TN = 128, TK = 32;
constexpr int LDK = TK;          // pitch of a [row][k] tile: 64 B, no padding; the four 16-byte chunks of a
                                 // row are stored XOR-swizzled by (row / 4) % 4, which makes both the
                                 // staging stores (4 rows x 4 chunks per 16 lanes) and the fragment
                                 // loads (16 rows x 1 chunk per 16 lanes) free of bank conflicts
constexpr int LDR = TM + 32;     // pitch of a [k][row] tile: 320 B = 80 banks, so the 4 k-rows that a
                                 // 16-lane group of a transposing read touches fall on disjoint banks
constexpr int TILE_ELEMS = 5120; // max(128 * LDK, 32 * LDR)
constexpr int PF = 2;            // K steps of global loads in flight (even)

__device__ __forceinline__ unsigned short f2bf(float x) {
  unsigned u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x0040u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (unsigned short)(u >> 16);
}
__device__ __forceinline__ float bf2f(unsigned short h) { return __uint_as_float((unsigned)h << 16); }

// 8 consecutive elements starting at src[idx], of which the first `valid` exist (others 0).
// FAST: the host has checked that every chunk is 16-byte aligned and either whole or absent
// (leading dimensions, extents along the chunk axis and replica strides multiples of 8), so the
// load is one branch-free 128-bit access -- an absent chunk reads src[0..7] and is zeroed.
template <bool FAST>
__device__ __forceinline__ us8 load8(const uint16_t* src, int64_t idx, int valid, bool vec_ok) {
  if (FAST) {
    const us8 v = *reinterpret_cast<const us8*>(src + (valid > 0 ? idx : 0));
    const us8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
    return valid > 0 ? v : zero;
  }
  if (valid >= 8 && vec_ok) return *reinterpret_cast<const us8*>(src + idx);
  us8 r = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
  for (int j = 0; j < 8; ++j)
    if (j < valid) r[j] = src[idx + j];
  return r;
}

// One operand tile: 128 rows of the output dimension x 32 of the contraction.
// KMAJOR: element (row, k) at src[row * ld + k], LDS tile[row][k];
// otherwise at src[k * ld + row], LDS tile[k][row].
template <bool KMAJOR, bool FAST>
struct operand {
  us8 reg[2];
  __device__ __forceinline__ void fetch(const uint16_t* src, int64_t ld, int row0, int rows, int k0, int kdim,
                                        bool vec_ok, int tid) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int c = tid + i * 256;
      if (KMAJOR) {
        const int row = row0 + (c >> 2), k = k0 + ((c & 3) << 3);
        reg[i] = load8<FAST>(src, (int64_t)row * ld + k, row < rows ? kdim - k : 0, vec_ok);
      } else {
        const int k = k0 + (c >> 4), row = row0 + ((c & 15) << 3);
        reg[i] = load8<FAST>(src, (int64_t)k * ld + row, k < kdim ? rows - row : 0, vec_ok);
      }
    }
  }
  __device__ __forceinline__ void commit(uint16_t* tile, int tid) const {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int c = tid + i * 256;
      if (KMAJOR) *reinterpret_cast<us8*>(tile + (c >> 2) * LDK + ((((c & 3) ^ (c >> 4)) & 3) << 3)) = reg[i];
      else *reinterpret_cast<us8*>(tile + (c >> 4) * LDR + ((c & 15) << 3)) = reg[i];
    }
  }
  // MFMA 32x32x16 operand fragment: lane l gets (row = r0 + l % 32, k = ks + 8 * (l / 32) + 0..7).
  static __device__ __forceinline__ bf16x8 fragment(const uint16_t* tile, int r0, int ks, int lane) {
    if (KMAJOR) {
      const int row = r0 + (lane & 31);
      const int chunk = ((ks >> 3) + (lane >> 5)) ^ ((row >> 2) & 3);
      return *reinterpret_cast<const bf16x8*>(tile + row * LDK + (chunk << 3));
    }
    // Transposing read: within a 16-lane group, lane p points at the 4 elements
    // (k = kb + p / 4, rows rb + 4 * (p % 4) .. + 3) and lane i receives (k = kb .. kb + 3, row rb + i).
    const int p = lane & 15;
    const int rb = r0 + (((lane >> 4) & 1) << 4);
    const int kb = ks + ((lane >> 5) << 3);
    const uint16_t* q = tile + (kb + (p >> 2)) * LDR + rb + ((p & 3) << 2);
    const s4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s4 __attribute__((address_space(3)))*)(q));
    const s4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s4 __attribute__((address_space(3)))*)(q + 4 * LDR));
    const s8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, both);
  }
};

}  // namespace

template <bool A_KMAJOR, bool B_KMAJOR, int EPI, bool FAST>
__global__ __launch_bounds__(256) void hdet_bgemm_kernel(const hdet_bgemm_args g) {
  __shared__ __attribute__((aligned(16))) uint16_t As[2][TILE_ELEMS];
  __shared__ __attribute__((aligned(16))) uint16_t Bs[2][TILE_ELEMS];
  const hdet_batch_index bi = hdet_split_batch(blockIdx.z, g.n1, g.n2);
  const int z = bi.z0;            // replica: bias and mask are per replica
  const uint16_t* A = g.a + hdet_batch_offset(bi, g.a_s);
  const uint16_t* B = g.b + hdet_batch_offset(bi, g.b_s);
  const int64_t c_base = hdet_batch_offset(bi, g.c_s);
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

  // Ring of PF register stages: the global loads of K step kt + PF are issued while step kt
  // is computed, so that about PF x 16 KB per block is in flight -- one step's MFMAs (about
  // 0.1 us) are far shorter than an HBM round trip.
  operand<A_KMAJOR, FAST> oa[PF];
  operand<B_KMAJOR, FAST> ob[PF];
  // The loop body is free of conditions: K steps past the end of the contraction load zeros
  // (absent chunks) and multiply them, so the count is simply rounded up to a multiple of PF.
  const int nk = ((g.k + TK - 1) / TK + PF - 1) / PF * PF;
#pragma unroll
  for (int d = 0; d < PF; ++d) {
    oa[d].fetch(A, g.lda, m0, g.m, d * TK, g.k, a_vec, tid);
    ob[d].fetch(B, g.ldb, n0, g.n, d * TK, g.k, b_vec, tid);
  }
  oa[0].commit(As[0], tid);
  ob[0].commit(Bs[0], tid);
  __syncthreads();
  oa[0].fetch(A, g.lda, m0, g.m, PF * TK, g.k, a_vec, tid);
  ob[0].fetch(B, g.ldb, n0, g.n, PF * TK, g.k, b_vec, tid);
  for (int kt0 = 0; kt0 < nk; kt0 += PF) {
#pragma unroll
    for (int d = 0; d < PF; ++d) {
      const int buf = d & 1;                 // PF is even, so (kt0 + d) & 1 == d & 1
#pragma unroll
      for (int ks = 0; ks < TK; ks += 16) {
        bf16x8 af[2], bfr[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          af[i] = operand<A_KMAJOR, FAST>::fragment(As[buf], wm + i * 32, ks, lane);
          bfr[i] = operand<B_KMAJOR, FAST>::fragment(Bs[buf], wn + i * 32, ks, lane);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
      }
      // stage tile kt0 + d + 1 into the other LDS buffer (last read before the previous
      // barrier) and refill its ring slot with tile kt0 + d + 1 + PF
      const int r = (d + 1) % PF;
      oa[r].commit(As[buf ^ 1], tid);
      ob[r].commit(Bs[buf ^ 1], tid);
      oa[r].fetch(A, g.lda, m0, g.m, (kt0 + d + 1 + PF) * TK, g.k, a_vec, tid);
      ob[r].fetch(B, g.ldb, n0, g.n, (kt0 + d + 1 + PF) * TK, g.k, b_vec, tid);
      __syncthreads();
    }
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
      if (EPI == HDET_EPI_BIAS_RELU_BF16 || EPI == HDET_EPI_BIAS_F32 || EPI == HDET_EPI_BIAS_BF16)
        bias = g.bias[(int64_t)z * g.bias_bs + col];
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int row = m0 + wm + i * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
        if (row >= g.m) continue;
        float v = acc[i][j][e];
        const int64_t off = c_base + (int64_t)row * g.ldc + col;
        if (EPI == HDET_EPI_F32) {
          reinterpret_cast<float*>(g.c)[off] = v;
        } else if (EPI == HDET_EPI_BIAS_F32) {
          reinterpret_cast<float*>(g.c)[off] = v + bias;
        } else if (EPI == HDET_EPI_BF16) {
          reinterpret_cast<uint16_t*>(g.c)[off] = f2bf(v);
        } else if (EPI == HDET_EPI_BIAS_BF16) {
          reinterpret_cast<uint16_t*>(g.c)[off] = f2bf(v + bias);
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

static bool chunk_regular(const void* base, int64_t ld, const int64_t* bs, int chunk_extent) {
  return (ld & 7) == 0 && ((bs[0] | bs[1] | bs[2]) & 7) == 0 && (chunk_extent & 7) == 0 &&
         (reinterpret_cast<uintptr_t>(base) & 15) == 0;
}

hipError_t hdet_launch_bgemm(const hdet_bgemm_args& g_in, bool a_kmajor, bool b_kmajor, int epi, int batch,
                             hipStream_t s) {
  hdet_bgemm_args g = g_in;
  if (g.n1 < 1) g.n1 = 1;
  if (g.n2 < 1) g.n2 = 1;
  dim3 grid((g.n + TN - 1) / TN, (g.m + TM - 1) / TM, batch);
  // a chunk is 8 elements along the operand's contiguous axis: k if k-major, else the row axis
  const bool fast = chunk_regular(g.a, g.lda, g.a_s, a_kmajor ? g.k : g.m) &&
                    chunk_regular(g.b, g.ldb, g.b_s, b_kmajor ? g.k : g.n);
#define HDET_BGEMM(AK, BK, E)                                                                          \
  do {                                                                                                 \
    if (fast) hipLaunchKernelGGL((hdet_bgemm_kernel<AK, BK, E, true>), grid, dim3(256), 0, s, g);      \
    else hipLaunchKernelGGL((hdet_bgemm_kernel<AK, BK, E, false>), grid, dim3(256), 0, s, g);          \
  } while (0)
#define HDET_BGEMM_EPI(AK, BK)                                                                         \
  switch (epi) {                                                                                       \
    case HDET_EPI_F32: HDET_BGEMM(AK, BK, HDET_EPI_F32); break;                                        \
    case HDET_EPI_BIAS_F32: HDET_BGEMM(AK, BK, HDET_EPI_BIAS_F32); break;                              \
    case HDET_EPI_BIAS_RELU_BF16: HDET_BGEMM(AK, BK, HDET_EPI_BIAS_RELU_BF16); break;                  \
    case HDET_EPI_MASK_BF16: HDET_BGEMM(AK, BK, HDET_EPI_MASK_BF16); break;                            \
    case HDET_EPI_BF16: HDET_BGEMM(AK, BK, HDET_EPI_BF16); break;                                      \
    case HDET_EPI_BIAS_BF16: HDET_BGEMM(AK, BK, HDET_EPI_BIAS_BF16); break;                            \
    default: return hipErrorInvalidValue;                                                              \
  }
  if (a_kmajor && b_kmajor) { HDET_BGEMM_EPI(true, true) }            // forward
  else if (a_kmajor && !b_kmajor) { HDET_BGEMM_EPI(true, false) }     // dgrad
  else if (!a_kmajor && !b_kmajor) { HDET_BGEMM_EPI(false, false) }   // wgrad
  else return hipErrorInvalidValue;
#undef HDET_BGEMM_EPI
#undef HDET_BGEMM
  return hipGetLastError();
}

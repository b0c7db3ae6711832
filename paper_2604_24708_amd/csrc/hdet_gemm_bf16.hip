// Replica-batched bf16 GEMM on the gfx950 matrix cores for the "Forward + backward" of
// Algorithm 1 in mixed precision: bf16 operands, fp32 accumulation, N independent weight
// sets with the replica on blockIdx.z.  This file holds the entry point and the general
// kernel, which takes any shape, leading dimension and alignment; products whose operands are
// made of whole, aligned 16-byte chunks are routed to the LDS-direct kernel
// (hdet_gemm_bf16_dma.hip).
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
// Tiling: each wavefront owns a 64x64 output tile (2x2 blocks of v_mfma_f32_32x32x16_bf16); a
// block is 2x2 wavefronts (128x128 tile).  K step 32, LDS double-buffered (one barrier per K
// step), the next step's global loads in flight during the MFMAs; launch indices are remapped so
// that each XCD's L2 serves a contiguous range of tiles.

#include "hdet_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f16v __attribute__((ext_vector_type(16)));
typedef unsigned short us8 __attribute__((ext_vector_type(8)));
typedef short s4 __attribute__((ext_vector_type(4)));
typedef short s8 __attribute__((ext_vector_type(8)));

constexpr int TK = 32;
constexpr int LDK = TK;          // pitch of a [row][k] tile: 64 B, no padding; the four 16-byte chunks of a
                                 // row are stored XOR-swizzled by (row / 4) % 4, which makes both the
                                 // staging stores (4 rows x 4 chunks per 16 lanes) and the fragment
                                 // loads (16 rows x 1 chunk per 16 lanes) free of bank conflicts
// pitch of a [k][row] tile of ROWS rows: ROWS + 32 elements, i.e. 16 banks past a multiple of 64, so
// the 4 k-rows that a 16-lane group of a transposing read touches fall on disjoint banks
__host__ __device__ constexpr int ldr(int rows) { return rows + 32; }
__host__ __device__ constexpr int tile_elems(int rows) { return TK * ldr(rows); }   // >= rows * LDK

__device__ __forceinline__ unsigned short f2bf(float x) {
  unsigned u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x0040u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (unsigned short)(u >> 16);
}
__device__ __forceinline__ float bf2f(unsigned short h) { return __uint_as_float((unsigned)h << 16); }

// 8 consecutive elements starting at src[idx], of which the first `valid` exist (others 0);
// one 128-bit access when the chunk is whole and 16-byte aligned
__device__ __forceinline__ us8 load8(const uint16_t* src, int64_t idx, int valid, bool vec_ok) {
  if (valid >= 8 && vec_ok) return *reinterpret_cast<const us8*>(src + idx);
  us8 r = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
  for (int j = 0; j < 8; ++j)
    if (j < valid) r[j] = src[idx + j];
  return r;
}

// One operand tile: ROWS (128 or 256) rows of the output dimension x 32 of the contraction.
// KMAJOR: element (row, k) at src[row * ld + k], LDS tile[row][k];
// otherwise at src[k * ld + row], LDS tile[k][row].
template <bool KMAJOR, int ROWS, int THREADS>
struct operand {
  static constexpr int NCH = ROWS * 4 / THREADS;   // 8-element chunks per thread and K step
  static constexpr int RCH = ROWS / 8;         // chunks per k-row of a [k][row] tile
  us8 reg[NCH];
  __device__ __forceinline__ void fetch(const uint16_t* src, int64_t ld, int row0, int rows, int k0, int kdim,
                                        bool vec_ok, int tid) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = tid + i * THREADS;
      int valid;
      if (KMAJOR) {
        const int row = row0 + (c >> 2), k = k0 + ((c & 3) << 3);
        valid = row < rows ? kdim - k : 0;
        reg[i] = load8(src, (int64_t)row * ld + k, valid, vec_ok);
      } else {
        const int k = k0 + c / RCH, row = row0 + ((c % RCH) << 3);
        valid = k < kdim ? rows - row : 0;
        reg[i] = load8(src, (int64_t)k * ld + row, valid, vec_ok);
      }
    }
  }
  __device__ __forceinline__ void commit(uint16_t* tile, int tid) const {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = tid + i * THREADS;
      const us8 v = reg[i];
      if (KMAJOR) *reinterpret_cast<us8*>(tile + (c >> 2) * LDK + ((((c & 3) ^ (c >> 4)) & 3) << 3)) = v;
      else *reinterpret_cast<us8*>(tile + (c / RCH) * ldr(ROWS) + ((c % RCH) << 3)) = v;
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
    const uint16_t* q = tile + (kb + (p >> 2)) * ldr(ROWS) + rb + ((p & 3) << 2);
    const s4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s4 __attribute__((address_space(3)))*)(q));
    const s4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s4 __attribute__((address_space(3)))*)(q + 4 * ldr(ROWS)));
    const s8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, both);
  }
};

}  // namespace

// WMT x WNT: 32x32 MFMA blocks per wavefront in m and n; WGM x 2 wavefronts per block
// (WGM = 2: 256 threads, WGM = 4: 512 threads), block tile (32 WMT WGM) x (64 WNT).
template <bool A_KMAJOR, bool B_KMAJOR, int EPI, int WMT, int WNT, int WGM>
__global__ __launch_bounds__(128 * WGM, WGM) void hdet_bgemm_kernel(const hdet_bgemm_args g) {
  constexpr int TM = 32 * WMT * WGM, TN = 64 * WNT, THREADS = 128 * WGM;
  __shared__ __attribute__((aligned(16))) uint16_t As[2][tile_elems(TM)];
  __shared__ __attribute__((aligned(16))) uint16_t Bs[2][tile_elems(TN)];
  // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2) in launch order.
  // Remap the launch index so that an XCD works on a contiguous range of tiles: the tiles that
  // share an A row-panel or a weight panel then meet in one L2 instead of eight.
  int bx = blockIdx.x, by = blockIdx.y, bz = blockIdx.z;
  {
    const unsigned total = gridDim.x * gridDim.y * gridDim.z;
    if ((total & 7u) == 0u) {
      const unsigned lin = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
      const unsigned t = (lin & 7u) * (total >> 3) + (lin >> 3);
      bx = t % gridDim.x;
      by = (t / gridDim.x) % gridDim.y;
      bz = t / (gridDim.x * gridDim.y);
    }
  }
  const hdet_batch_index bi = hdet_split_batch(bz, g.n1, g.n2);
  const int z = bi.z0;            // replica: bias and mask are per replica
  const uint16_t* A = g.a + hdet_batch_offset(bi, g.a_s);
  const uint16_t* B = g.b + hdet_batch_offset(bi, g.b_s);
  const int64_t c_base = hdet_batch_offset(bi, g.c_s);
  const int m0 = by * TM, n0 = bx * TN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = (wave >> 1) * (32 * WMT), wn = (wave & 1) * (32 * WNT);
  const bool a_vec = (g.lda & 7) == 0 && (reinterpret_cast<uintptr_t>(A) & 15) == 0;
  const bool b_vec = (g.ldb & 7) == 0 && (reinterpret_cast<uintptr_t>(B) & 15) == 0;

  f16v acc[WMT][WNT];
#pragma unroll
  for (int i = 0; i < WMT; ++i)
#pragma unroll
    for (int j = 0; j < WNT; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // One register stage: the global loads of K step kt + 1 are issued before the MFMAs of step
  // kt and written to the other LDS buffer after them (one barrier per step); other blocks
  // on the same CU cover the rest of the memory latency.  The step past the end loads nothing
  // (all chunks absent) and its zeros are never used.
  operand<A_KMAJOR, TM, THREADS> oa;
  operand<B_KMAJOR, TN, THREADS> ob;
  const int nk = (g.k + TK - 1) / TK;
  oa.fetch(A, g.lda, m0, g.m, 0, g.k, a_vec, tid);
  ob.fetch(B, g.ldb, n0, g.n, 0, g.k, b_vec, tid);
  oa.commit(As[0], tid);
  ob.commit(Bs[0], tid);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    oa.fetch(A, g.lda, m0, g.m, (kt + 1) * TK, g.k, a_vec, tid);
    ob.fetch(B, g.ldb, n0, g.n, (kt + 1) * TK, g.k, b_vec, tid);
    __builtin_amdgcn_sched_barrier(0);     // keep the loads ahead of the MFMAs ...
#pragma unroll
    for (int ks = 0; ks < TK; ks += 16) {
      bf16x8 af[WMT], bfr[WNT];
#pragma unroll
      for (int i = 0; i < WMT; ++i) af[i] = operand<A_KMAJOR, TM, THREADS>::fragment(As[buf], wm + i * 32, ks, lane);
#pragma unroll
      for (int j = 0; j < WNT; ++j) bfr[j] = operand<B_KMAJOR, TN, THREADS>::fragment(Bs[buf], wn + j * 32, ks, lane);
#pragma unroll
      for (int i = 0; i < WMT; ++i)
#pragma unroll
        for (int j = 0; j < WNT; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);     // ... and every use of the loaded data behind them
    oa.commit(As[buf ^ 1], tid);      // last read before the previous barrier
    ob.commit(Bs[buf ^ 1], tid);
    __syncthreads();
  }

  // epilogue: accumulator element e of lane l is C(row, col) with
  //   row = (e / 4) * 8 + (l / 32) * 4 + e % 4,  col = l % 32   inside its 32x32 block
#pragma unroll
  for (int i = 0; i < WMT; ++i)
#pragma unroll
    for (int j = 0; j < WNT; ++j) {
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

hipError_t hdet_launch_bgemm(const hdet_bgemm_args& g_in, bool a_kmajor, bool b_kmajor, int epi, int batch,
                             hipStream_t s) {
  hdet_bgemm_args g = g_in;
  if (g.n1 < 1) g.n1 = 1;
  if (g.n2 < 1) g.n2 = 1;
  if (hdet_bgemm_dma_eligible(g, a_kmajor, b_kmajor, epi)) return hdet_launch_bgemm_dma(g, a_kmajor, b_kmajor, epi, batch, s);
  dim3 grid((g.n + 127) / 128, (g.m + 127) / 128, batch);
#define HDET_BGEMM(AK, BK, E) hipLaunchKernelGGL((hdet_bgemm_kernel<AK, BK, E, 2, 2, 2>), grid, dim3(256), 0, s, g)
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

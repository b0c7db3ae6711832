// Causal self-attention of the transformer replicas in mixed precision, forward and backward,
// with the scores kept on chip ("Forward + backward" of Algorithm 1 for the attention part of a
// block).  For head size 64 and sequence lengths that are multiples of 64 up to 512 this
// replaces five batched GEMMs, two softmax kernels and the [S][S] score and probability tensors
// in HBM by three kernels that read q, k, v (and the output gradient) once per 64-row block.
//
// Arithmetic follows the unfused path operation by operation, so both agree to the rounding
// of the bf16 tensors they share:
//   forward   s = (q k^T) * scale (fp32), causal mask, p = bf16(exp(s - max) / sum), a = bf16(p v)
//   backward  dp = da v^T, dot = sum_j dp_j p_j, ds = bf16(p (dp - dot) scale),
//             dq = bf16(ds k), dk = bf16(ds^T q), dv = bf16(p^T da)
// with scale = 1 / (sqrt(d_head) tau_r), tau_r the replica's attention temperature when that is
// an explored channel (Remark 1).  The row maximum and 1/sum of the forward are kept ([rows]
// fp32 each) so that the backward rebuilds p without a reduction.
//
// Layout: qkv [N][B][S][3d] bf16 (q | k | v, head h in columns h*64..), a and da [N][B][S][d],
// dqkv like qkv.  A block is 4 wavefronts; tiles are v_mfma_f32_32x32x16_bf16 blocks fed from
// LDS tiles of pitch 72 (or S + 8) elements, which keeps the 128-bit fragment reads free of bank
// conflicts; operands that are contracted along their row index are read with the transposing
// LDS load, so nothing is transposed in memory.
//   forward  : block = (64 queries, sequence, head, replica); wavefront w owns key block w
//              (4 wavefronts for S <= 256, 8 beyond)
//   backward : 1. same mapping: rebuilds p, forms dp, the row dots (kept for step 2), ds and dq
//                 (q and da fragments go from global memory straight to registers)
//              2. block = (64 keys, sequence, head, replica), loop over the query blocks at or
//                 below the diagonal: dk, dv accumulate in registers in ascending query order
// Every sum has a fixed order: results do not depend on scheduling.

#include "hdet_internal.h"
#include "hdet_elem.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f16v __attribute__((ext_vector_type(16)));
typedef short s4 __attribute__((ext_vector_type(4)));
typedef short s8 __attribute__((ext_vector_type(8)));
typedef unsigned short us8 __attribute__((ext_vector_type(8)));

constexpr int DH = 64;            // head size
constexpr int QB = 64;            // rows per block
constexpr int PT = DH + 8;        // pitch of a [rows][64] tile
constexpr int SMAX = 512;         // longest sequence: one key block of 64 per wavefront, at most 8 wavefronts

__device__ __forceinline__ unsigned short f2bf(float x) { return __builtin_bit_cast(unsigned short, (__bf16)x); }
__device__ __forceinline__ float bf2f(unsigned short h) { return __uint_as_float((unsigned)h << 16); }
__device__ __forceinline__ float bf16_round(float x) { return bf2f(f2bf(x)); }

// MFMA 32x32x16 operand fragment of lane l: (row = r0 + l % 32, k = ks + 8 * (l / 32) + 0..7).
// Tile stored [row][k] with `pitch` elements per row (pitch a multiple of 8).
__device__ __forceinline__ bf16x8 frag_k(const uint16_t* t, int pitch, int r0, int ks, int lane) {
  return *reinterpret_cast<const bf16x8*>(t + (r0 + (lane & 31)) * pitch + ks + ((lane >> 5) << 3));
}
// The same fragment from a tile stored [k][row] (contracted along the tile's row index): within a
// 16-lane group, lane p points at the 4 elements (k = kb + p / 4, rows rb + 4 * (p % 4) .. + 3) and lane i
// receives (k = kb .. kb + 3, row rb + i) from the transposing read.
__device__ __forceinline__ bf16x8 frag_t(const uint16_t* t, int pitch, int r0, int ks, int lane) {
  const int p = lane & 15;
  const int row = r0 + (((lane >> 4) & 1) << 4) + ((p & 3) << 2);
  const int k = ks + ((lane >> 5) << 3) + (p >> 2);
  const uint16_t* q = t + k * pitch + row;
  const s4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s4 __attribute__((address_space(3)))*)(q));
  const s4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s4 __attribute__((address_space(3)))*)(q + 4 * pitch));
  const s8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, both);
}
__device__ __forceinline__ f16v mfma(bf16x8 a, bf16x8 b, f16v c) { return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0); }
__device__ __forceinline__ f16v zero16() {
  f16v z;
#pragma unroll
  for (int e = 0; e < 16; ++e) z[e] = 0.f;
  return z;
}
// accumulator element e of lane l sits at (row = (e / 4) * 8 + (l / 32) * 4 + e % 4, col = l % 32) of its 32x32 block
__device__ __forceinline__ int acc_row(int e, int lane) { return ((e >> 2) << 3) + ((lane >> 5) << 2) + (e & 3); }

// rows x 64 bf16 from global (row pitch `ld` elements) into an LDS tile of pitch PT by THREADS threads,
// in two phases so that all loads of a block are in flight together: fetch() issues up to NC
// 16-byte loads per thread, commit() writes them to LDS.
template <int NC, int THREADS = 256>
struct tile_loader {
  us8 v[NC];
  __device__ __forceinline__ void fetch(const uint16_t* src, int64_t ld, int rows, int tid) {
#pragma unroll
    for (int i = 0; i < NC; ++i) {
      const int c = tid + i * THREADS;
      if (c < rows * 8) v[i] = *reinterpret_cast<const us8*>(src + (int64_t)(c >> 3) * ld + ((c & 7) << 3));
    }
  }
  __device__ __forceinline__ void commit(uint16_t* dst, int rows, int tid) const {
#pragma unroll
    for (int i = 0; i < NC; ++i) {
      const int c = tid + i * THREADS;
      if (c < rows * 8) *reinterpret_cast<us8*>(dst + (c >> 3) * PT + ((c & 7) << 3)) = v[i];
    }
  }
};
constexpr int NCQ = QB * 8 / 256;        // chunks per thread of a 64-row tile (256 threads)
constexpr int NCK = 8;                   // ... of all keys / values of a sequence (64 rows per wavefront)
struct attn_args {
  const uint16_t* qkv;      // [N][B][S][3d]
  uint16_t* a;              // forward: [N][B][S][d] output
  const uint16_t* da;       // backward: gradient at a
  uint16_t* dqkv;           // backward: [N][B][S][3d]
  float* row_max;           // [N][B][heads][S]
  float* row_inv;
  float* row_dot;
  const hdet_ctrl* ctrl;
  int temp_channel;
  float scale;              // 1 / sqrt(d_head)
  int B, S, heads, d;
};

__device__ __forceinline__ float replica_scale(const attn_args& g, int r) {
  return g.temp_channel >= 0 ? g.scale / (float)hdet_channel_value(g.ctrl, g.temp_channel, r, 0.0) : g.scale;
}

// 64 x 64 scores of (query block in A, key block in B): 2 x 2 accumulator blocks, contraction 64
__device__ __forceinline__ void qk_tile(f16v (&acc)[2][2], const uint16_t* rows_a, const uint16_t* rows_b, int lane) {
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = zero16();
#pragma unroll
  for (int ks = 0; ks < DH; ks += 16) {
    bf16x8 fa[2], fb[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) fa[i] = frag_k(rows_a, PT, i * 32, ks, lane);
#pragma unroll
    for (int j = 0; j < 2; ++j) fb[j] = frag_k(rows_b, PT, j * 32, ks, lane);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) acc[i][j] = mfma(fa[i], fb[j], acc[i][j]);
  }
}

// Score tiles are formed transposed, keys x queries: a lane then holds ONE query (column l % 32 of
// the accumulator block) and 16 keys of it per block, in runs of 4 consecutive keys.  Row
// statistics of a query are in-lane reductions plus one exchange between the two half-wavefronts,
// and the probabilities go to LDS 4 keys (8 bytes) at a time.
// local key index of accumulator element e in key block i: i * 32 + acc_row(e, lane); query: j * 32 + lane % 32
typedef unsigned short us4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float other_half(float x) { return __shfl_xor(x, 32); }
// exp on the hardware exp2 (relative error about 1e-7); forward and backward use the same one, so
// the backward rebuilds exactly the probabilities of the forward
__device__ __forceinline__ float exp_fast(float x) { return __expf(x); }

// ---------------------------------------------------------------------------------------------
// forward
// ---------------------------------------------------------------------------------------------
// NW wavefronts: sequences of up to 64 NW keys (4: two blocks per CU; 8: one)
template <int NW>
__global__ __launch_bounds__(64 * NW, 2) void attn_fwd_kernel(const attn_args g) {
  constexpr int PP = 64 * NW + 8;                                        // pitch of the [64][S] tile
  __shared__ __attribute__((aligned(16))) uint16_t Qs[QB * PT];
  __shared__ __attribute__((aligned(16))) uint16_t KVs[64 * NW * PT];   // keys, then values
  __shared__ __attribute__((aligned(16))) uint16_t Ps[QB * PP];
  __shared__ float red[NW][QB];
  __shared__ float stat[2][QB];                                          // row max, 1 / row sum
  const int qb = blockIdx.x, bh = blockIdx.y, r = blockIdx.z;
  const int b = bh / g.heads, h = bh - b * g.heads;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int kmax = (qb + 1) * QB;
  const int64_t ld = 3 * (int64_t)g.d;
  const uint16_t* base = g.qkv + (((int64_t)r * g.B + b) * g.S) * ld + h * DH;
  const float scale = replica_scale(g, r);

  tile_loader<QB * 8 / (64 * NW), 64 * NW> lq;
  tile_loader<NCK, 64 * NW> lk, lv;
  lq.fetch(base + (int64_t)qb * QB * ld, ld, QB, tid);
  lk.fetch(base + g.d, ld, kmax, tid);
  lv.fetch(base + 2 * g.d, ld, kmax, tid);          // consumed after the softmax
  lq.commit(Qs, QB, tid);
  lk.commit(KVs, kmax, tid);
  __syncthreads();

  // wavefront w: scores of key block w (if it is at or below the diagonal), [key][query]
  const bool active = w <= qb;
  f16v sc[2][2];
  if (active) qk_tile(sc, KVs + w * QB * PT, Qs, lane);
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int q = j * 32 + (lane & 31);
    float m = -INFINITY;
    if (active) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int key = i * 32 + acc_row(e, lane);
          const bool keep = w < qb || key <= q;                          // causal: key <= query
          sc[i][j][e] = keep ? sc[i][j][e] * scale : -INFINITY;
          m = fmaxf(m, sc[i][j][e]);
        }
    }
    m = fmaxf(m, other_half(m));
    if (lane < 32) red[w][q] = m;
  }
  __syncthreads();
  if (tid < QB) {
    float m = red[0][tid];
#pragma unroll
    for (int x = 1; x < NW; ++x) m = fmaxf(m, red[x][tid]);
    stat[0][tid] = m;
  }
  __syncthreads();
  // exponentials and row sums
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int q = j * 32 + (lane & 31);
    const float mx = stat[0][q];
    float sum = 0.f;
    if (active) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) { sc[i][j][e] = exp_fast(sc[i][j][e] - mx); sum += sc[i][j][e]; }
    }
    sum += other_half(sum);
    if (lane < 32) red[w][q] = sum;
  }
  __syncthreads();
  if (tid < QB) {
    float sum = red[0][tid];
#pragma unroll
    for (int x = 1; x < NW; ++x) sum += red[x][tid];
    const float inv = 1.f / sum;
    stat[1][tid] = inv;
    const int64_t gr = (((int64_t)r * g.B + b) * g.heads + h) * g.S + qb * QB + tid;
    g.row_max[gr] = stat[0][tid];
    g.row_inv[gr] = inv;
  }
  __syncthreads();
  // probabilities as the second product reads them: bf16 [query][key]
  if (active) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int q = j * 32 + (lane & 31);
      const float inv = stat[1][q];
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
          const us4 o = {f2bf(sc[i][j][4 * e4] * inv), f2bf(sc[i][j][4 * e4 + 1] * inv), f2bf(sc[i][j][4 * e4 + 2] * inv),
                         f2bf(sc[i][j][4 * e4 + 3] * inv)};
          *reinterpret_cast<us4*>(Ps + q * PP + w * QB + i * 32 + acc_row(4 * e4, lane)) = o;
        }
    }
  }
  __syncthreads();                       // all reads of the keys are done as well
  lv.commit(KVs, kmax, tid);
  __syncthreads();
  // a = p v: wavefront w < 4 owns the 32 x 32 block (w / 2, w % 2) of the 64 x 64 output
  if (w >= 4) return;
  const int r0 = (w >> 1) * 32, c0 = (w & 1) * 32;
  f16v out = zero16();
  for (int ks = 0; ks < kmax; ks += 16) out = mfma(frag_k(Ps, PP, r0, ks, lane), frag_t(KVs, PT, c0, ks, lane), out);
  uint16_t* dst = g.a + (((int64_t)r * g.B + b) * g.S + qb * QB) * g.d + h * DH;
#pragma unroll
  for (int e = 0; e < 16; ++e) dst[(int64_t)(r0 + acc_row(e, lane)) * g.d + c0 + (lane & 31)] = f2bf(out[e]);
}

// The probability as the unfused path stores it (bf16), rebuilt from the scaled score and the
// row statistics of the forward.
__device__ __forceinline__ float prob(float s, float mx, float inv) { return bf16_round(exp_fast(s - mx) * inv); }

// ---------------------------------------------------------------------------------------------
// backward, step 1: dq and the row dots
// ---------------------------------------------------------------------------------------------
template <int NW>
__global__ __launch_bounds__(64 * NW, 2) void attn_bwd_dq_kernel(const attn_args g) {
  constexpr int PP = 64 * NW + 8;
  __shared__ __attribute__((aligned(16))) uint16_t Ks[64 * NW * PT];
  __shared__ __attribute__((aligned(16))) uint16_t Vs[64 * NW * PT];    // values, then ds [query][key] with pitch PP
  __shared__ float red[NW][QB];
  __shared__ float stat[3][QB];                                          // row max, 1 / row sum, row dot
  static_assert(QB * PP <= 64 * NW * PT, "ds must fit into the value tile");
  uint16_t* dSs = Vs;
  const int qb = blockIdx.x, bh = blockIdx.y, r = blockIdx.z;
  const int b = bh / g.heads, h = bh - b * g.heads;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int kmax = (qb + 1) * QB;
  const int64_t ld = 3 * (int64_t)g.d;
  const int64_t tok0 = ((int64_t)r * g.B + b) * g.S;
  const uint16_t* base = g.qkv + tok0 * ld + h * DH;
  const int64_t gr0 = (((int64_t)r * g.B + b) * g.heads + h) * g.S + qb * QB;
  const float scale = replica_scale(g, r);

  // The 64 queries and their output gradients are operands of every wavefront's two products and
  // of nothing else: each wavefront takes its fragments straight from global memory into
  // registers, which leaves the LDS to the keys and values (two 4-wavefront blocks per CU).
  bf16x8 fq[2][4], fda[2][4];
  {
    tile_loader<NCK, 64 * NW> lk, lv;
    lk.fetch(base + g.d, ld, kmax, tid);
    lv.fetch(base + 2 * g.d, ld, kmax, tid);
    const uint16_t* qsrc = base + (int64_t)qb * QB * ld;
    const uint16_t* dasrc = g.da + (tok0 + qb * QB) * g.d + h * DH;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int k4 = 0; k4 < 4; ++k4) {
        const int row = j * 32 + (lane & 31), col = k4 * 16 + ((lane >> 5) << 3);
        fq[j][k4] = *reinterpret_cast<const bf16x8*>(qsrc + (int64_t)row * ld + col);
        fda[j][k4] = *reinterpret_cast<const bf16x8*>(dasrc + (int64_t)row * g.d + col);
      }
    if (tid < QB) { stat[0][tid] = g.row_max[gr0 + tid]; stat[1][tid] = g.row_inv[gr0 + tid]; }
    lk.commit(Ks, kmax, tid);
    lv.commit(Vs, kmax, tid);
  }
  __syncthreads();

  // p and dp = da v^T of key block w, both [key][query]
  const bool active = w <= qb;
  f16v p[2][2], dp[2][2];
  if (active) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) { p[i][j] = zero16(); dp[i][j] = zero16(); }
#pragma unroll
    for (int k4 = 0; k4 < 4; ++k4) {
      bf16x8 fk[2], fv[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        fk[i] = frag_k(Ks + w * QB * PT, PT, i * 32, k4 * 16, lane);
        fv[i] = frag_k(Vs + w * QB * PT, PT, i * 32, k4 * 16, lane);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          p[i][j] = mfma(fk[i], fq[j][k4], p[i][j]);
          dp[i][j] = mfma(fv[i], fda[j][k4], dp[i][j]);
        }
    }
  }
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int q = j * 32 + (lane & 31);
    const float mx = stat[0][q], inv = stat[1][q];
    float sum = 0.f;
    if (active) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int key = i * 32 + acc_row(e, lane);
          const bool keep = w < qb || key <= q;
          p[i][j][e] = keep ? prob(p[i][j][e] * scale, mx, inv) : 0.f;
          sum += dp[i][j][e] * p[i][j][e];
        }
    }
    sum += other_half(sum);
    if (lane < 32) red[w][q] = sum;
  }
  __syncthreads();                       // also: every wavefront is done with the values
  if (tid < QB) {
    float dot = red[0][tid];
#pragma unroll
    for (int x = 1; x < NW; ++x) dot += red[x][tid];
    stat[2][tid] = dot;
    g.row_dot[gr0 + tid] = dot;
  }
  __syncthreads();
  if (active) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int q = j * 32 + (lane & 31);
      const float dot = stat[2][q];
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
          us4 o;
#pragma unroll
          for (int u = 0; u < 4; ++u) o[u] = f2bf(p[i][j][4 * e4 + u] * (dp[i][j][4 * e4 + u] - dot) * scale);
          *reinterpret_cast<us4*>(dSs + q * PP + w * QB + i * 32 + acc_row(4 * e4, lane)) = o;
        }
    }
  }
  __syncthreads();
  // dq = ds k: wavefront w < 4 owns the 32 x 32 block (w / 2, w % 2); keys are the contraction
  if (w >= 4) return;
  const int r0 = (w >> 1) * 32, c0 = (w & 1) * 32;
  f16v out = zero16();
  for (int ks = 0; ks < kmax; ks += 16) out = mfma(frag_k(dSs, PP, r0, ks, lane), frag_t(Ks, PT, c0, ks, lane), out);
  uint16_t* dst = g.dqkv + (tok0 + qb * QB) * ld + h * DH;
#pragma unroll
  for (int e = 0; e < 16; ++e) dst[(int64_t)(r0 + acc_row(e, lane)) * ld + c0 + (lane & 31)] = f2bf(out[e]);
}

// ---------------------------------------------------------------------------------------------
// backward, step 2: dk and dv of one key block
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256, 2) void attn_bwd_dkv_kernel(const attn_args g) {
  __shared__ __attribute__((aligned(16))) uint16_t Ks[QB * PT];
  __shared__ __attribute__((aligned(16))) uint16_t Vs[QB * PT];
  __shared__ __attribute__((aligned(16))) uint16_t Qs[QB * PT];
  __shared__ __attribute__((aligned(16))) uint16_t dAs[QB * PT];
  __shared__ __attribute__((aligned(16))) uint16_t Ps[QB * PT];          // [query][key]
  __shared__ __attribute__((aligned(16))) uint16_t dSs[QB * PT];
  __shared__ float stat[3][QB];
  const int kb = blockIdx.x, bh = blockIdx.y, r = blockIdx.z;
  const int b = bh / g.heads, h = bh - b * g.heads;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int nqb = g.S / QB;
  const int64_t ld = 3 * (int64_t)g.d;
  const int64_t tok0 = ((int64_t)r * g.B + b) * g.S;
  const uint16_t* base = g.qkv + tok0 * ld + h * DH;
  const int64_t gr0 = (((int64_t)r * g.B + b) * g.heads + h) * g.S;
  const float scale = replica_scale(g, r);

  tile_loader<NCQ> lq, la;
  {
    tile_loader<NCQ> lk, lv;
    lk.fetch(base + g.d + (int64_t)kb * QB * ld, ld, QB, tid);
    lv.fetch(base + 2 * g.d + (int64_t)kb * QB * ld, ld, QB, tid);
    lq.fetch(base + (int64_t)kb * QB * ld, ld, QB, tid);
    la.fetch(g.da + (tok0 + kb * QB) * g.d + h * DH, g.d, QB, tid);
    lk.commit(Ks, QB, tid);
    lv.commit(Vs, QB, tid);
  }
  // the wavefront's 32 x 32 block of every 64 x 64 tile: keys k0.. x queries q0.. of p and ds,
  // keys k0.. x columns q0.. of dk and dv
  const int k0 = (w >> 1) * 32, q0 = (w & 1) * 32;
  f16v dk = zero16(), dv = zero16();
  for (int qb = kb; qb < nqb; ++qb) {
    __syncthreads();                                     // the previous round's tiles are no longer read
    lq.commit(Qs, QB, tid);                              // fetched one round ahead
    la.commit(dAs, QB, tid);
    if (tid < QB) {
      stat[0][tid] = g.row_max[gr0 + qb * QB + tid];
      stat[1][tid] = g.row_inv[gr0 + qb * QB + tid];
      stat[2][tid] = g.row_dot[gr0 + qb * QB + tid];
    }
    if (qb + 1 < nqb) {
      lq.fetch(base + (int64_t)(qb + 1) * QB * ld, ld, QB, tid);
      la.fetch(g.da + (tok0 + (qb + 1) * QB) * g.d + h * DH, g.d, QB, tid);
    }
    __syncthreads();
    f16v s = zero16(), dp = zero16();                    // [key][query]
#pragma unroll
    for (int ks = 0; ks < DH; ks += 16) {
      s = mfma(frag_k(Ks, PT, k0, ks, lane), frag_k(Qs, PT, q0, ks, lane), s);
      dp = mfma(frag_k(Vs, PT, k0, ks, lane), frag_k(dAs, PT, q0, ks, lane), dp);
    }
    const int q = q0 + (lane & 31);
    const float mx = stat[0][q], inv = stat[1][q], dot = stat[2][q];
#pragma unroll
    for (int e4 = 0; e4 < 4; ++e4) {
      us4 po, so;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int key = k0 + acc_row(4 * e4 + u, lane);
        const bool keep = kb < qb || key <= q;
        const float pv = keep ? prob(s[4 * e4 + u] * scale, mx, inv) : 0.f;
        po[u] = f2bf(pv);
        so[u] = f2bf(pv * (dp[4 * e4 + u] - dot) * scale);
      }
      *reinterpret_cast<us4*>(Ps + q * PT + k0 + acc_row(4 * e4, lane)) = po;
      *reinterpret_cast<us4*>(dSs + q * PT + k0 + acc_row(4 * e4, lane)) = so;
    }
    __syncthreads();
    // dv += p^T da, dk += ds^T q: block (keys k0.., columns q0..), queries are the contraction
#pragma unroll
    for (int ks = 0; ks < QB; ks += 16) {
      dv = mfma(frag_t(Ps, PT, k0, ks, lane), frag_t(dAs, PT, q0, ks, lane), dv);
      dk = mfma(frag_t(dSs, PT, k0, ks, lane), frag_t(Qs, PT, q0, ks, lane), dk);
    }
  }
  uint16_t* dst = g.dqkv + (tok0 + kb * QB) * ld + h * DH;
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    const int64_t o = (int64_t)(k0 + acc_row(e, lane)) * ld + q0 + (lane & 31);
    dst[o + g.d] = f2bf(dk[e]);
    dst[o + 2 * g.d] = f2bf(dv[e]);
  }
}

attn_args make_args(const hdet_attn_desc& a) {
  attn_args g;
  g.qkv = a.qkv; g.a = a.a; g.da = a.da; g.dqkv = a.dqkv;
  g.row_max = a.row_max; g.row_inv = a.row_inv; g.row_dot = a.row_dot;
  g.ctrl = a.ctrl; g.temp_channel = a.temp_channel; g.scale = a.scale;
  g.B = a.batch; g.S = a.seq_len; g.heads = a.heads; g.d = a.d_model;
  return g;
}

}  // namespace

bool hdet_attn_fusable(int seq_len, int d_model, int heads) {
  return heads > 0 && d_model == heads * DH && seq_len % QB == 0 && seq_len >= QB && seq_len <= SMAX && d_model % 8 == 0;
}

hipError_t hdet_launch_attn_fwd(const hdet_attn_desc& a, hipStream_t s) {
  if (!hdet_attn_fusable(a.seq_len, a.d_model, a.heads)) return hipErrorInvalidValue;
  const dim3 grid(a.seq_len / QB, a.batch * a.heads, a.n_replicas);
  if (a.seq_len <= 256) hipLaunchKernelGGL(attn_fwd_kernel<4>, grid, dim3(256), 0, s, make_args(a));
  else hipLaunchKernelGGL(attn_fwd_kernel<8>, grid, dim3(512), 0, s, make_args(a));
  return hipGetLastError();
}

hipError_t hdet_launch_attn_bwd(const hdet_attn_desc& a, hipStream_t s) {
  if (!hdet_attn_fusable(a.seq_len, a.d_model, a.heads)) return hipErrorInvalidValue;
  const dim3 grid(a.seq_len / QB, a.batch * a.heads, a.n_replicas);
  if (a.seq_len <= 256) hipLaunchKernelGGL(attn_bwd_dq_kernel<4>, grid, dim3(256), 0, s, make_args(a));
  else hipLaunchKernelGGL(attn_bwd_dq_kernel<8>, grid, dim3(512), 0, s, make_args(a));
  hipLaunchKernelGGL(attn_bwd_dkv_kernel, grid, dim3(256), 0, s, make_args(a));
  return hipGetLastError();
}

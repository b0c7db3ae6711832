// Causal self-attention of the transformer replicas in mixed precision, forward and backward,
// with the scores kept on chip ("Forward + backward" of Algorithm 1 for the attention part of a
// block).  For head size 64 and sequence lengths that are multiples of 64 this replaces five
// batched GEMMs, two softmax kernels and the [S][S] score and probability tensors in HBM by
// three kernels that stream 64-row tiles of k, v (or q and the output gradient) through LDS.
//
// Arithmetic follows the unfused path operation by operation, so both agree to the rounding
// of the bf16 tensors they share:
//   forward   s = (q k^T) * scale (fp32), causal mask, p = bf16(exp(s - max) / sum), a = bf16(p v)
//   backward  dp = da v^T, dot = sum_j dp_j p_j, ds = bf16(p (dp - dot) scale),
//             dq = bf16(ds k), dk = bf16(ds^T q), dv = bf16(p^T da)
// with scale = 1 / (sqrt(d_head) tau_r), tau_r the replica's attention temperature when that is
// an explored channel (Remark 1).  Because p is rounded after the normalisation, every kernel
// that needs a row-wide quantity first (max and sum in the forward, dot in the backward) walks
// its tiles twice: once for the quantity, once for the product.  The exponential is the
// hardware's exp2 of fma(s, scale * log2 e, -max); the row maximum (in that scaled form) and
// 1/sum of the forward are kept ([rows] fp32 each) and the backward rebuilds p from them with
// the same expression, hence bit for bit.
//
// Layout: qkv [N][B][S][3d] bf16 (q | k | v, head h in columns h*64..), a and da [N][B][S][d],
// dqkv like qkv.  A block is 4 wavefronts; a wavefront owns 32 rows (queries in the forward and
// in the dq kernel, keys in the dk/dv kernel) whose operand fragments it loads once from global
// memory into registers, and walks the 64-row tiles of the other side, which the block stages
// in LDS (pitch 72 elements: the 128-bit fragment reads are free of bank conflicts) one tile
// ahead, with one barrier per tile.  Tiles are v_mfma_f32_32x32x16_bf16 blocks.  The first
// product is formed with the wavefront's own rows as the accumulator's COLUMNS, so that a lane
// holds one of its rows and 16 entries of the other side per block: row reductions stay inside
// a lane (plus one exchange between the half-wavefronts at the very end), and the accumulator
// registers, rounded to bf16, are directly the second product's B operand (contraction index =
// accumulator row) -- probabilities and ds never pass through LDS.  The accumulator keeps the
// rows of a 16-row step in the order (0..3, 8..11 | 4..7, 12..15) over the two half-wavefronts;
// the A operand of the second product is read from its LDS tile in that same order with the
// transposing LDS load, so nothing is transposed or permuted in memory.
// Every sum has a fixed order: results do not depend on scheduling.

#include "hdet_internal.h"
#include "hdet_elem.h"

// the forward and the two backward kernels must evaluate the exponent identically: one explicit fma, nothing contracted
#pragma clang fp contract(off)

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f16v __attribute__((ext_vector_type(16)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef short s4 __attribute__((ext_vector_type(4)));
typedef short s8 __attribute__((ext_vector_type(8)));
typedef unsigned short us8 __attribute__((ext_vector_type(8)));
typedef unsigned short us4 __attribute__((ext_vector_type(4)));

constexpr int DH = 64;            // head size
constexpr int TB = 64;            // rows of a streamed LDS tile
constexpr int PT = DH + 8;        // pitch of a [rows][64] tile
constexpr int WR = 32;            // rows a wavefront owns
constexpr int NWV = 4;            // wavefronts per block
constexpr int RB = WR * NWV;      // rows a block owns
constexpr int THREADS = 64 * NWV;
constexpr int TILE = TB * PT;     // elements of one LDS tile
constexpr int SMAX = 16384;       // longest sequence accepted
constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ unsigned short f2bf(float x) { return __builtin_bit_cast(unsigned short, (__bf16)x); }
__device__ __forceinline__ float bf2f(unsigned short h) { return __uint_as_float((unsigned)h << 16); }
__device__ __forceinline__ float bf16_round(float x) { return bf2f(f2bf(x)); }

// MFMA 32x32x16 operand fragment of lane l: (row = r0 + l % 32, k = ks + 8 * (l / 32) + 0..7).
// Tile stored [row][k] with `pitch` elements per row (pitch a multiple of 8).
__device__ __forceinline__ bf16x8 frag_k(const uint16_t* t, int pitch, int r0, int ks, int lane) {
  return *reinterpret_cast<const bf16x8*>(t + (r0 + (lane & 31)) * pitch + ks + ((lane >> 5) << 3));
}
// The same kind of fragment from global memory (row pitch ld elements)
__device__ __forceinline__ bf16x8 frag_g(const uint16_t* src, int64_t ld, int ks, int lane) {
  return *reinterpret_cast<const bf16x8*>(src + (int64_t)(lane & 31) * ld + ks + ((lane >> 5) << 3));
}
// Fragment of an operand that is contracted along its tile's ROW index (tile stored [k][row]),
// with the 16 k of the step in accumulator order: half-wavefront h holds k = ks + 4h + 0..3 and
// ks + 8 + 4h + 0..3.  Within a 16-lane group, lane p points at the 4 elements
// (k = kb + p / 4, rows rb + 4 * (p % 4) .. + 3) and lane i receives (k = kb .. kb + 3, row rb + i)
// from the transposing read.
__device__ __forceinline__ bf16x8 frag_tp(const uint16_t* t, int pitch, int r0, int ks, int lane) {
  const int p = lane & 15;
  const int row = r0 + (((lane >> 4) & 1) << 4) + ((p & 3) << 2);
  const int k = ks + ((lane >> 5) << 2) + (p >> 2);
  const uint16_t* q = t + k * pitch + row;
  const s4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s4 __attribute__((address_space(3)))*)(q));
  const s4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s4 __attribute__((address_space(3)))*)(q + 8 * pitch));
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
// elements 8 j .. 8 j + 7 of an accumulator block as the B fragment of contraction step j
__device__ __forceinline__ bf16x8 acc_frag(const float (&x)[16], int j) {
  bf16x8 f;
#pragma unroll
  for (int t = 0; t < 8; ++t) f[t] = (__bf16)x[8 * j + t];
  return f;
}
__device__ __forceinline__ float other_half(float x) { return __shfl_xor(x, 32); }
__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }
// The probability as the unfused path stores it (bf16), from the raw score s, c = scale log2 e,
// the row's maximum of s c and 1 / (row sum)
__device__ __forceinline__ float prob(float s, float c, float mx, float inv) { return bf16_round(exp2_fast(__builtin_fmaf(s, c, -mx)) * inv); }

// entries of an accumulator block whose row index (row0 + row in block) exceeds `limit` become `fill`
__device__ __forceinline__ void fill_above(float (&x)[16], int row0, int limit, int lane, float fill) {
#pragma unroll
  for (int e = 0; e < 16; ++e) x[e] = row0 + acc_row(e, lane) > limit ? fill : x[e];
}
// ... whose row index is below `limit`
__device__ __forceinline__ void fill_below(float (&x)[16], int row0, int limit, int lane, float fill) {
#pragma unroll
  for (int e = 0; e < 16; ++e) x[e] = row0 + acc_row(e, lane) < limit ? fill : x[e];
}

// One 64 x 64 bf16 tile from global memory (row pitch ld) to LDS (pitch PT) by the block's 256
// threads, in two phases so that the loads are in flight while the previous tile is worked on.
struct tile64 {
  us8 v[2];
  __device__ __forceinline__ void fetch(const uint16_t* src, int64_t ld, int tid) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int c = tid + i * THREADS;
      v[i] = *reinterpret_cast<const us8*>(src + (int64_t)(c >> 3) * ld + ((c & 7) << 3));
    }
  }
  __device__ __forceinline__ void commit(uint16_t* dst, int tid) const {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int c = tid + i * THREADS;
      *reinterpret_cast<us8*>(dst + (c >> 3) * PT + ((c & 7) << 3)) = v[i];
    }
  }
};

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

// Blocks reach the chip's 8 XCDs round-robin in launch order, and with causal masking the work of
// a block grows with its position in the sequence: left alone, an XCD would always receive the
// same position.  Launch index -> (row block, sequence and head, replica) such that every XCD
// works through a contiguous range of (replica, sequence, head) with all row blocks of each,
// which also keeps the tiles those share in one L2.
struct block_id { int x, bh, r; };
__device__ __forceinline__ block_id remap_block() {
  const unsigned nx = gridDim.x, ny = gridDim.y, total = nx * ny * gridDim.z;
  unsigned lin = blockIdx.x + nx * (blockIdx.y + ny * blockIdx.z);
  if ((total & 7u) == 0u) lin = (lin & 7u) * (total >> 3) + (lin >> 3);
  block_id b;
  const unsigned grp = lin / nx;
  // within an XCD the blocks go round-robin over shader engines and their CUs as well: rotate the
  // row block from one (sequence, head) to the next so that no unit keeps seeing the same one
  b.x = (lin % nx + grp + (grp >> 3) + (grp >> 6)) % nx;
  b.bh = grp % ny;
  b.r = grp / ny;
  return b;
}

// The wavefront's [32 rows][64] result, held transposed in two accumulator blocks (block dt:
// columns 32 dt .., lane = row), goes to `dst` (row pitch ld) through the wavefront's LDS strip
// so that every global store writes 16 bytes of a row.
__device__ __forceinline__ void store_rows(const f16v (&o)[2], uint16_t* stg, uint16_t* dst, int64_t ld, bool on, int lane) {
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int e4 = 0; e4 < 4; ++e4) {
      const us4 x = {f2bf(o[dt][4 * e4]), f2bf(o[dt][4 * e4 + 1]), f2bf(o[dt][4 * e4 + 2]), f2bf(o[dt][4 * e4 + 3])};
      *reinterpret_cast<us4*>(stg + (lane & 31) * PT + dt * 32 + acc_row(4 * e4, lane)) = x;
    }
  __syncthreads();
  if (on) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int c = lane + 64 * i, row = c >> 3, col = (c & 7) << 3;
      *reinterpret_cast<us8*>(dst + (int64_t)row * ld + col) = *reinterpret_cast<const us8*>(stg + row * PT + col);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// forward: block = 128 queries of one (replica, sequence, head)
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(THREADS, 4) void attn_fwd_kernel(const attn_args g) {
  __shared__ __attribute__((aligned(16))) uint16_t smem[4 * TILE];        // keys x 2, values x 2
  const block_id blk = remap_block();
  const int qblk = gridDim.x - 1 - blk.x, bh = blk.bh, r = blk.r;         // longest blocks first
  const int b = bh / g.heads, h = bh - b * g.heads;
  const int tid = threadIdx.x, lane = tid & 63, qi = lane & 31;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int64_t ld = 3 * (int64_t)g.d;
  const int64_t tok0 = ((int64_t)r * g.B + b) * g.S;
  const uint16_t* base = g.qkv + tok0 * ld + h * DH;
  const uint16_t* ksrc = base + g.d;
  const uint16_t* vsrc = base + 2 * g.d;
  const int q0 = qblk * RB, wq0 = q0 + w * WR;
  const bool on = wq0 < g.S;                                               // S is a multiple of 64, not of 128
  const int nkb = (q0 + RB < g.S ? q0 + RB : g.S) / TB;                    // key tiles the block walks
  const int nkw = on ? (wq0 + WR - 1) / TB + 1 : 0;                        // ... and this wavefront
  const float c = replica_scale(g, r) * kLog2e;

  bf16x8 fq[4];
#pragma unroll
  for (int k4 = 0; k4 < 4; ++k4) fq[k4] = frag_g(base + (int64_t)(on ? wq0 : 0) * ld, ld, k4 * 16, lane);

  // Raw scores of 32-key block i of key tile kb, [key][query], -inf above the diagonal
  auto scores = [&](const uint16_t* kt, int kb, int i, float (&x)[16]) {
    f16v s = zero16();
#pragma unroll
    for (int k4 = 0; k4 < 4; ++k4) s = mfma(frag_k(kt, PT, 32 * i, k4 * 16, lane), fq[k4], s);
#pragma unroll
    for (int e = 0; e < 16; ++e) x[e] = s[e];
    const int key0 = kb * TB + 32 * i;
    if (key0 + 31 > wq0) fill_above(x, key0, wq0 + qi, lane, -INFINITY);
  };
  // the second block of a tile is left out when it lies above the diagonal altogether
  auto blocks_of = [&](int kb) { return kb * TB + 32 > wq0 + WR - 1 ? 1 : 2; };

  // pass 1: row maximum (of the raw scores) and sum, each half-wavefront over its own keys
  tile64 lk, lv;
  float m = -1e30f, l = 0.f;
  lk.fetch(ksrc, ld, tid);
  lk.commit(smem, tid);
  if (nkb > 1) lk.fetch(ksrc + (int64_t)TB * ld, ld, tid);
  __syncthreads();
  for (int kb = 0; kb < nkb; ++kb) {
    if (kb + 1 < nkb) lk.commit(smem + ((kb + 1) & 1) * TILE, tid);
    if (kb + 2 < nkb) lk.fetch(ksrc + (int64_t)(kb + 2) * TB * ld, ld, tid);
    if (kb < nkw) {
      const int nb = blocks_of(kb);
      for (int i = 0; i < nb; ++i) {
        float x[16];
        scores(smem + (kb & 1) * TILE, kb, i, x);
        float top = m;
#pragma unroll
        for (int e = 0; e < 16; ++e) top = fmaxf(top, x[e]);
        const float tc = top * c;
        float sum = 0.f;
#pragma unroll
        for (int e = 0; e < 16; ++e) sum += exp2_fast(__builtin_fmaf(x[e], c, -tc));
        l = l * exp2_fast((m - top) * c) + sum;
        m = top;
      }
    }
    __syncthreads();
  }
  const float mo = other_half(m), lo = other_half(l);
  const float top = fmaxf(m, mo);
  const float mx = top * c;
  const float inv = 1.f / (l * exp2_fast((m - top) * c) + lo * exp2_fast((mo - top) * c));
  if (on && lane < 32) {
    const int64_t gr = (((int64_t)r * g.B + b) * g.heads + h) * g.S + wq0 + qi;
    g.row_max[gr] = mx;
    g.row_inv[gr] = inv;
  }

  // pass 2: a^T = v^T p^T, [column][query]
  f16v o[2] = {zero16(), zero16()};
  lk.fetch(ksrc, ld, tid);
  lv.fetch(vsrc, ld, tid);
  lk.commit(smem, tid);
  lv.commit(smem + 2 * TILE, tid);
  if (nkb > 1) { lk.fetch(ksrc + (int64_t)TB * ld, ld, tid); lv.fetch(vsrc + (int64_t)TB * ld, ld, tid); }
  __syncthreads();
  for (int kb = 0; kb < nkb; ++kb) {
    if (kb + 1 < nkb) { lk.commit(smem + ((kb + 1) & 1) * TILE, tid); lv.commit(smem + (2 + ((kb + 1) & 1)) * TILE, tid); }
    if (kb + 2 < nkb) { lk.fetch(ksrc + (int64_t)(kb + 2) * TB * ld, ld, tid); lv.fetch(vsrc + (int64_t)(kb + 2) * TB * ld, ld, tid); }
    if (kb < nkw) {
      const uint16_t* vt = smem + (2 + (kb & 1)) * TILE;
      const int nb = blocks_of(kb);
      for (int i = 0; i < nb; ++i) {
        float x[16];
        scores(smem + (kb & 1) * TILE, kb, i, x);
#pragma unroll
        for (int e = 0; e < 16; ++e) x[e] = exp2_fast(__builtin_fmaf(x[e], c, -mx)) * inv;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const bf16x8 pf = acc_frag(x, j);
#pragma unroll
          for (int dt = 0; dt < 2; ++dt) o[dt] = mfma(frag_tp(vt, PT, 32 * dt, 32 * i + 16 * j, lane), pf, o[dt]);
        }
      }
    }
    __syncthreads();
  }
  store_rows(o, smem + w * WR * PT, g.a + (tok0 + (on ? wq0 : 0)) * g.d + h * DH, g.d, on, lane);
}

// ---------------------------------------------------------------------------------------------
// backward, step 1: the row dots and dq; block = 128 queries
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(THREADS, 2) void attn_bwd_dq_kernel(const attn_args g) {
  __shared__ __attribute__((aligned(16))) uint16_t smem[4 * TILE];        // keys x 2, values x 2
  const block_id blk = remap_block();
  const int qblk = gridDim.x - 1 - blk.x, bh = blk.bh, r = blk.r;
  const int b = bh / g.heads, h = bh - b * g.heads;
  const int tid = threadIdx.x, lane = tid & 63, qi = lane & 31;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int64_t ld = 3 * (int64_t)g.d;
  const int64_t tok0 = ((int64_t)r * g.B + b) * g.S;
  const uint16_t* base = g.qkv + tok0 * ld + h * DH;
  const uint16_t* ksrc = base + g.d;
  const uint16_t* vsrc = base + 2 * g.d;
  const int q0 = qblk * RB, wq0 = q0 + w * WR;
  const bool on = wq0 < g.S;
  const int nkb = (q0 + RB < g.S ? q0 + RB : g.S) / TB;
  const int nkw = on ? (wq0 + WR - 1) / TB + 1 : 0;
  const float scale = replica_scale(g, r);
  const float c = scale * kLog2e;
  const int64_t gr = (((int64_t)r * g.B + b) * g.heads + h) * g.S + (on ? wq0 : 0) + qi;
  const float mx = g.row_max[gr], inv = g.row_inv[gr];

  bf16x8 fq[4], fda[4];
#pragma unroll
  for (int k4 = 0; k4 < 4; ++k4) {
    fq[k4] = frag_g(base + (int64_t)(on ? wq0 : 0) * ld, ld, k4 * 16, lane);
    fda[k4] = frag_g(g.da + (tok0 + (on ? wq0 : 0)) * g.d + h * DH, g.d, k4 * 16, lane);
  }

  // p and dp = v da^T of key block i of tile kb, both [key][query]; false above the diagonal
  auto p_and_dp = [&](const uint16_t* kt, const uint16_t* vt, int kb, int i, float (&p)[16], f16v& dp) -> bool {
    const int key0 = kb * TB + 32 * i;
    if (key0 > wq0 + WR - 1) return false;
    f16v s = zero16();
    dp = zero16();
#pragma unroll
    for (int k4 = 0; k4 < 4; ++k4) {
      s = mfma(frag_k(kt, PT, 32 * i, k4 * 16, lane), fq[k4], s);
      dp = mfma(frag_k(vt, PT, 32 * i, k4 * 16, lane), fda[k4], dp);
    }
#pragma unroll
    for (int e = 0; e < 16; ++e) p[e] = prob(s[e], c, mx, inv);
    if (key0 + 31 > wq0) fill_above(p, key0, wq0 + qi, lane, 0.f);
    return true;
  };

  tile64 lk, lv;
  auto prologue = [&]() {
    lk.fetch(ksrc, ld, tid);
    lv.fetch(vsrc, ld, tid);
    lk.commit(smem, tid);
    lv.commit(smem + 2 * TILE, tid);
    if (nkb > 1) { lk.fetch(ksrc + (int64_t)TB * ld, ld, tid); lv.fetch(vsrc + (int64_t)TB * ld, ld, tid); }
    __syncthreads();
  };
  auto advance = [&](int kb) {
    if (kb + 1 < nkb) { lk.commit(smem + ((kb + 1) & 1) * TILE, tid); lv.commit(smem + (2 + ((kb + 1) & 1)) * TILE, tid); }
    if (kb + 2 < nkb) { lk.fetch(ksrc + (int64_t)(kb + 2) * TB * ld, ld, tid); lv.fetch(vsrc + (int64_t)(kb + 2) * TB * ld, ld, tid); }
  };

  // pass 1: dot = sum over the keys of dp p
  float dot = 0.f;
  prologue();
  for (int kb = 0; kb < nkb; ++kb) {
    advance(kb);
    if (kb < nkw) {
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        float p[16];
        f16v dp;
        if (!p_and_dp(smem + (kb & 1) * TILE, smem + (2 + (kb & 1)) * TILE, kb, i, p, dp)) continue;
#pragma unroll
        for (int e = 0; e < 16; ++e) dot = __builtin_fmaf(dp[e], p[e], dot);
      }
    }
    __syncthreads();
  }
  dot += other_half(dot);
  if (on && lane < 32) g.row_dot[gr] = dot;

  // pass 2: dq^T = k^T ds^T, [column][query]
  f16v o[2] = {zero16(), zero16()};
  prologue();
  for (int kb = 0; kb < nkb; ++kb) {
    advance(kb);
    if (kb < nkw) {
      const uint16_t* kt = smem + (kb & 1) * TILE;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        float p[16];
        f16v dp;
        if (!p_and_dp(kt, smem + (2 + (kb & 1)) * TILE, kb, i, p, dp)) continue;
#pragma unroll
        for (int e = 0; e < 16; ++e) p[e] = p[e] * (dp[e] - dot) * scale;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const bf16x8 dsf = acc_frag(p, j);
#pragma unroll
          for (int dt = 0; dt < 2; ++dt) o[dt] = mfma(frag_tp(kt, PT, 32 * dt, 32 * i + 16 * j, lane), dsf, o[dt]);
        }
      }
    }
    __syncthreads();
  }
  store_rows(o, smem + w * WR * PT, g.dqkv + (tok0 + (on ? wq0 : 0)) * ld + h * DH, ld, on, lane);
}

// ---------------------------------------------------------------------------------------------
// backward, step 2: dk and dv; block = 128 keys, walks the query tiles at or below the diagonal
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(THREADS, 2) void attn_bwd_dkv_kernel(const attn_args g) {
  __shared__ __attribute__((aligned(16))) uint16_t smem[4 * TILE];        // queries x 2, output gradients x 2
  __shared__ __attribute__((aligned(16))) float st[2][3][TB];             // row max, 1 / row sum, row dot of the tile's queries
  const block_id blk = remap_block();
  const int kblk = blk.x, bh = blk.bh, r = blk.r;                          // the first blocks walk the most tiles
  const int b = bh / g.heads, h = bh - b * g.heads;
  const int tid = threadIdx.x, lane = tid & 63, ki = lane & 31;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int64_t ld = 3 * (int64_t)g.d;
  const int64_t tok0 = ((int64_t)r * g.B + b) * g.S;
  const uint16_t* base = g.qkv + tok0 * ld + h * DH;
  const uint16_t* dasrc = g.da + tok0 * g.d + h * DH;
  const int64_t gr0 = (((int64_t)r * g.B + b) * g.heads + h) * g.S;
  const int k0 = kblk * RB, wk0 = k0 + w * WR;
  const bool on = wk0 < g.S;
  const int qb0 = k0 / TB, nqb = g.S / TB;
  const float scale = replica_scale(g, r);
  const float c = scale * kLog2e;

  bf16x8 fk[4], fv[4];
#pragma unroll
  for (int k4 = 0; k4 < 4; ++k4) {
    fk[k4] = frag_g(base + g.d + (int64_t)(on ? wk0 : 0) * ld, ld, k4 * 16, lane);
    fv[k4] = frag_g(base + 2 * g.d + (int64_t)(on ? wk0 : 0) * ld, ld, k4 * 16, lane);
  }

  tile64 lq, la;
  float sv = 0.f;                                                          // one row statistic per thread < 192
  const float* ssrc = tid < TB ? g.row_max : tid < 2 * TB ? g.row_inv : g.row_dot;
  auto fetch = [&](int qb) {
    lq.fetch(base + (int64_t)qb * TB * ld, ld, tid);
    la.fetch(dasrc + (int64_t)qb * TB * g.d, g.d, tid);
    if (tid < 3 * TB) sv = ssrc[gr0 + qb * TB + (tid & (TB - 1))];
  };
  auto commit = [&](int buf) {
    lq.commit(smem + buf * TILE, tid);
    la.commit(smem + (2 + buf) * TILE, tid);
    if (tid < 3 * TB) st[buf][tid >> 6][tid & (TB - 1)] = sv;
  };

  f16v dk[2] = {zero16(), zero16()}, dv[2] = {zero16(), zero16()};        // [column][key]
  fetch(qb0);
  commit(0);
  if (qb0 + 1 < nqb) fetch(qb0 + 1);
  __syncthreads();
  for (int qb = qb0; qb < nqb; ++qb) {
    const int buf = (qb - qb0) & 1;
    if (qb + 1 < nqb) commit(buf ^ 1);
    if (qb + 2 < nqb) fetch(qb + 2);
    if (on && qb * TB + TB - 1 >= wk0) {
      const uint16_t* qt = smem + buf * TILE;
      const uint16_t* dat = smem + (2 + buf) * TILE;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int qr0 = qb * TB + 32 * i;                                  // first query of the block
        if (qr0 + 31 < wk0) continue;                                      // all its queries precede the keys
        f16v s = zero16(), dp = zero16();                                  // [query][key]
#pragma unroll
        for (int k4 = 0; k4 < 4; ++k4) {
          s = mfma(frag_k(qt, PT, 32 * i, k4 * 16, lane), fk[k4], s);
          dp = mfma(frag_k(dat, PT, 32 * i, k4 * 16, lane), fv[k4], dp);
        }
        float p[16], ds[16];
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
          const int row = 32 * i + acc_row(4 * e4, lane);                  // 4 consecutive queries of the tile
          const f4 mx = *reinterpret_cast<const f4*>(&st[buf][0][row]);
          const f4 inv = *reinterpret_cast<const f4*>(&st[buf][1][row]);
#pragma unroll
          for (int u = 0; u < 4; ++u) p[4 * e4 + u] = prob(s[4 * e4 + u], c, mx[u], inv[u]);
        }
        if (qr0 < wk0 + WR - 1) fill_below(p, qr0, wk0 + ki, lane, 0.f);   // causal: query >= key
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
          const f4 dot = *reinterpret_cast<const f4*>(&st[buf][2][32 * i + acc_row(4 * e4, lane)]);
#pragma unroll
          for (int u = 0; u < 4; ++u) ds[4 * e4 + u] = p[4 * e4 + u] * (dp[4 * e4 + u] - dot[u]) * scale;
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const bf16x8 pf = acc_frag(p, j), dsf = acc_frag(ds, j);
#pragma unroll
          for (int dt = 0; dt < 2; ++dt) {
            dv[dt] = mfma(frag_tp(dat, PT, 32 * dt, 32 * i + 16 * j, lane), pf, dv[dt]);
            dk[dt] = mfma(frag_tp(qt, PT, 32 * dt, 32 * i + 16 * j, lane), dsf, dk[dt]);
          }
        }
      }
    }
    __syncthreads();
  }
  uint16_t* dst = g.dqkv + (tok0 + (on ? wk0 : 0)) * ld + h * DH;
  store_rows(dk, smem + w * WR * PT, dst + g.d, ld, on, lane);
  __syncthreads();
  store_rows(dv, smem + w * WR * PT, dst + 2 * g.d, ld, on, lane);
}

attn_args make_args(const hdet_attn_desc& a) {
  attn_args g;
  g.qkv = a.qkv; g.a = a.a; g.da = a.da; g.dqkv = a.dqkv;
  g.row_max = a.row_max; g.row_inv = a.row_inv; g.row_dot = a.row_dot;
  g.ctrl = a.ctrl; g.temp_channel = a.temp_channel; g.scale = a.scale;
  g.B = a.batch; g.S = a.seq_len; g.heads = a.heads; g.d = a.d_model;
  return g;
}

dim3 attn_grid(const hdet_attn_desc& a) { return dim3((a.seq_len + RB - 1) / RB, a.batch * a.heads, a.n_replicas); }

}  // namespace

bool hdet_attn_fusable(int seq_len, int d_model, int heads, int batch) {
  return heads > 0 && batch > 0 && d_model == heads * DH && seq_len % TB == 0 && seq_len >= TB && seq_len <= SMAX &&
         (int64_t)batch * heads <= 65535;
}

hipError_t hdet_launch_attn_fwd(const hdet_attn_desc& a, hipStream_t s) {
  if (!hdet_attn_fusable(a.seq_len, a.d_model, a.heads, a.batch)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(attn_fwd_kernel, attn_grid(a), dim3(THREADS), 0, s, make_args(a));
  return hipGetLastError();
}

hipError_t hdet_launch_attn_bwd(const hdet_attn_desc& a, hipStream_t s) {
  if (!hdet_attn_fusable(a.seq_len, a.d_model, a.heads, a.batch)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(attn_bwd_dq_kernel, attn_grid(a), dim3(THREADS), 0, s, make_args(a));
  hipLaunchKernelGGL(attn_bwd_dkv_kernel, attn_grid(a), dim3(THREADS), 0, s, make_args(a));
  return hipGetLastError();
}

// "Forward + backward" of Algorithm 1 for a decoder-only transformer, replica-batched: every
// launch covers all N replicas (independent weight sets, the replica is the outermost batch
// index of each GEMM and grid.y of each row/elementwise kernel).
//
// Model (what the benchmark configurations leave open is fixed here): pre-LayerNorm blocks,
// learned positional embeddings, tanh-GELU MLP, causal softmax attention, biases on every
// Linear, untied output head with bias, final LayerNorm, eps 1e-5, mean next-token
// cross-entropy over all B*S positions.  Dropout (Remark 1: the dropout rate as an explored
// hyperparameter) acts on the two residual branches of a block with keep-scaling 1/(1-p), the
// rate being replica r's value of the dropout channel; the mask is regenerated in the backward
// pass from Philox-4x32-10 keyed on (seed, step, replica, site, element), never stored.
//
// All matrix products go through the replica-batched GEMMs (matrix cores in bf16 precision,
// LDS-tiled fp32 otherwise); attention is the unfused chain scores -> softmax -> P V with the
// (replica, sequence, head) triple as the batch index.  Activations that go to memory are of
// type T: float, or bfloat16 in mixed precision (logits, attention scores and LayerNorm
// statistics stay fp32).

#include <vector>

#include "hdet_elem.h"
#include "hdet_internal.h"

namespace {

constexpr float kLnEps = 1e-5f;
constexpr uint32_t kDropStream = 0x44524F50u;   // "DROP"
constexpr int kColsumRows = 128;                // rows per block in stage 1 of the column sums

// ------------------------------------------------------------------------------------------
// elementwise / row kernels; blockIdx.y = replica
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void embed_fwd_kernel(const float* theta, int64_t ps, int64_t tok_off, int64_t pos_off,
                                                        const int32_t* ids, int M, int S, int d, T* x) {
  const int r = blockIdx.y;
  const float* tok = theta + (int64_t)r * ps + tok_off;
  const float* pos = theta + (int64_t)r * ps + pos_off;
  const int64_t n = (int64_t)M * d;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const int m = (int)(i / d), c = (int)(i % d);
    const int id = ids[(int64_t)r * M + m];
    hdet_st(x + (int64_t)r * n + i, tok[(int64_t)id * d + c] + pos[(int64_t)(m % S) * d + c]);
  }
}

// dtok[ids[m]] += dx[m] with fp32 atomics (the region is zeroed first), for the shapes the ordered
// kernels below do not take: the one sum of the backward pass whose order is then left to the hardware.
template <typename T>
__global__ __launch_bounds__(256) void embed_bwd_kernel(float* grads, int64_t ps, int64_t tok_off, const int32_t* ids, int M, int d,
                                                        const T* dx) {
  const int r = blockIdx.y;
  float* tok = grads + (int64_t)r * ps + tok_off;
  const int64_t n = (int64_t)M * d;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const int m = (int)(i / d), c = (int)(i % d);
    atomicAdd(tok + (int64_t)ids[(int64_t)r * M + m] * d + c, hdet_ld(dx + (int64_t)r * n + i));
  }
}
// The same sum in a fixed order, for M up to 16384 rows per replica and d a multiple of 8 up to 2048:
// (1) one block per replica sorts the keys (token id, row) in LDS (bitonic network over the next power
// of two, padded with all-ones keys), so that the rows of a token id are adjacent and ascending;
// (2) one wavefront per sorted position: where a new id starts, it adds that id's rows of dx in
// ascending row order and writes the token's gradient row (the region is zeroed first for the ids
// that do not occur).
template <int P2>
__global__ __launch_bounds__(1024) void tok_sort_kernel(const int32_t* ids, int M, unsigned long long* sorted) {
  __shared__ unsigned long long keys[P2];
  const int r = blockIdx.x, tid = threadIdx.x;
  for (int i = tid; i < P2; i += 1024)
    keys[i] = i < M ? ((unsigned long long)(uint32_t)ids[(int64_t)r * M + i] << 32) | (uint32_t)i : ~0ull;
  __syncthreads();
  for (int k = 2; k <= P2; k <<= 1)
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int t = tid; t < P2 / 2; t += 1024) {
        const int i = 2 * j * (t / j) + (t % j);
        const unsigned long long a = keys[i], b = keys[i + j];
        if ((a > b) == ((i & k) == 0)) { keys[i] = b; keys[i + j] = a; }
      }
      __syncthreads();
    }
  for (int i = tid; i < M; i += 1024) sorted[(int64_t)r * M + i] = keys[i];
}
// Step (2) runs in two levels so that a frequent token does not serialise one wavefront: level 1
// sums the rows of every segment -- a maximal run of one id inside a block of kTokChunk sorted
// positions -- into seg[first position of the segment]; level 2 adds the segments of each id in
// ascending order and writes the token's gradient row.
constexpr int kTokChunk = 32;
__device__ __forceinline__ uint32_t key_id(unsigned long long key) { return (uint32_t)(key >> 32); }
template <int NCH>
__device__ __forceinline__ void add_row(hdet_f8 (&acc)[NCH], const hdet_f8 (&v)[NCH], int lane, int d8) {
#pragma unroll
  for (int i = 0; i < NCH; ++i)
    if (lane + 64 * i < d8) {
#pragma unroll
      for (int c = 0; c < 8; ++c) acc[i].v[c] += v[i].v[c];
    }
}
template <typename T, int NCH>
__global__ __launch_bounds__(256) void tok_segment_kernel(const unsigned long long* sorted, int M, int d, const T* dx, float* seg) {
  constexpr int U = NCH == 1 ? 8 : 4;               // rows in flight, by register budget
  const int r = blockIdx.y, lane = threadIdx.x & 63;
  const int j0 = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (j0 >= M) return;
  const unsigned long long* sk = sorted + (int64_t)r * M;
  const uint32_t id = key_id(sk[j0]);
  if (j0 % kTokChunk != 0 && key_id(sk[j0 - 1]) == id) return;      // inside a segment
  const int jend = (j0 / kTokChunk + 1) * kTokChunk < M ? (j0 / kTokChunk + 1) * kTokChunk : M;
  const int d8 = d >> 3;
  const T* src = dx + (int64_t)r * M * d;
  hdet_f8 acc[NCH];
#pragma unroll
  for (int i = 0; i < NCH; ++i)
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[i].v[c] = 0.f;
  for (int j = j0; j < jend; j += U) {
    hdet_f8 v[U][NCH];
    unsigned long long key[U];
#pragma unroll
    for (int u = 0; u < U; ++u) key[u] = sk[j + u < jend ? j + u : jend - 1];
    int n = 0;                                                       // rows of this id among the next U positions
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (n == u && j + u < jend && key_id(key[u]) == id) n = u + 1;
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (u < n) {
        const int64_t row = (int64_t)(uint32_t)key[u] * d;
#pragma unroll
        for (int i = 0; i < NCH; ++i)
          if (lane + 64 * i < d8) v[u][i] = hdet_ld8(src + row + 8 * (lane + 64 * i));
      }
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (u < n) add_row<NCH>(acc, v[u], lane, d8);
    if (n < U) break;
  }
  float* dst = seg + ((int64_t)r * M + j0) * d;
#pragma unroll
  for (int i = 0; i < NCH; ++i)
    if (lane + 64 * i < d8) hdet_st8(dst + 8 * (lane + 64 * i), acc[i]);
}
template <int NCH>
__global__ __launch_bounds__(256) void tok_total_kernel(const unsigned long long* sorted, int M, int d, const float* seg, float* grads,
                                                        int64_t ps, int64_t tok_off) {
  constexpr int U = NCH == 1 ? 8 : 4;               // rows in flight, by register budget
  const int r = blockIdx.y, lane = threadIdx.x & 63;
  const int j0 = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (j0 >= M) return;
  const unsigned long long* sk = sorted + (int64_t)r * M;
  const uint32_t id = key_id(sk[j0]);
  if (j0 > 0 && key_id(sk[j0 - 1]) == id) return;                    // not the first row of its id
  const int d8 = d >> 3;
  const float* src = seg + (int64_t)r * M * d;
  hdet_f8 acc[NCH];
#pragma unroll
  for (int i = 0; i < NCH; ++i) acc[i] = hdet_ld8(src + (int64_t)j0 * d + 8 * (lane + 64 * i < d8 ? lane + 64 * i : 0));
  // the id's further segments start at the multiples of kTokChunk behind j0, as long as the id goes on
  for (int j = (j0 / kTokChunk + 1) * kTokChunk; j < M; j += U * kTokChunk) {
    hdet_f8 v[U][NCH];
    uint32_t kid[U];
#pragma unroll
    for (int u = 0; u < U; ++u) kid[u] = key_id(sk[j + u * kTokChunk < M ? j + u * kTokChunk : M - 1]);
    int n = 0;
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (n == u && j + u * kTokChunk < M && kid[u] == id) n = u + 1;
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (u < n) {
#pragma unroll
        for (int i = 0; i < NCH; ++i)
          if (lane + 64 * i < d8) v[u][i] = hdet_ld8(src + (int64_t)(j + u * kTokChunk) * d + 8 * (lane + 64 * i));
      }
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (u < n) add_row<NCH>(acc, v[u], lane, d8);
    if (n < U) break;
  }
  float* dst = grads + (int64_t)r * ps + tok_off + (int64_t)id * d;
#pragma unroll
  for (int i = 0; i < NCH; ++i)
    if (lane + 64 * i < d8) hdet_st8(dst + 8 * (lane + 64 * i), acc[i]);
}

// dpos[s] = sum over the sequences b, in ascending order, of dx[b S + s]
template <typename T>
__global__ __launch_bounds__(256) void pos_bwd_kernel(float* grads, int64_t ps, int64_t pos_off, int B, int S, int d, const T* dx) {
  const int r = blockIdx.y;
  float* pos = grads + (int64_t)r * ps + pos_off;
  const int64_t n = (int64_t)S * d;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    float a = 0.f;
    for (int b = 0; b < B; ++b) a += hdet_ld(dx + ((int64_t)r * B + b) * n + i);
    pos[i] = a;
  }
}

// Weight gradient formed in `splits` pieces along the contraction (the rows of the batch): dW = sum of the pieces in
// the order 0 .. splits-1.  part[(replica * splits + piece) * len + i], len a multiple of 4.
__global__ __launch_bounds__(256) void wgrad_sum_kernel(const float* part, int splits, int64_t len, float* grads, int64_t ps, int64_t w_off) {
  typedef float f4 __attribute__((ext_vector_type(4)));
  const int r = blockIdx.y;
  const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i >= len) return;
  const float* src = part + (int64_t)r * splits * len + i;
  f4 acc = *reinterpret_cast<const f4*>(src);
  for (int sidx = 1; sidx < splits; ++sidx) acc += *reinterpret_cast<const f4*>(src + sidx * len);
  *reinterpret_cast<f4*>(grads + (int64_t)r * ps + w_off + i) = acc;
}

__global__ __launch_bounds__(256) void zero_kernel(float* p, int64_t ps, int64_t off, int64_t n) {
  float* q = p + (int64_t)blockIdx.y * ps + off;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) q[i] = 0.f;
}

// LayerNorm forward, one wavefront per row: two passes (mean, then variance about it).
template <typename T>
__global__ __launch_bounds__(256) void ln_fwd_kernel(const T* x, const float* theta, int64_t ps, int64_t g_off,
                                                     int64_t b_off, int M, int d, T* y, float* mean, float* rstd) {
  const int r = blockIdx.y, lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= M) return;
  const int64_t base = ((int64_t)r * M + row) * d;
  const float* g = theta + (int64_t)r * ps + g_off;
  const float* b = theta + (int64_t)r * ps + b_off;
  float s = 0.f;
  for (int c = lane; c < d; c += 64) s += hdet_ld(x + base + c);
  const float mu = hdet_wave_sum(s) / (float)d;
  float v = 0.f;
  for (int c = lane; c < d; c += 64) { const float t = hdet_ld(x + base + c) - mu; v += t * t; }
  const float rs = 1.f / sqrtf(hdet_wave_sum(v) / (float)d + kLnEps);
  for (int c = lane; c < d; c += 64) hdet_st(y + base + c, (hdet_ld(x + base + c) - mu) * rs * g[c] + b[c]);
  if (lane == 0) { mean[(int64_t)r * M + row] = mu; rstd[(int64_t)r * M + row] = rs; }
}

// dx = rstd * (dxhat - mean(dxhat) - xhat * mean(dxhat * xhat)) [+ resid], dxhat = dy * g
template <typename T>
__global__ __launch_bounds__(256) void ln_bwd_dx_kernel(const T* dy, const T* x, const float* mean, const float* rstd,
                                                        const float* theta, int64_t ps, int64_t g_off, int M, int d,
                                                        const T* resid, T* dx) {
  const int r = blockIdx.y, lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= M) return;
  const int64_t base = ((int64_t)r * M + row) * d;
  const float* g = theta + (int64_t)r * ps + g_off;
  const float mu = mean[(int64_t)r * M + row], rs = rstd[(int64_t)r * M + row];
  float s1 = 0.f, s2 = 0.f;
  for (int c = lane; c < d; c += 64) {
    const float dxh = hdet_ld(dy + base + c) * g[c];
    s1 += dxh;
    s2 += dxh * ((hdet_ld(x + base + c) - mu) * rs);
  }
  const float m1 = hdet_wave_sum(s1) / (float)d, m2 = hdet_wave_sum(s2) / (float)d;
  for (int c = lane; c < d; c += 64) {
    const float xh = (hdet_ld(x + base + c) - mu) * rs;
    float v = rs * (hdet_ld(dy + base + c) * g[c] - m1 - xh * m2);
    if (resid) v += hdet_ld(resid + base + c);
    hdet_st(dx + base + c, v);
  }
}

// Vector forms of the two LayerNorm row kernels for d % 8 == 0, d <= 2048: the row lives in
// registers (lane l owns the 8-element chunks l, l + 64, ...), so it is read from memory once.
template <typename T, int NCH>
__global__ __launch_bounds__(256) void ln_fwd_vec_kernel(const T* x, const float* theta, int64_t ps, int64_t g_off,
                                                         int64_t b_off, int M, int d, T* y, float* mean, float* rstd) {
  const int r = blockIdx.y, lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= M) return;
  const int64_t base = ((int64_t)r * M + row) * d;
  const float* g = theta + (int64_t)r * ps + g_off;
  const float* b = theta + (int64_t)r * ps + b_off;
  const int d8 = d >> 3;
  hdet_f8 xv[NCH];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int ch = lane + 64 * i;
    if (ch < d8) {
      xv[i] = hdet_ld8(x + base + 8 * ch);
#pragma unroll
      for (int j = 0; j < 8; ++j) s += xv[i].v[j];
    }
  }
  const float mu = hdet_wave_sum(s) / (float)d;
  float v = 0.f;
#pragma unroll
  for (int i = 0; i < NCH; ++i)
    if (lane + 64 * i < d8) {
#pragma unroll
      for (int j = 0; j < 8; ++j) { const float t = xv[i].v[j] - mu; v += t * t; }
    }
  const float rs = 1.f / sqrtf(hdet_wave_sum(v) / (float)d + kLnEps);
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int ch = lane + 64 * i;
    if (ch < d8) {
      const hdet_f8 gv = hdet_ld8(g + 8 * ch), bv = hdet_ld8(b + 8 * ch);
      hdet_f8 o;
#pragma unroll
      for (int j = 0; j < 8; ++j) o.v[j] = (xv[i].v[j] - mu) * rs * gv.v[j] + bv.v[j];
      hdet_st8(y + base + 8 * ch, o);
    }
  }
  if (lane == 0) { mean[(int64_t)r * M + row] = mu; rstd[(int64_t)r * M + row] = rs; }
}

template <typename T, int NCH>
__global__ __launch_bounds__(256) void ln_bwd_dx_vec_kernel(const T* dy, const T* x, const float* mean, const float* rstd,
                                                            const float* theta, int64_t ps, int64_t g_off, int M, int d,
                                                            const T* resid, T* dx) {
  const int r = blockIdx.y, lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= M) return;
  const int64_t base = ((int64_t)r * M + row) * d;
  const float* g = theta + (int64_t)r * ps + g_off;
  const float mu = mean[(int64_t)r * M + row], rs = rstd[(int64_t)r * M + row];
  const int d8 = d >> 3;
  hdet_f8 dxh[NCH], xh[NCH];
  float s1 = 0.f, s2 = 0.f;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int ch = lane + 64 * i;
    if (ch < d8) {
      const hdet_f8 dyv = hdet_ld8(dy + base + 8 * ch), xv = hdet_ld8(x + base + 8 * ch), gv = hdet_ld8(g + 8 * ch);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        dxh[i].v[j] = dyv.v[j] * gv.v[j];
        xh[i].v[j] = (xv.v[j] - mu) * rs;
        s1 += dxh[i].v[j];
        s2 += dxh[i].v[j] * xh[i].v[j];
      }
    }
  }
  const float m1 = hdet_wave_sum(s1) / (float)d, m2 = hdet_wave_sum(s2) / (float)d;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int ch = lane + 64 * i;
    if (ch < d8) {
      hdet_f8 o;
#pragma unroll
      for (int j = 0; j < 8; ++j) o.v[j] = rs * (dxh[i].v[j] - m1 - xh[i].v[j] * m2);
      if (resid) {
        const hdet_f8 rv = hdet_ld8(resid + base + 8 * ch);
#pragma unroll
        for (int j = 0; j < 8; ++j) o.v[j] += rv.v[j];
      }
      hdet_st8(dx + base + 8 * ch, o);
    }
  }
}

// Dropout of a residual branch.  Element e of the replica's [M][d] tensor is kept iff word
// (e mod 4) of philox(counter = (e div 4, step, replica * 65536 + site, kDropStream), key = seed)
// is >= floor(p * 2^32).  A thread handles the four elements of one Philox block.
struct drop_args {
  const hdet_ctrl* ctrl;
  int channel;          // dropout channel index or -1 (no dropout)
  uint32_t step, seed_lo, seed_hi;
  int site;
};

__device__ __forceinline__ void drop_setup(const drop_args& da, int r, uint32_t* thresh, float* keep_scale) {
  float p = 0.f;
  if (da.channel >= 0) p = (float)hdet_channel_value(da.ctrl, da.channel, r, 0.0);
  *thresh = (uint32_t)floor((double)p * 4294967296.0);
  *keep_scale = 1.f / (1.f - p);
}

// LayerNorm backward with the parameter gradients' stage 1 fused in: block = kLnRows consecutive
// rows of a replica, wavefront w takes rows w, w+4, ... (one or two in flight), writes dx like the
// kernel above and keeps, per column it holds, sum dy xhat and sum dy over its rows in ascending
// order; the four wavefronts' sums are added in the order w = 0..3 and written as row chunk
// blockIdx.x of part[replica][row chunk][col] (sum dy: a second array right behind the first).
constexpr int kLnRows = 32;
template <typename T, int NCH>
__global__ __launch_bounds__(256) void ln_bwd_fused_kernel(const T* dy, const T* x, const float* mean, const float* rstd,
                                                           const float* theta, int64_t ps, int64_t g_off, int M, int d,
                                                           const T* resid, T* dx, float* part, T* dropped, const drop_args da,
                                                           float* part_out) {
  __shared__ float l1[4][NCH * 512], l2[4][NCH * 512];
  uint32_t thresh = 0u;
  float ks = 1.f;
  if (dropped) drop_setup(da, blockIdx.y, &thresh, &ks);
  const int r = blockIdx.y, lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const float* g = theta + (int64_t)r * ps + g_off;
  const int d8 = d >> 3;
  hdet_f8 gv[NCH], ag[NCH], ab[NCH], ao[NCH];     // ao: column sums of what the next branch receives (dx, or dx dropped out), as stored
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int ch = lane + 64 * i;
#pragma unroll
    for (int j = 0; j < 8; ++j) { ag[i].v[j] = 0.f; ab[i].v[j] = 0.f; ao[i].v[j] = 0.f; gv[i].v[j] = 0.f; }
    if (ch < d8) gv[i] = hdet_ld8(g + 8 * ch);
  }
  const int row0 = blockIdx.x * kLnRows + w;
  constexpr int U = NCH == 1 ? 2 : 1;                 // rows in flight per wavefront, by register budget
  for (int it = 0; it < kLnRows / 4; it += U) {
    hdet_f8 dyv[U][NCH], xh[U][NCH];
    float mu[U], rs[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int row = row0 + 4 * (it + u);
      if (row < M) {
        const int64_t base = ((int64_t)r * M + row) * d;
        mu[u] = mean[(int64_t)r * M + row];
        rs[u] = rstd[(int64_t)r * M + row];
#pragma unroll
        for (int i = 0; i < NCH; ++i)
          if (lane + 64 * i < d8) { dyv[u][i] = hdet_ld8(dy + base + 8 * (lane + 64 * i)); xh[u][i] = hdet_ld8(x + base + 8 * (lane + 64 * i)); }
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int row = row0 + 4 * (it + u);
      if (row >= M) continue;                         // uniform over the wavefront
      const int64_t base = ((int64_t)r * M + row) * d;
      hdet_f8 rv[NCH];                                // in flight while the row's sums are formed
      if (resid) {
#pragma unroll
        for (int i = 0; i < NCH; ++i)
          if (lane + 64 * i < d8) rv[i] = hdet_ld8(resid + base + 8 * (lane + 64 * i));
      }
      float s1 = 0.f, s2 = 0.f;
#pragma unroll
      for (int i = 0; i < NCH; ++i)
        if (lane + 64 * i < d8) {
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const float dyj = dyv[u][i].v[j];
            xh[u][i].v[j] = (xh[u][i].v[j] - mu[u]) * rs[u];
            ag[i].v[j] += dyj * xh[u][i].v[j];
            ab[i].v[j] += dyj;
            dyv[u][i].v[j] = dyj * gv[i].v[j];
            s1 += dyv[u][i].v[j];
            s2 += dyv[u][i].v[j] * xh[u][i].v[j];
          }
        }
      const float m1 = hdet_wave_sum(s1) / (float)d, m2 = hdet_wave_sum(s2) / (float)d;
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        const int ch = lane + 64 * i;
        if (ch < d8) {
          hdet_f8 o;
#pragma unroll
          for (int j = 0; j < 8; ++j) o.v[j] = rs[u] * (dyv[u][i].v[j] - m1 - xh[u][i].v[j] * m2);
          if (resid) {
#pragma unroll
            for (int j = 0; j < 8; ++j) o.v[j] += rv[i].v[j];
          }
          hdet_st8(dx + base + 8 * ch, o);
          if (part_out && !dropped) {
#pragma unroll
            for (int j = 0; j < 8; ++j) ao[i].v[j] += sizeof(T) == 2 ? __uint_as_float(hdet_bf16_bits(o.v[j]) << 16) : o.v[j];
          }
          if (dropped) {      // the gradient through the dropout of the branch below, from dx as it is stored
            const int64_t e = (int64_t)row * d + 8 * ch;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
              hdet_philox4 wd = {{0xffffffffu, 0xffffffffu, 0xffffffffu, 0xffffffffu}};
              if (thresh != 0u)
                wd = hdet_philox4x32_10((uint32_t)((e >> 2) + h), da.step, (uint32_t)r * 65536u + (uint32_t)da.site, kDropStream,
                                        da.seed_lo, da.seed_hi);
#pragma unroll
              for (int j = 0; j < 4; ++j) {
                const float stored = sizeof(T) == 2 ? __uint_as_float(hdet_bf16_bits(o.v[4 * h + j]) << 16) : o.v[4 * h + j];
                o.v[4 * h + j] = thresh == 0u ? stored : (wd.x[j] >= thresh ? stored * ks : 0.f);
              }
            }
            hdet_st8(dropped + base + 8 * ch, o);
            if (part_out) {
#pragma unroll
              for (int j = 0; j < 8; ++j) ao[i].v[j] += sizeof(T) == 2 ? __uint_as_float(hdet_bf16_bits(o.v[j]) << 16) : o.v[j];
            }
          }
        }
      }
    }
  }
#pragma unroll
  for (int i = 0; i < NCH; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) { l1[w][(lane + 64 * i) * 8 + j] = ag[i].v[j]; l2[w][(lane + 64 * i) * 8 + j] = ab[i].v[j]; }
  __syncthreads();
  const int64_t pbase = ((int64_t)r * gridDim.x + blockIdx.x) * d;
  const int64_t second = (int64_t)gridDim.y * gridDim.x * d;
  for (int c = threadIdx.x; c < d; c += 256) {
    part[pbase + c] = ((l1[0][c] + l1[1][c]) + l1[2][c]) + l1[3][c];
    part[second + pbase + c] = ((l2[0][c] + l2[1][c]) + l2[2][c]) + l2[3][c];
  }
  if (part_out) {
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NCH; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j) l1[w][(lane + 64 * i) * 8 + j] = ao[i].v[j];
    __syncthreads();
    for (int c = threadIdx.x; c < d; c += 256) part_out[pbase + c] = ((l1[0][c] + l1[1][c]) + l1[2][c]) + l1[3][c];
  }
}

// Two-stage column reduction for cols % 8 == 0: stage 1, block (512 columns x rows_per_block
// rows x replica), wavefront w adds rows w, w+4, ... of the chunk (loaded eight rows at a time,
// added in ascending order), the four partial sums are added in the order w = 0..3 and written
// to part[replica][row chunk][col] (MODE 1: a second array of the same shape right behind the
// first); stage 2, once per backward pass for all reductions together, adds the row chunks in
// ascending order.  Same two modes as colsum_kernel.
template <typename T, int MODE>
__global__ __launch_bounds__(256) void colsum_part_kernel(const T* src, int64_t src_rs, int64_t src_bs, int M, int cols,
                                                          int rows_per_block, const T* x, const float* mean,
                                                          const float* rstd, float* part) {
  __shared__ float l1[4][512], l2[4][512];
  constexpr int U = 8;
  const int r = blockIdx.z, lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int col = blockIdx.x * 512 + lane * 8;
  const int m0 = blockIdx.y * rows_per_block;
  const int m1 = m0 + rows_per_block < M ? m0 + rows_per_block : M;
  float a1[8] = {0, 0, 0, 0, 0, 0, 0, 0}, a2[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if (col < cols) {
    for (int mb = m0 + w; mb < m1; mb += 4 * U) {
      hdet_f8 v[U], xv[U];
      float mu[U], rs[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int m = mb + 4 * u;
        if (m < m1) {
          v[u] = hdet_ld8(src + (int64_t)r * src_bs + (int64_t)m * src_rs + col);
          if (MODE == 1) {
            xv[u] = hdet_ld8(x + ((int64_t)r * M + m) * cols + col);
            mu[u] = mean[(int64_t)r * M + m];
            rs[u] = rstd[(int64_t)r * M + m];
          }
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (mb + 4 * u < m1) {
          if (MODE == 1) {
#pragma unroll
            for (int j = 0; j < 8; ++j) { a1[j] += v[u].v[j] * ((xv[u].v[j] - mu[u]) * rs[u]); a2[j] += v[u].v[j]; }
          } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) a1[j] += v[u].v[j];
          }
        }
    }
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) { l1[w][lane * 8 + j] = a1[j]; l2[w][lane * 8 + j] = a2[j]; }
  __syncthreads();
  const int64_t pbase = ((int64_t)r * gridDim.y + blockIdx.y) * cols;
  const int64_t second = (int64_t)gridDim.z * gridDim.y * cols;
  for (int c = threadIdx.x; c < 512; c += 256) {
    const int gc = blockIdx.x * 512 + c;
    if (gc < cols) {
      part[pbase + gc] = ((l1[0][c] + l1[1][c]) + l1[2][c]) + l1[3][c];
      if (MODE == 1) part[second + pbase + gc] = ((l2[0][c] + l2[1][c]) + l2[2][c]) + l2[3][c];
    }
  }
}

// Stage 2 of every two-stage column reduction of a backward pass in one launch.  Job j owns the
// blocks first_block .. of the grid's x range, 256 columns each; grid.y = replica.
struct colsum_job {
  int64_t part_off;       // floats from the head of the partial-sum area
  int64_t out_off;        // offset of the result inside a gradient plane (second result of MODE 1: out2_off)
  int64_t out2_off;
  int32_t cols, mode, first_block, nchunks;   // nchunks: row chunks stage 1 produced
};
__global__ __launch_bounds__(256) void colsum_final_kernel(const colsum_job* jobs, int njobs, const float* part,
                                                           int n_replicas, float* grads, int64_t ps) {
  int lo = 0, hi = njobs - 1;                       // last job whose first block is <= blockIdx.x
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (jobs[mid].first_block <= (int)blockIdx.x) lo = mid; else hi = mid - 1;
  }
  const colsum_job j = jobs[lo];
  const int nchunks = j.nchunks;
  const int r = blockIdx.y, c = (blockIdx.x - j.first_block) * 256 + threadIdx.x;
  if (c >= j.cols) return;
  // chunks added in ascending order, eight loads in flight
  auto total = [&](const float* q) {
    float a = 0.f;
    for (int k = 0; k < nchunks; k += 8) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = k + u < nchunks ? q[(int64_t)(k + u) * j.cols] : 0.f;
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (k + u < nchunks) a += v[u];
    }
    return a;
  };
  const float* p1 = part + j.part_off + (int64_t)r * nchunks * j.cols + c;
  grads[(int64_t)r * ps + j.out_off + c] = total(p1);
  if (j.mode == 1) grads[(int64_t)r * ps + j.out2_off + c] = total(p1 + (int64_t)n_replicas * nchunks * j.cols);
}

// Column reductions over the M rows: block = 64 columns x 16 row phases; thread (c, q) adds
// rows q, q+16, ... in ascending order, the 16 partial sums are then added in the order q = 0..15.
//   MODE 0: out[c]  = sum_m src[m][c]                                   (bias gradients)
//   MODE 1: out[c]  = sum_m src[m][c] * xhat[m][c],  out2[c] = sum_m src[m][c]   (LayerNorm g, b)
template <typename T, int MODE>
__global__ __launch_bounds__(1024) void colsum_kernel(const T* src, int64_t src_rs, int64_t src_bs, int M, int cols,
                                                      const T* x, const float* mean, const float* rstd,
                                                      float* out, float* out2, int64_t out_bs) {
  __shared__ float p1[16][64], p2[16][64];
  const int r = blockIdx.y, c = threadIdx.x & 63, q = threadIdx.x >> 6;
  const int col = blockIdx.x * 64 + c;
  float s1 = 0.f, s2 = 0.f;
  if (col < cols) {
    for (int m = q; m < M; m += 16) {
      const float v = hdet_ld(src + (int64_t)r * src_bs + (int64_t)m * src_rs + col);
      if (MODE == 1) {
        const float xh = (hdet_ld(x + ((int64_t)r * M + m) * cols + col) - mean[(int64_t)r * M + m]) * rstd[(int64_t)r * M + m];
        s1 += v * xh;
        s2 += v;
      } else {
        s1 += v;
      }
    }
  }
  p1[q][c] = s1; p2[q][c] = s2;
  __syncthreads();
  if (q == 0 && col < cols) {
    float a = 0.f, b = 0.f;
    for (int i = 0; i < 16; ++i) { a += p1[i][c]; b += p2[i][c]; }
    out[(int64_t)r * out_bs + col] = a;
    if (MODE == 1) out2[(int64_t)r * out_bs + col] = b;
  }
}

// Score scale of the replica that owns `row`: 1 / sqrt(d_head), divided by the replica's
// attention temperature when that is an explored channel (Remark 1).
struct temp_args { const hdet_ctrl* ctrl; int channel; int64_t rows_per_replica; };
__device__ __forceinline__ float score_scale(float scale, const temp_args& t, int64_t row) {
  return t.channel >= 0 ? scale / (float)hdet_channel_value(t.ctrl, t.channel, (int)(row / t.rows_per_replica), 0.0) : scale;
}

// Causal softmax over scaled scores, one wavefront per query row i: keys j <= i.
template <typename T>
__global__ __launch_bounds__(256) void softmax_fwd_kernel(const float* scores, int64_t rows_total, int S, float scale0, temp_args ta, T* p) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows_total) return;
  const float scale = score_scale(scale0, ta, row);
  const int i = (int)(row % S);
  const float* s = scores + row * S;
  float mx = -INFINITY;
  for (int j = lane; j <= i; j += 64) mx = fmaxf(mx, s[j] * scale);
  mx = hdet_wave_max(mx);
  float se = 0.f;
  for (int j = lane; j <= i; j += 64) se += expf(s[j] * scale - mx);
  const float inv = 1.f / hdet_wave_sum(se);
  for (int j = lane; j < S; j += 64) hdet_st(p + row * S + j, j <= i ? expf(s[j] * scale - mx) * inv : 0.f);
}

// ds = p * (dp - sum_j dp_j p_j) * scale  (zero above the diagonal, where p = 0)
template <typename T>
__global__ __launch_bounds__(256) void softmax_bwd_kernel(const float* dp, const T* p, int64_t rows_total, int S,
                                                          float scale0, temp_args ta, T* ds) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows_total) return;
  const float scale = score_scale(scale0, ta, row);
  const int i = (int)(row % S);
  float dot = 0.f;
  for (int j = lane; j <= i; j += 64) dot += dp[row * S + j] * hdet_ld(p + row * S + j);
  dot = hdet_wave_sum(dot);
  for (int j = lane; j < S; j += 64)
    hdet_st(ds + row * S + j, j <= i ? hdet_ld(p + row * S + j) * (dp[row * S + j] - dot) * scale : 0.f);
}

// Vector forms for S % 4 == 0, S <= 1024: lane l owns the 4-element chunks l, l + 64, ... of a row.
template <typename T, int NCH>
__global__ __launch_bounds__(256) void softmax_fwd_vec_kernel(const float* scores, int64_t rows_total, int S, float scale0, temp_args ta, T* p) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows_total) return;
  const float scale = score_scale(scale0, ta, row);
  const int i = (int)(row % S), s4 = S >> 2;
  hdet_f4 v[NCH];
  float mx = -INFINITY;
#pragma unroll
  for (int k = 0; k < NCH; ++k) {
    const int ch = lane + 64 * k;
    if (ch < s4) {
      v[k] = hdet_ld4(scores + row * S + 4 * ch);
#pragma unroll
      for (int j = 0; j < 4; ++j) { v[k].v[j] *= scale; if (4 * ch + j <= i) mx = fmaxf(mx, v[k].v[j]); }
    }
  }
  mx = hdet_wave_max(mx);
  float se = 0.f;
#pragma unroll
  for (int k = 0; k < NCH; ++k) {
    const int ch = lane + 64 * k;
    if (ch < s4) {
#pragma unroll
      for (int j = 0; j < 4; ++j) { v[k].v[j] = 4 * ch + j <= i ? expf(v[k].v[j] - mx) : 0.f; se += v[k].v[j]; }
    }
  }
  const float inv = 1.f / hdet_wave_sum(se);
#pragma unroll
  for (int k = 0; k < NCH; ++k) {
    const int ch = lane + 64 * k;
    if (ch < s4) {
#pragma unroll
      for (int j = 0; j < 4; ++j) v[k].v[j] *= inv;
      hdet_st4(p + row * S + 4 * ch, v[k]);
    }
  }
}

template <typename T, int NCH>
__global__ __launch_bounds__(256) void softmax_bwd_vec_kernel(const float* dp, const T* p, int64_t rows_total, int S,
                                                              float scale0, temp_args ta, T* ds) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows_total) return;
  const float scale = score_scale(scale0, ta, row);
  const int s4 = S >> 2;
  hdet_f4 dv[NCH], pv[NCH];
  float dot = 0.f;
#pragma unroll
  for (int k = 0; k < NCH; ++k) {
    const int ch = lane + 64 * k;
    if (ch < s4) {
      dv[k] = hdet_ld4(dp + row * S + 4 * ch);
      pv[k] = hdet_ld4(p + row * S + 4 * ch);          // zero above the diagonal
#pragma unroll
      for (int j = 0; j < 4; ++j) dot += dv[k].v[j] * pv[k].v[j];
    }
  }
  dot = hdet_wave_sum(dot);
#pragma unroll
  for (int k = 0; k < NCH; ++k) {
    const int ch = lane + 64 * k;
    if (ch < s4) {
      hdet_f4 o;
#pragma unroll
      for (int j = 0; j < 4; ++j) o.v[j] = pv[k].v[j] * (dv[k].v[j] - dot) * scale;
      hdet_st4(ds + row * S + 4 * ch, o);
    }
  }
}


// 8 elements per thread and access; the n % 8 tail is done element-wise by the first threads
template <typename T>
__global__ __launch_bounds__(256) void gelu_fwd_kernel(const T* z, T* f, int64_t n) {
  const int64_t n8 = n >> 3, tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  for (int64_t i = tid; i < n8; i += (int64_t)gridDim.x * 256) {
    hdet_f8 v = hdet_ld8(z + 8 * i);
#pragma unroll
    for (int j = 0; j < 8; ++j) v.v[j] = hdet_gelu_tanh(v.v[j]);
    hdet_st8(f + 8 * i, v);
  }
  if (tid < (n & 7)) hdet_st(f + 8 * n8 + tid, hdet_gelu_tanh(hdet_ld(z + 8 * n8 + tid)));
}
template <typename T>
__global__ __launch_bounds__(256) void gelu_bwd_kernel(const T* df, const T* z, T* dz, int64_t n) {
  const int64_t n8 = n >> 3, tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  for (int64_t i = tid; i < n8; i += (int64_t)gridDim.x * 256) {
    hdet_f8 v = hdet_ld8(df + 8 * i);
    const hdet_f8 zv = hdet_ld8(z + 8 * i);
#pragma unroll
    for (int j = 0; j < 8; ++j) v.v[j] *= hdet_gelu_tanh_grad(zv.v[j]);
    hdet_st8(dz + 8 * i, v);
  }
  if (tid < (n & 7)) hdet_st(dz + 8 * n8 + tid, hdet_ld(df + 8 * n8 + tid) * hdet_gelu_tanh_grad(hdet_ld(z + 8 * n8 + tid)));
}

// out = x + drop(branch)            (ADD)        forward residual add
// out = drop'(branch) = branch * keep / (1-p)    backward through the dropout
template <typename T, bool ADD>
__global__ __launch_bounds__(256) void dropout_kernel(const T* x, const T* branch, T* out, int64_t n, const drop_args da) {
  const int r = blockIdx.y;
  uint32_t thresh; float ks;
  drop_setup(da, r, &thresh, &ks);
  const int64_t nblk = n >> 2;
  for (int64_t b = (int64_t)blockIdx.x * 256 + threadIdx.x; b < nblk; b += (int64_t)gridDim.x * 256) {
    hdet_philox4 w = {{0xffffffffu, 0xffffffffu, 0xffffffffu, 0xffffffffu}};
    if (thresh != 0u)
      w = hdet_philox4x32_10((uint32_t)b, da.step, (uint32_t)r * 65536u + (uint32_t)da.site, kDropStream, da.seed_lo, da.seed_hi);
    const int64_t i = (int64_t)r * n + (b << 2);
    hdet_f4 v = hdet_ld4(branch + i);
    if (thresh != 0u) {
#pragma unroll
      for (int j = 0; j < 4; ++j) v.v[j] = w.x[j] >= thresh ? v.v[j] * ks : 0.f;
    }
    if (ADD) {
      const hdet_f4 xv = hdet_ld4(x + i);
#pragma unroll
      for (int j = 0; j < 4; ++j) v.v[j] += xv.v[j];
    }
    hdet_st4(out + i, v);
  }
}

int grid_for(int64_t n) { int64_t b = (n + 255) / 256; return (int)(b > 8192 ? 8192 : (b < 1 ? 1 : b)); }

}  // namespace

// xent and loss reduction live with the MLP path
hipError_t hdet_launch_xent(bool bf16, const float* logits, const int32_t* labels, int rows, int classes, void* dlogits,
                            float* row_loss, int n_replicas, const hdet_ctrl* ctrl, int ls_channel, hipStream_t s,
                            float* colsum = nullptr, int rows_per_block = 0, int grad_rows = 0);
bool hdet_xent_wide(int classes);
hipError_t hdet_launch_loss_reduce(const float* row_loss, int rows, hdet_ctrl* ctrl, int n_replicas, hipStream_t s);

// Rows per block of the wide-row loss kernel when it also forms stage 1 of the head bias gradient: enough rows
// to make the partial sums few, as long as about four blocks per compute unit remain; 0 = a separate pass does it.
static int xent_rows_per_block(int64_t M, int64_t N, int64_t V) {
  if (!hdet_xent_wide((int)V) || V % 8 != 0) return 0;
  const int64_t r = M * N / 1024;
  return r < 8 ? 0 : (int)(r > 64 ? 64 : r);
}

struct tf_block_off { int64_t ln1_g, ln1_b, w_qkv, b_qkv, w_o, b_o, ln2_g, ln2_b, w_1, b_1, w_2, b_2; };

struct hdet_tf_plan {
  hdet_config cfg;
  hdet_buffers buf;
  bool bf16;
  int N, B, S, M, d, nh, dh, ff, V, L;
  int drop_channel;
  int ls_channel;       // label-smoothing channel or -1
  int temp_channel;     // attention-temperature channel or -1
  int64_t tok, pos, lnf_g, lnf_b, w_head, b_head;
  std::vector<tf_block_off> blk;
  // activations (type T), per replica sizes in elements
  std::vector<char*> x_in, x_mid, h1, h2, qkv, p, a, z, f;   // [L] (+1 for x_in)
  std::vector<float*> st1_mean, st1_rstd, st2_mean, st2_rstd;
  char *hf, *tmp_d, *dxa, *dxb, *dtmp, *dtmp2, *dff, *dqkv, *ds, *dlogits;
  float *stf_mean, *stf_rstd, *scores, *logits, *row_loss;
  std::vector<float*> att_max, att_inv;      // [L] row statistics of the fused attention
  float* att_dot;
  unsigned long long* tok_sorted;            // [N][M] keys (token id, row) in ascending order
  float* tok_seg;                            // [N][M][d] partial rows of the token-embedding gradient
  bool fused_attn;                           // bf16, head size 64, S a multiple of 64
  float* part;               // partial column sums, one [N][row chunks][cols] array (two for LayerNorm) per reduction
  int nrc;                   // row chunks of the two-stage column sums
  std::vector<colsum_job> jobs;   // the two-stage reductions of a backward pass, by position in the parameter plane
  colsum_job* jobs_dev;
  int final_blocks;          // x extent of the stage-2 launch
  // shared-gradient mode: the weight matrices whose gradient is formed as one product over all replicas' rows
  // (offset, length), ascending; every other gradient is left per replica
  std::vector<std::pair<int64_t, int64_t>> summed;
};

static size_t al(size_t x) { return (x + 255) & ~(size_t)255; }

// Shared-gradient mode: a weight gradient dW [rows][cols] is formed as ONE product over the K = N M rows of all
// replicas when that product alone has enough 256 x 256 tiles to occupy the chip (the output head); a smaller matrix
// keeps one product per replica, K = M, whose N results are added up with the vector parameters' gradients.
static bool tf_wgrad_one_product(int64_t rows, int64_t cols) { return ((rows + 255) / 256) * ((cols + 255) / 256) >= 128; }

// Walks the workspace layout; with base == nullptr only the size is computed.
static size_t tf_carve(hdet_tf_plan* p, char* base) {
  const size_t e = p->bf16 ? 2 : 4;
  const size_t N = p->N, M = p->M, d = p->d, ff = p->ff, V = p->V, S = p->S;
  const size_t heads = (size_t)p->B * p->nh;
  size_t off = 0;
  auto take = [&](size_t bytes) { char* q = base ? base + off : nullptr; off += al(bytes); return q; };
  const int L = p->L;
  p->x_in.assign(L + 1, nullptr); p->x_mid.assign(L, nullptr); p->h1.assign(L, nullptr); p->h2.assign(L, nullptr);
  p->qkv.assign(L, nullptr); p->p.assign(L, nullptr); p->a.assign(L, nullptr); p->z.assign(L, nullptr); p->f.assign(L, nullptr);
  p->st1_mean.assign(L, nullptr); p->st1_rstd.assign(L, nullptr); p->st2_mean.assign(L, nullptr); p->st2_rstd.assign(L, nullptr);
  p->att_max.assign(L, nullptr); p->att_inv.assign(L, nullptr);
  for (int l = 0; l <= L; ++l) p->x_in[l] = take(N * M * d * e);
  for (int l = 0; l < L; ++l) {
    p->x_mid[l] = take(N * M * d * e); p->h1[l] = take(N * M * d * e); p->h2[l] = take(N * M * d * e);
    p->qkv[l] = take(N * M * 3 * d * e); p->p[l] = take(N * heads * S * S * e); p->a[l] = take(N * M * d * e);
    p->z[l] = take(N * M * ff * e); p->f[l] = take(N * M * ff * e);
    p->st1_mean[l] = (float*)take(N * M * 4); p->st1_rstd[l] = (float*)take(N * M * 4);
    p->st2_mean[l] = (float*)take(N * M * 4); p->st2_rstd[l] = (float*)take(N * M * 4);
    p->att_max[l] = (float*)take(N * heads * S * 4); p->att_inv[l] = (float*)take(N * heads * S * 4);
  }
  p->hf = take(N * M * d * e); p->tmp_d = take(N * M * d * e);
  p->dxa = take(N * M * d * e); p->dxb = take(N * M * d * e); p->dtmp = take(N * M * d * e); p->dtmp2 = take(N * M * d * e);
  p->dff = take(N * M * ff * e); p->dqkv = take(N * M * 3 * d * e); p->ds = take(N * heads * S * S * e);
  p->dlogits = take(N * M * V * e);
  p->stf_mean = (float*)take(N * M * 4); p->stf_rstd = (float*)take(N * M * 4);
  p->scores = (float*)take(N * heads * S * S * 4); p->logits = (float*)take(N * M * V * 4);
  p->row_loss = (float*)take(N * M * 4);
  p->att_dot = (float*)take(N * heads * S * 4);
  p->tok_sorted = (unsigned long long*)take(N * M * 8);
  p->tok_seg = (float*)take(N * M * d * 4);
  p->nrc = (int)((M + kColsumRows - 1) / kColsumRows);
  // per block: biases of the four Linear layers (3d + d + ff + d columns) and two LayerNorms (2 x 2d); then final LayerNorm, head bias
  // (the LayerNorm pairs in chunks of kLnRows rows when their backward kernel produces them itself)
  const size_t ln_chunks = (M + kLnRows - 1) / kLnRows;
  const int xr = xent_rows_per_block(M, N, V);
  const size_t head_chunks = xr ? (M + xr - 1) / xr : p->nrc;
  p->part = (float*)take(N * (p->nrc * ((size_t)L * (3 * d + ff)) + head_chunks * V + ln_chunks * (2 * d * (2 * (size_t)L + 1) + 2 * d * (size_t)L)) * 4);
  p->jobs_dev = (colsum_job*)take((6 * (size_t)L + 2) * sizeof(colsum_job));
  return off;
}

static void tf_dims(hdet_tf_plan* p, const hdet_config& cfg) {
  p->cfg = cfg;
  p->bf16 = cfg.precision == HDET_BF16_GEMM_FP32_MASTER;
  p->N = cfg.n_replicas; p->B = cfg.dims.batch; p->S = cfg.dims.seq_len; p->M = p->B * p->S;
  p->d = cfg.dims.d_model; p->nh = cfg.dims.n_heads; p->dh = p->d / p->nh; p->ff = cfg.dims.d_ff;
  p->V = cfg.dims.vocab; p->L = cfg.dims.n_blocks;
  p->fused_attn = p->bf16 && hdet_attn_fusable(p->S, p->d, p->nh, p->B);
}

int64_t hdet_tf_param_count(const hdet_config& cfg) {
  const int64_t d = cfg.dims.d_model, ff = cfg.dims.d_ff, V = cfg.dims.vocab, S = cfg.dims.seq_len, L = cfg.dims.n_blocks;
  return V * d + S * d + L * (2 * d + 3 * d * d + 3 * d + d * d + d + 2 * d + ff * d + ff + d * ff + d) + 2 * d + V * d + V;
}

int hdet_tf_validate(const hdet_config& cfg, std::string* err) {
  const hdet_model_dims& m = cfg.dims;
  if (m.n_blocks < 1 || m.n_blocks > 64 || m.d_model < 4 || m.n_heads < 1 || m.d_ff < 1 || m.seq_len < 1 || m.vocab < 2 || m.batch < 1) {
    *err = "transformer dimensions out of range"; return HDET_EINVAL;
  }
  if (m.d_model % m.n_heads != 0) { *err = "d_model must be a multiple of n_heads"; return HDET_EINVAL; }
  if (m.d_model % 4 != 0) { *err = "d_model must be a multiple of 4"; return HDET_EINVAL; }
  return HDET_OK;
}

int hdet_tf_workspace_bytes(const hdet_config& cfg, size_t* bytes, std::string* err) {
  int rc = hdet_tf_validate(cfg, err);
  if (rc != HDET_OK) return rc;
  hdet_tf_plan p;
  tf_dims(&p, cfg);
  *bytes = tf_carve(&p, nullptr);
  return HDET_OK;
}

// whether the LayerNorm with its gain at g_off takes the vector kernels, and whether its backward kernel
// also produces stage 1 of the parameter gradients (up to d = 1024: beyond, the registers that takes
// cost more than the separate reduction)
static bool hdet_tf_ln_vector(const hdet_tf_plan* p, int64_t g_off) {
  return p->d % 8 == 0 && p->d <= 2048 && g_off % 4 == 0 && p->buf.plane_stride % 4 == 0;
}
static bool hdet_tf_ln_fused(const hdet_tf_plan* p, int64_t g_off) { return hdet_tf_ln_vector(p, g_off) && p->d <= 1024; }

hdet_tf_plan* hdet_tf_create(const hdet_config& cfg, const hdet_buffers& buf, int drop_channel, int ls_channel,
                             int temp_channel, std::string* err) {
  if (hdet_tf_validate(cfg, err) != HDET_OK) return nullptr;
  hdet_tf_plan* p = new hdet_tf_plan();
  tf_dims(p, cfg);
  p->buf = buf;
  p->drop_channel = drop_channel;
  p->ls_channel = ls_channel;
  p->temp_channel = temp_channel;
  const size_t need = tf_carve(p, nullptr);
  if (!buf.workspace_dev || buf.workspace_bytes < need) { *err = "workspace_dev is too small"; delete p; return nullptr; }
  tf_carve(p, (char*)buf.workspace_dev);
  const int64_t d = p->d, ff = p->ff, V = p->V, S = p->S;
  int64_t off = 0;
  p->tok = off; off += V * d;
  p->pos = off; off += S * d;
  for (int l = 0; l < p->L; ++l) {
    tf_block_off b;
    b.ln1_g = off; off += d; b.ln1_b = off; off += d;
    b.w_qkv = off; off += 3 * d * d; b.b_qkv = off; off += 3 * d;
    b.w_o = off; off += d * d; b.b_o = off; off += d;
    b.ln2_g = off; off += d; b.ln2_b = off; off += d;
    b.w_1 = off; off += ff * d; b.b_1 = off; off += ff;
    b.w_2 = off; off += d * ff; b.b_2 = off; off += d;
    p->blk.push_back(b);
  }
  p->lnf_g = off; off += d; p->lnf_b = off; off += d;
  p->w_head = off; off += V * d; p->b_head = off; off += V;
  // stage 2 of the column reductions: one job per bias vector and LayerNorm parameter pair
  int64_t part_off = 0;
  int first_block = 0;
  // producer_g: for the bias of an output projection, the gain offset of the LayerNorm whose backward kernel
  // produces that bias gradient's input (and, when it is of the fused kind, stage 1 of its column sum); -1 otherwise
  auto add_job = [&](int cols, int mode, int64_t out_off, int64_t out2_off, int64_t producer_g = -1, int chunks = 0) {
    if (cols % 8 != 0) return;                       // such widths take the single-stage kernel
    const bool by_ln = (mode == 1 && hdet_tf_ln_fused(p, out_off)) || (producer_g >= 0 && hdet_tf_ln_fused(p, producer_g));
    const int nchunks = chunks ? chunks : by_ln ? (p->M + kLnRows - 1) / kLnRows : p->nrc;
    colsum_job j = {part_off, out_off, out2_off, cols, mode, first_block, nchunks};
    p->jobs.push_back(j);
    part_off += (int64_t)(mode == 1 ? 2 : 1) * p->N * nchunks * cols;
    first_block += (cols + 255) / 256;
  };
  const int xr = xent_rows_per_block(p->M, p->N, V);
  add_job((int)V, 0, p->b_head, 0, -1, xr ? (p->M + xr - 1) / xr : 0);
  add_job((int)d, 1, p->lnf_g, p->lnf_b);
  for (int l = 0; l < p->L; ++l) {
    const tf_block_off& b = p->blk[l];
    add_job((int)d, 0, b.b_2, 0, l + 1 < p->L ? p->blk[l + 1].ln1_g : p->lnf_g);
    add_job((int)ff, 0, b.b_1, 0);
    add_job((int)d, 1, b.ln2_g, b.ln2_b);
    add_job((int)d, 0, b.b_o, 0, b.ln2_g);
    add_job(3 * (int)d, 0, b.b_qkv, 0);
    add_job((int)d, 1, b.ln1_g, b.ln1_b);
  }
  p->final_blocks = first_block;
  if (cfg.grad_mode == HDET_GRAD_SHARED) {
    for (int l = 0; l < p->L; ++l) {
      const tf_block_off& o = p->blk[l];
      if (tf_wgrad_one_product(3 * d, d)) p->summed.push_back({o.w_qkv, 3 * d * d});
      if (tf_wgrad_one_product(d, d)) p->summed.push_back({o.w_o, d * d});
      if (tf_wgrad_one_product(ff, d)) p->summed.push_back({o.w_1, ff * d});
      if (tf_wgrad_one_product(d, ff)) p->summed.push_back({o.w_2, d * ff});
    }
    if (tf_wgrad_one_product(V, d)) p->summed.push_back({p->w_head, V * d});
  }
  // on the handle's stream, like all other work; the host copy lives as long as the plan
  if (!p->jobs.empty() &&
      hipMemcpyAsync(p->jobs_dev, p->jobs.data(), p->jobs.size() * sizeof(colsum_job), hipMemcpyHostToDevice,
                     (hipStream_t)cfg.stream) != hipSuccess) {
    *err = "could not upload the column-reduction table"; delete p; return nullptr;
  }
  return p;
}

void hdet_tf_destroy(hdet_tf_plan* p) { delete p; }

void hdet_tf_summed_slices(const hdet_tf_plan* p, std::vector<std::pair<int64_t, int64_t>>* out) { *out = p->summed; }

void hdet_tf_set_fused_attention(hdet_tf_plan* p, bool on) {
  p->fused_attn = on && p->bf16 && hdet_attn_fusable(p->S, p->d, p->nh, p->B);
}

namespace {

// ---- launch helpers: vector kernels where the shape allows, element-wise ones otherwise ----
#define HDET_NCH_SWITCH(nch, CALL) \
  switch (nch) { case 1: CALL(1); break; case 2: CALL(2); break; case 3: CALL(3); break; default: CALL(4); break; }

template <typename T>
void launch_ln_fwd(const hdet_tf_plan* p, const void* x, int64_t g_off, int64_t b_off, void* y, float* mean, float* rstd, hipStream_t s) {
  const int M = p->M, d = p->d;
  const int64_t ps = p->buf.plane_stride;
  const float* theta = p->buf.params_dev;
  const dim3 grid((M + 3) / 4, p->N);
  if (d % 8 == 0 && d <= 2048 && g_off % 4 == 0 && b_off % 4 == 0 && ps % 4 == 0) {
    const int nch = (d / 8 + 63) / 64;
#define CALL(K) hipLaunchKernelGGL((ln_fwd_vec_kernel<T, K>), grid, dim3(256), 0, s, (const T*)x, theta, ps, g_off, b_off, M, d, (T*)y, mean, rstd)
    HDET_NCH_SWITCH(nch, CALL)
#undef CALL
  } else {
    hipLaunchKernelGGL(ln_fwd_kernel<T>, grid, dim3(256), 0, s, (const T*)x, theta, ps, g_off, b_off, M, d, (T*)y, mean, rstd);
  }
}

// dx of a LayerNorm (plus `resid`); true when the launch also produced stage 1 of the parameter gradients
template <typename T>
bool launch_ln_bwd_dx(const hdet_tf_plan* p, const void* dy, const void* x, const float* mean, const float* rstd, int64_t g_off,
                      const void* resid, void* dx, hipStream_t s, void* dropped = nullptr, const drop_args* da = nullptr,
                      bool* dropped_done = nullptr, int64_t next_bias_off = -1, bool* bias_done = nullptr) {
  const int M = p->M, d = p->d;
  const int64_t ps = p->buf.plane_stride;
  const float* theta = p->buf.params_dev;
  if (hdet_tf_ln_vector(p, g_off)) {
    const colsum_job* job = nullptr;
    if (hdet_tf_ln_fused(p, g_off))
      for (const colsum_job& j : p->jobs)
        if (j.out_off == g_off && j.mode == 1) { job = &j; break; }
    const int nch = (d / 8 + 63) / 64;
    if (job) {
      const dim3 grid(job->nchunks, p->N);
      const drop_args none = {nullptr, -1, 0, 0, 0, 0};
      const bool with_drop = dropped && da;
      // stage 1 of the bias gradient of the output projection that receives this kernel's output
      float* part_out = nullptr;
      if (next_bias_off >= 0)
        for (const colsum_job& j : p->jobs)
          if (j.out_off == next_bias_off && j.mode == 0 && j.cols == d && j.nchunks == job->nchunks) { part_out = p->part + j.part_off; break; }
      if (bias_done) *bias_done = part_out != nullptr;
#define CALL(K) hipLaunchKernelGGL((ln_bwd_fused_kernel<T, K>), grid, dim3(256), 0, s, (const T*)dy, (const T*)x, mean, rstd, theta, ps, g_off, M, d, (const T*)resid, (T*)dx, p->part + job->part_off, with_drop ? (T*)dropped : (T*)nullptr, with_drop ? *da : none, part_out)
      if (nch == 1) CALL(1); else CALL(2);
#undef CALL
      if (dropped_done) *dropped_done = with_drop;
      return true;
    }
    const dim3 grid((M + 3) / 4, p->N);
#define CALL(K) hipLaunchKernelGGL((ln_bwd_dx_vec_kernel<T, K>), grid, dim3(256), 0, s, (const T*)dy, (const T*)x, mean, rstd, theta, ps, g_off, M, d, (const T*)resid, (T*)dx)
    HDET_NCH_SWITCH(nch, CALL)
#undef CALL
  } else {
    const dim3 grid((M + 3) / 4, p->N);
    hipLaunchKernelGGL(ln_bwd_dx_kernel<T>, grid, dim3(256), 0, s, (const T*)dy, (const T*)x, mean, rstd, theta, ps, g_off, M, d, (const T*)resid, (T*)dx);
  }
  return false;
}

template <typename T>
void launch_softmax_fwd(const float* scores, int64_t rows, int S, float scale, temp_args ta, void* prob, hipStream_t s) {
  const dim3 grid((unsigned)((rows + 3) / 4));
  if (S % 4 == 0 && S <= 1024) {
    const int nch = (S / 4 + 63) / 64;
#define CALL(K) hipLaunchKernelGGL((softmax_fwd_vec_kernel<T, K>), grid, dim3(256), 0, s, scores, rows, S, scale, ta, (T*)prob)
    HDET_NCH_SWITCH(nch, CALL)
#undef CALL
  } else {
    hipLaunchKernelGGL(softmax_fwd_kernel<T>, grid, dim3(256), 0, s, scores, rows, S, scale, ta, (T*)prob);
  }
}

template <typename T>
void launch_softmax_bwd(const float* dp, const void* prob, int64_t rows, int S, float scale, temp_args ta, void* ds, hipStream_t s) {
  const dim3 grid((unsigned)((rows + 3) / 4));
  if (S % 4 == 0 && S <= 1024) {
    const int nch = (S / 4 + 63) / 64;
#define CALL(K) hipLaunchKernelGGL((softmax_bwd_vec_kernel<T, K>), grid, dim3(256), 0, s, dp, (const T*)prob, rows, S, scale, ta, (T*)ds)
    HDET_NCH_SWITCH(nch, CALL)
#undef CALL
  } else {
    hipLaunchKernelGGL(softmax_bwd_kernel<T>, grid, dim3(256), 0, s, dp, (const T*)prob, rows, S, scale, ta, (T*)ds);
  }
}

// Column reductions described at colsum_kernel into the gradient plane offsets out_off (and out2_off),
// per replica.  Widths that are multiples of 8 only run stage 1 here; launch_colsum_final ends the pass.
template <typename T, int MODE>
hipError_t launch_colsum(const hdet_tf_plan* p, const void* src, int cols, const void* x, const float* mean, const float* rstd,
                         int64_t out_off, int64_t out2_off, hipStream_t s) {
  const int M = p->M, N = p->N;
  const int64_t ps = p->buf.plane_stride;
  float* grads = p->buf.grads_dev;
  if (cols % 8 == 0) {
    const colsum_job* job = nullptr;
    for (const colsum_job& j : p->jobs)
      if (j.out_off == out_off && j.cols == cols && j.mode == MODE) { job = &j; break; }
    if (!job) return hipErrorInvalidValue;
    hipLaunchKernelGGL((colsum_part_kernel<T, MODE>), dim3((cols + 511) / 512, job->nchunks, N), dim3(256), 0, s, (const T*)src, (int64_t)cols,
                       (int64_t)M * cols, M, cols, (M + job->nchunks - 1) / job->nchunks, (const T*)x, mean, rstd, p->part + job->part_off);
  } else {
    hipLaunchKernelGGL((colsum_kernel<T, MODE>), dim3((cols + 63) / 64, N), dim3(1024), 0, s, (const T*)src, (int64_t)cols, (int64_t)M * cols, M, cols,
                       (const T*)x, mean, rstd, grads + out_off, grads + out2_off, ps);
  }
  return hipGetLastError();
}

hipError_t launch_colsum_final(const hdet_tf_plan* p, hipStream_t s) {
  if (p->jobs.empty()) return hipSuccess;
  hipLaunchKernelGGL(colsum_final_kernel, dim3(p->final_blocks, p->N), dim3(256), 0, s, p->jobs_dev, (int)p->jobs.size(), p->part,
                     p->N, p->buf.grads_dev, p->buf.plane_stride);
  return hipGetLastError();
}

enum { NT = 0, NN = 1, TN = 2 };      // forward / dgrad / wgrad operand orders (see the GEMM files)

struct mat { const void* p; int64_t ld; int64_t s[3]; };

// C = A B in the given operand order; the output is of the activation type (act_out) or
// fp32; bias (fp32, per replica) is optional.  Element offsets inside `p` are in elements of
// the operand's own type.
// GELU fused into the bf16 GEMMs around it.  gelu_out: the product is the pre-activation z
// (written to c) and f = gelu(z) goes to gelu_out; gelu_pre: the product is the gradient at f and
// c receives the gradient at z = that * gelu'(gelu_pre).  `*fused` tells whether the GEMM took
// them (it does on the LDS-direct path); otherwise the caller runs the element-wise kernel.
// What a GEMM may fold into its epilogue when the fast bf16 kernel takes the product: the GELU after
// it (second output), the GELU gradient at the pre-activation, or the residual stream it is added to
// (the sum then goes to resid_out instead of c; with `drop`, the layer's output is dropped out first); with the GELU
// gradient, colsum_out receives stage 1 of the column sums of the result.  *fused tells the caller whether it happened.
struct gelu_fusion { void* gelu_out; const void* gelu_pre; bool* fused; const void* resid; void* resid_out; const drop_args* drop; float* colsum_out; };

template <typename T>
hipError_t gemm(const hdet_tf_plan* pl, int form, mat A, mat B, void* c, int64_t ldc, const int64_t* c_s, bool act_out,
                int m, int n, int k, int n1, int n2, const float* bias, int64_t bias_bs, hipStream_t s,
                const gelu_fusion* gf = nullptr, bool one_item = false) {
  // one_item: a single product instead of one per replica (the replicas' rows stacked along the contraction)
  const int batch = one_item ? 1 : pl->N * (n1 < 1 ? 1 : n1) * (n2 < 1 ? 1 : n2);
  if (gf) *gf->fused = false;
  if (sizeof(T) == 2) {
    hdet_bgemm_args g = {};
    g.a = (const uint16_t*)A.p; g.b = (const uint16_t*)B.p; g.c = c;
    g.m = m; g.n = n; g.k = k; g.n1 = n1 < 1 ? 1 : n1; g.n2 = n2 < 1 ? 1 : n2;
    g.lda = A.ld; g.ldb = B.ld; g.ldc = ldc;
    for (int i = 0; i < 3; ++i) { g.a_s[i] = A.s[i]; g.b_s[i] = B.s[i]; g.c_s[i] = c_s[i]; }
    g.bias = bias; g.bias_bs = bias_bs;
    int epi = act_out ? (bias ? HDET_EPI_BIAS_BF16 : HDET_EPI_BF16) : (bias ? HDET_EPI_BIAS_F32 : HDET_EPI_F32);
    if (gf && act_out) {
      hdet_bgemm_args f = g;
      int fepi;
      if (gf->gelu_out) { f.c2 = gf->gelu_out; fepi = HDET_EPI_BIAS_GELU_BF16; }
      else if (gf->resid) {
        f.c = gf->resid_out; f.mask = (const uint16_t*)gf->resid; f.mask_ld = ldc; f.mask_bs = c_s[0];
        fepi = HDET_EPI_BIAS_RESID_BF16;
        if (gf->drop) {
          fepi = HDET_EPI_BIAS_DROP_RESID_BF16;
          f.drop_ctrl = gf->drop->ctrl; f.drop_channel = gf->drop->channel; f.drop_step = gf->drop->step;
          f.drop_site = (uint32_t)gf->drop->site; f.drop_stream = kDropStream;
          f.drop_seed_lo = gf->drop->seed_lo; f.drop_seed_hi = gf->drop->seed_hi;
        }
      }
      else { f.mask = (const uint16_t*)gf->gelu_pre; f.mask_ld = ldc; f.mask_bs = c_s[0]; f.colsum = gf->colsum_out; fepi = HDET_EPI_GELUGRAD_BF16; }
      if ((fepi == HDET_EPI_GELUGRAD_BF16 || bias) && hdet_bgemm_dma_eligible(f, form != TN, form == NT, fepi)) {
        *gf->fused = true;
        return hdet_launch_bgemm(f, form != TN, form == NT, fepi, batch, s);
      }
    }
    return hdet_launch_bgemm(g, form != TN, form == NT, epi, batch, s);
  }
  hdet_sgemm_args g = {};
  g.a = (const float*)A.p; g.b = (const float*)B.p; g.c = (float*)c;
  g.m = m; g.n = n; g.k = k; g.n1 = n1; g.n2 = n2;
  if (form == TN) { g.a_rs = 1; g.a_cs = A.ld; } else { g.a_rs = A.ld; g.a_cs = 1; }
  if (form == NT) { g.b_rs = 1; g.b_cs = B.ld; } else { g.b_rs = B.ld; g.b_cs = 1; }
  g.c_rs = ldc;
  for (int i = 0; i < 3; ++i) { g.a_s[i] = A.s[i]; g.b_s[i] = B.s[i]; g.c_s[i] = c_s[i]; }
  g.bias = bias; g.bias_bs = bias_bs;
  return hdet_launch_sgemm(g, bias ? HDET_SEPI_BIAS : HDET_SEPI_NONE, batch, s);
}

#define TF_CHECK(expr) do { hipError_t e_ = (expr); if (e_ != hipSuccess) return e_; } while (0)

template <typename T>
hipError_t run(hdet_tf_plan* p, const int32_t* ids, const int32_t* targets, hdet_ctrl* ctrl, uint32_t step, hipStream_t s,
               const hdet_update_args* fuse, hdet_slices* fused) {
  const int N = p->N, M = p->M, S = p->S, d = p->d, ff = p->ff, V = p->V, L = p->L, nh = p->nh, dh = p->dh, B = p->B;
  const int64_t ps = p->buf.plane_stride;
  const float* theta = p->buf.params_dev;
  const T* wts = sizeof(T) == 2 ? (const T*)p->buf.params_bf16_dev : (const T*)p->buf.params_dev;
  float* grads = p->buf.grads_dev;
  const float scale = 1.f / sqrtf((float)dh);
  const int64_t heads_rows = (int64_t)N * B * nh * S;
  const int64_t nd = (int64_t)M * d, nff = (int64_t)M * ff;
  // Shared-gradient mode (Algorithm 1, "AllReduce gradients"): a large weight gradient (tf_wgrad_one_product) is formed as
  // one product over the K = N M rows of all replicas -- the sum of the replicas' gradients, in plane 0 of the gradient
  // buffer --, everything else per replica as usual; the update kernel turns both into the replica mean.
  const bool shared = p->cfg.grad_mode == HDET_GRAD_SHARED;
  drop_args da = {ctrl, p->drop_channel, step, (uint32_t)(p->cfg.seed & 0xffffffffu), (uint32_t)(p->cfg.seed >> 32), 0};
  const bool drop = p->drop_channel >= 0;
  const temp_args ta = {ctrl, p->temp_channel, (int64_t)B * nh * S};

  // batch strides: activations [N][M][w]; weights per replica plane; attention operands per (replica, sequence, head)
  auto act = [&](const void* q, int w) { mat t = {q, w, {(int64_t)M * w, 0, 0}}; return t; };
  auto wt = [&](int64_t off, int ld) { mat t = {wts + off, ld, {ps, 0, 0}}; return t; };
  auto qkv_part = [&](const void* base, int part) {      // q, k or v of head z2 in sequence z1: [S][dh], ld 3d
    mat t = {(const T*)base + (int64_t)part * d, 3 * (int64_t)d, {(int64_t)M * 3 * d, (int64_t)S * 3 * d, dh}};
    return t;
  };
  auto head_sq = [&](const void* base) {                  // [S][S] matrix of (replica, sequence, head)
    mat t = {base, S, {(int64_t)B * nh * S * S, (int64_t)nh * S * S, (int64_t)S * S}};
    return t;
  };
  auto head_cols = [&](const void* base) {                // columns of head z2 inside [M][d]
    mat t = {base, d, {(int64_t)M * d, (int64_t)S * d, dh}};
    return t;
  };
  auto attn_desc = [&](int l) {
    hdet_attn_desc ad;
    ad.qkv = (const uint16_t*)p->qkv[l]; ad.a = (uint16_t*)p->a[l]; ad.da = (const uint16_t*)p->dtmp; ad.dqkv = (uint16_t*)p->dqkv;
    ad.row_max = p->att_max[l]; ad.row_inv = p->att_inv[l]; ad.row_dot = p->att_dot;
    ad.ctrl = ctrl; ad.temp_channel = p->temp_channel; ad.scale = scale;
    ad.n_replicas = N; ad.batch = B; ad.seq_len = S; ad.heads = nh; ad.d_model = d;
    return ad;
  };
  const int64_t act_d[3] = {(int64_t)M * d, 0, 0}, act_3d[3] = {(int64_t)M * 3 * d, 0, 0}, act_ff[3] = {(int64_t)M * ff, 0, 0},
                act_v[3] = {(int64_t)M * V, 0, 0}, plane[3] = {ps, 0, 0};

  // ---- forward ------------------------------------------------------------------------
  hipLaunchKernelGGL(embed_fwd_kernel<T>, dim3(grid_for(nd), N), dim3(256), 0, s, theta, ps, p->tok, p->pos, ids, M, S, d, (T*)p->x_in[0]);
  for (int l = 0; l < L; ++l) {
    const tf_block_off& o = p->blk[l];
    launch_ln_fwd<T>(p, p->x_in[l], o.ln1_g, o.ln1_b, p->h1[l], p->st1_mean[l], p->st1_rstd[l], s);
    TF_CHECK(gemm<T>(p, NT, act(p->h1[l], d), wt(o.w_qkv, d), p->qkv[l], 3 * d, act_3d, true, M, 3 * d, d, 1, 1, theta + o.b_qkv, ps, s));
    if (p->fused_attn) {
      hdet_attn_desc ad = attn_desc(l);
      TF_CHECK(hdet_launch_attn_fwd(ad, s));
    } else {
      {   // scores = q k^T per (replica, sequence, head)
        const mat sc = head_sq(p->scores);
        TF_CHECK(gemm<T>(p, NT, qkv_part(p->qkv[l], 0), qkv_part(p->qkv[l], 1), p->scores, S, sc.s, false, S, S, dh, B, nh, nullptr, 0, s));
      }
      launch_softmax_fwd<T>(p->scores, heads_rows, S, scale, ta, p->p[l], s);
      {   // a = p v
        const mat ac = head_cols(p->a[l]);
        TF_CHECK(gemm<T>(p, NN, head_sq(p->p[l]), qkv_part(p->qkv[l], 2), p->a[l], d, ac.s, true, S, dh, S, B, nh, nullptr, 0, s));
      }
    }
    {   // x_mid = x_in + drop(a W_o^T + b_o), the sum (and the dropout) in the GEMM's epilogue where the fast kernel applies
      bool fused = false;
      da.site = 2 * l;
      const gelu_fusion rf = {nullptr, nullptr, &fused, p->x_in[l], p->x_mid[l], drop ? &da : nullptr, nullptr};
      TF_CHECK(gemm<T>(p, NT, act(p->a[l], d), wt(o.w_o, d), p->tmp_d, d, act_d, true, M, d, d, 1, 1, theta + o.b_o, ps, s, &rf));
      if (!fused)
        hipLaunchKernelGGL((dropout_kernel<T, true>), dim3(grid_for(nd / 4), N), dim3(256), 0, s, (const T*)p->x_in[l], (const T*)p->tmp_d, (T*)p->x_mid[l], nd, da);
    }
    launch_ln_fwd<T>(p, p->x_mid[l], o.ln2_g, o.ln2_b, p->h2[l], p->st2_mean[l], p->st2_rstd[l], s);
    {
      bool fused = false;
      const gelu_fusion gf = {p->f[l], nullptr, &fused, nullptr, nullptr, nullptr, nullptr};
      TF_CHECK(gemm<T>(p, NT, act(p->h2[l], d), wt(o.w_1, d), p->z[l], ff, act_ff, true, M, ff, d, 1, 1, theta + o.b_1, ps, s, &gf));
      if (!fused)
        hipLaunchKernelGGL(gelu_fwd_kernel<T>, dim3(grid_for((int64_t)N * nff)), dim3(256), 0, s, (const T*)p->z[l], (T*)p->f[l], (int64_t)N * nff);
    }
    {
      bool fused = false;
      da.site = 2 * l + 1;
      const gelu_fusion rf = {nullptr, nullptr, &fused, p->x_mid[l], p->x_in[l + 1], drop ? &da : nullptr, nullptr};
      TF_CHECK(gemm<T>(p, NT, act(p->f[l], ff), wt(o.w_2, ff), p->tmp_d, d, act_d, true, M, d, ff, 1, 1, theta + o.b_2, ps, s, &rf));
      if (!fused)
        hipLaunchKernelGGL((dropout_kernel<T, true>), dim3(grid_for(nd / 4), N), dim3(256), 0, s, (const T*)p->x_mid[l], (const T*)p->tmp_d, (T*)p->x_in[l + 1], nd, da);
    }
  }
  launch_ln_fwd<T>(p, p->x_in[L], p->lnf_g, p->lnf_b, p->hf, p->stf_mean, p->stf_rstd, s);
  TF_CHECK(gemm<T>(p, NT, act(p->hf, d), wt(p->w_head, d), p->logits, V, act_v, false, M, V, d, 1, 1, theta + p->b_head, ps, s));
  // the loss kernel for wide rows also forms stage 1 of the head bias gradient, xr rows per chunk
  float* head_part = nullptr;
  const int xr = xent_rows_per_block(M, N, V);
  if (xr)
    for (const colsum_job& j : p->jobs)
      if (j.out_off == p->b_head && j.mode == 0 && j.cols == V && j.nchunks == (M + xr - 1) / xr) { head_part = p->part + j.part_off; break; }
  TF_CHECK(hdet_launch_xent(sizeof(T) == 2, p->logits, targets, M, V, p->dlogits, p->row_loss, N, ctrl, p->ls_channel, s, head_part, xr));
  TF_CHECK(hdet_launch_loss_reduce(p->row_loss, M, ctrl, N, s));

  // ---- backward -----------------------------------------------------------------------
  auto colsum = [&](const void* src, int cols, int64_t out_off) {
    return launch_colsum<T, 0>(p, src, cols, nullptr, nullptr, nullptr, out_off, 0, s);
  };
  auto ln_params = [&](const void* dy, const void* x, const float* mean, const float* rstd, int64_t g_off, int64_t b_off) {
    return launch_colsum<T, 1>(p, dy, d, x, mean, rstd, g_off, b_off, s);
  };
  // Every weight gradient is formed after the input gradient of its layer (which reads the weights): with `fuse` the
  // product applies the update of W at once (Eq. 2) and dW never goes to memory.
  auto wgrad = [&](const void* dy, int wy, const void* x, int wx, int64_t w_off) -> hipError_t {      // dW[wy][wx] = dy^T x
    const bool one = shared && tf_wgrad_one_product(wy, wx);
    if (sizeof(T) == 2 && fuse && !shared) {
      hdet_bgemm_args g = {};
      g.a = (const uint16_t*)dy; g.lda = wy; g.a_s[0] = (int64_t)M * wy;
      g.b = (const uint16_t*)x; g.ldb = wx; g.b_s[0] = (int64_t)M * wx;
      g.ldc = wx; g.c_s[0] = ps;
      g.m = wy; g.n = wx; g.k = M; g.n1 = g.n2 = 1;
      if (hdet_fuse_args_for(p->cfg, *fuse, w_off, wy, wx, &g.upd) && hdet_bgemm_dma_eligible(g, false, false, HDET_EPI_ADAMW)) {
        fused->push_back({w_off, (int64_t)wy * wx});
        return hdet_launch_bgemm_dma(g, false, false, HDET_EPI_ADAMW, N, s);
      }
    }
    // A small matrix's product has too few tiles for the chip (d x d at d = 512: 128 tiles of 128 x 128 on 256 CUs,
    // each with the whole K = M to walk): it is formed in 2 or 4 pieces along the contraction, as extra batch items into
    // the logits buffer (dead since the loss kernel ran), and the pieces are added in a fixed order.
    if (sizeof(T) == 2 && !one) {
      const int64_t len = (int64_t)wy * wx, tiles = (int64_t)((wy + 127) / 128) * ((wx + 127) / 128) * N;
      const int cus = hdet_compute_units();
      int splits = 1;
      for (int c = 4; c >= 2; c >>= 1)
        if (tiles * c <= 2 * (int64_t)cus && M % (c * 64) == 0 && M / c >= 512) { splits = c; break; }
      if (splits > 1 && tiles < cus && (len & 3) == 0 && (w_off & 3) == 0 && (ps & 3) == 0 &&
          (int64_t)N * splits * len <= (int64_t)N * M * V) {
        const int kc = M / splits;
        const mat a = {dy, wy, {(int64_t)M * wy, (int64_t)kc * wy, 0}}, b = {x, wx, {(int64_t)M * wx, (int64_t)kc * wx, 0}};
        const int64_t cs[3] = {splits * len, len, 0};
        TF_CHECK(gemm<T>(p, TN, a, b, p->logits, wx, cs, false, wy, wx, kc, splits, 1, nullptr, 0, s));
        hipLaunchKernelGGL(wgrad_sum_kernel, dim3((unsigned)((len / 4 + 255) / 256), N), dim3(256), 0, s, p->logits, splits, len, grads, ps, w_off);
        return hipGetLastError();
      }
    }
    return gemm<T>(p, TN, act(dy, wy), act(x, wx), grads + w_off, wx, plane, false, wy, wx, one ? N * M : M, 1, 1, nullptr, 0, s,
                   nullptr, one);
  };

  if (!head_part) TF_CHECK(colsum(p->dlogits, V, p->b_head));
  TF_CHECK(gemm<T>(p, NN, act(p->dlogits, V), wt(p->w_head, d), p->dtmp, d, act_d, true, M, d, V, 1, 1, nullptr, 0, s));
  TF_CHECK(wgrad(p->dlogits, V, p->hf, d, p->w_head));
  // With a dropout channel, the gradient that enters a residual branch is the stream's gradient passed
  // through that branch's dropout; the LayerNorm backward kernel that produces the stream's gradient
  // writes it as a second output where it can (dropped_done), else a separate pass does.
  bool dropped_done = false, b2_done = false, bo_done = false;    // *_done: stage 1 of that bias gradient came with the LayerNorm kernel
  da.site = 2 * (L - 1) + 1;
  if (!launch_ln_bwd_dx<T>(p, p->dtmp, p->x_in[L], p->stf_mean, p->stf_rstd, p->lnf_g, nullptr, p->dxa, s, drop ? p->dtmp2 : nullptr, &da, &dropped_done,
                           p->blk[L - 1].b_2, &b2_done))
    TF_CHECK(ln_params(p->dtmp, p->x_in[L], p->stf_mean, p->stf_rstd, p->lnf_g, p->lnf_b));
  for (int l = L - 1; l >= 0; --l) {
    const tf_block_off& o = p->blk[l];
    // MLP branch: x_out = x_mid + drop(y)
    const void* dy = p->dxa;
    if (drop) {
      da.site = 2 * l + 1;
      if (!dropped_done)
        hipLaunchKernelGGL((dropout_kernel<T, false>), dim3(grid_for(nd / 4), N), dim3(256), 0, s, (const T*)nullptr, (const T*)p->dxa, (T*)p->dtmp2, nd, da);
      dy = p->dtmp2;
    }
    if (!b2_done) TF_CHECK(colsum(dy, d, o.b_2));
    bool b1_done = false;
    {
      bool fused = false;
      // stage 1 of the first MLP layer's bias gradient comes with the product when its epilogue forms the GELU gradient
      float* b1_part = nullptr;
      for (const colsum_job& j : p->jobs)
        if (j.out_off == o.b_1 && j.mode == 0 && j.cols == ff && j.nchunks == (M + 127) / 128) { b1_part = p->part + j.part_off; break; }
      const gelu_fusion gf = {nullptr, p->z[l], &fused, nullptr, nullptr, nullptr, b1_part};
      TF_CHECK(gemm<T>(p, NN, act(dy, d), wt(o.w_2, ff), p->dff, ff, act_ff, true, M, ff, d, 1, 1, nullptr, 0, s, &gf));
      if (!fused)
        hipLaunchKernelGGL(gelu_bwd_kernel<T>, dim3(grid_for((int64_t)N * nff)), dim3(256), 0, s, (const T*)p->dff, (const T*)p->z[l], (T*)p->dff, (int64_t)N * nff);
      b1_done = fused && b1_part;
    }
    TF_CHECK(wgrad(dy, d, p->f[l], ff, o.w_2));
    if (!b1_done) TF_CHECK(colsum(p->dff, ff, o.b_1));
    TF_CHECK(gemm<T>(p, NN, act(p->dff, ff), wt(o.w_1, d), p->dtmp, d, act_d, true, M, d, ff, 1, 1, nullptr, 0, s));
    TF_CHECK(wgrad(p->dff, ff, p->h2[l], d, o.w_1));
    dropped_done = false;
    da.site = 2 * l;
    bo_done = false;
    if (!launch_ln_bwd_dx<T>(p, p->dtmp, p->x_mid[l], p->st2_mean[l], p->st2_rstd[l], o.ln2_g, p->dxa, p->dxb, s, drop ? p->dtmp2 : nullptr, &da, &dropped_done,
                             o.b_o, &bo_done))
      TF_CHECK(ln_params(p->dtmp, p->x_mid[l], p->st2_mean[l], p->st2_rstd[l], o.ln2_g, o.ln2_b));
    // attention branch: x_mid = x_in + drop(o)
    const void* dob = p->dxb;
    if (drop) {
      if (!dropped_done)
        hipLaunchKernelGGL((dropout_kernel<T, false>), dim3(grid_for(nd / 4), N), dim3(256), 0, s, (const T*)nullptr, (const T*)p->dxb, (T*)p->dtmp2, nd, da);
      dob = p->dtmp2;
    }
    if (!bo_done) TF_CHECK(colsum(dob, d, o.b_o));
    TF_CHECK(gemm<T>(p, NN, act(dob, d), wt(o.w_o, d), p->dtmp, d, act_d, true, M, d, d, 1, 1, nullptr, 0, s));   // da
    TF_CHECK(wgrad(dob, d, p->a[l], d, o.w_o));
    if (p->fused_attn) {
      hdet_attn_desc ad = attn_desc(l);
      TF_CHECK(hdet_launch_attn_bwd(ad, s));
    } else {
      const mat sc = head_sq(p->scores);
      const mat dq = qkv_part(p->dqkv, 0), dk = qkv_part(p->dqkv, 1), dv = qkv_part(p->dqkv, 2);
      // dp = da v^T
      TF_CHECK(gemm<T>(p, NT, head_cols(p->dtmp), qkv_part(p->qkv[l], 2), p->scores, S, sc.s, false, S, S, dh, B, nh, nullptr, 0, s));
      // dv = p^T da
      TF_CHECK(gemm<T>(p, TN, head_sq(p->p[l]), head_cols(p->dtmp), (void*)dv.p, 3 * d, dv.s, true, S, dh, S, B, nh, nullptr, 0, s));
      launch_softmax_bwd<T>(p->scores, p->p[l], heads_rows, S, scale, ta, p->ds, s);
      // dq = ds k,  dk = ds^T q
      TF_CHECK(gemm<T>(p, NN, head_sq(p->ds), qkv_part(p->qkv[l], 1), (void*)dq.p, 3 * d, dq.s, true, S, dh, S, B, nh, nullptr, 0, s));
      TF_CHECK(gemm<T>(p, TN, head_sq(p->ds), qkv_part(p->qkv[l], 0), (void*)dk.p, 3 * d, dk.s, true, S, dh, S, B, nh, nullptr, 0, s));
    }
    TF_CHECK(colsum(p->dqkv, 3 * d, o.b_qkv));
    TF_CHECK(gemm<T>(p, NN, act(p->dqkv, 3 * d), wt(o.w_qkv, d), p->dtmp, d, act_d, true, M, d, 3 * d, 1, 1, nullptr, 0, s));
    TF_CHECK(wgrad(p->dqkv, 3 * d, p->h1[l], d, o.w_qkv));
    dropped_done = false;
    da.site = 2 * (l - 1) + 1;                     // the MLP branch of the block below
    b2_done = false;
    if (!launch_ln_bwd_dx<T>(p, p->dtmp, p->x_in[l], p->st1_mean[l], p->st1_rstd[l], o.ln1_g, p->dxb, p->dxa, s, drop && l > 0 ? p->dtmp2 : nullptr, &da, &dropped_done,
                             l > 0 ? p->blk[l - 1].b_2 : -1, &b2_done))
      TF_CHECK(ln_params(p->dtmp, p->x_in[l], p->st1_mean[l], p->st1_rstd[l], o.ln1_g, o.ln1_b));
  }
  hipLaunchKernelGGL(zero_kernel, dim3(grid_for((int64_t)V * d), N), dim3(256), 0, s, grads, ps, p->tok, (int64_t)V * d);
  if (M <= 16384 && d % 8 == 0 && d <= 2048 && p->tok % 4 == 0 && ps % 4 == 0) {
#define SORT(P2) hipLaunchKernelGGL(tok_sort_kernel<P2>, dim3(N), dim3(1024), 0, s, ids, M, p->tok_sorted)
    if (M <= 1024) SORT(1024); else if (M <= 2048) SORT(2048); else if (M <= 4096) SORT(4096); else if (M <= 8192) SORT(8192); else SORT(16384);
#undef SORT
    const int nch = (d / 8 + 63) / 64;
    float* seg = p->tok_seg;
#define CALL(K) hipLaunchKernelGGL((tok_segment_kernel<T, K>), dim3((M + 3) / 4, N), dim3(256), 0, s, p->tok_sorted, M, d, (const T*)p->dxa, seg)
    HDET_NCH_SWITCH(nch, CALL)
#undef CALL
#define CALL(K) hipLaunchKernelGGL((tok_total_kernel<K>), dim3((M + 3) / 4, N), dim3(256), 0, s, p->tok_sorted, M, d, seg, grads, ps, p->tok)
    HDET_NCH_SWITCH(nch, CALL)
#undef CALL
  } else {
    hipLaunchKernelGGL(embed_bwd_kernel<T>, dim3(grid_for(nd), N), dim3(256), 0, s, grads, ps, p->tok, ids, M, d, (const T*)p->dxa);
  }
  hipLaunchKernelGGL(pos_bwd_kernel<T>, dim3(grid_for((int64_t)S * d), N), dim3(256), 0, s, grads, ps, p->pos, B, S, d, (const T*)p->dxa);
  TF_CHECK(launch_colsum_final(p, s));
  return hipGetLastError();
}

}  // namespace

hipError_t hdet_tf_forward_backward(hdet_tf_plan* p, const int32_t* ids, const int32_t* targets, hdet_ctrl* ctrl,
                                    uint32_t step, hipStream_t s, const hdet_update_args* fuse, hdet_slices* fused) {
  if (!fused) fuse = nullptr;
  return p->bf16 ? run<uint16_t>(p, ids, targets, ctrl, step, s, fuse, fused) : run<float>(p, ids, targets, ctrl, step, s, nullptr, nullptr);
}

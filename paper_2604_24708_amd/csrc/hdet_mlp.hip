// "Forward + backward" of Algorithm 1 for an MLP, replica-batched: N independent weight sets,
// one launch per layer and direction with the replica on blockIdx.z.
//
// Model: Linear+bias layers, ReLU between layers, none after the last, mean cross-entropy
// over the B rows of a replica.  Parameters of a replica are one flat plane
// [W_1 (d_out x d_in, row-major), b_1, W_2, b_2, ...]; gradients use the same layout, so the
// update kernel can stream both without any gather.
//
// fp32 precision: an LDS-tiled SGEMM with fused bias/ReLU (forward) and ReLU-mask (dgrad)
// epilogues.  bf16 precision (fp32 master weights): the matrix-core GEMM of
// hdet_gemm_bf16.hip on the bf16 copy of the parameters; every activation and activation
// gradient that goes to memory is bf16 except the logits; biases, loss and parameter
// gradients are fp32.  Both: a column-sum for the bias gradients and a wavefront-per-row
// softmax cross-entropy whose per-replica mean is reduced in a fixed order.

#include <vector>

#include "hdet_elem.h"
#include "hdet_internal.h"

namespace {

__device__ __forceinline__ float as_float(float x) { return x; }
__device__ __forceinline__ float as_float(uint16_t h) { return __uint_as_float((unsigned)h << 16); }
__device__ __forceinline__ void put(float* p, float x) { *p = x; }
__device__ __forceinline__ void put(uint16_t* p, float x) {
  unsigned u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) { *p = (uint16_t)((u >> 16) | 0x0040u); return; }
  u += 0x7fffu + ((u >> 16) & 1u);
  *p = (uint16_t)(u >> 16);
}

// db[z][o] = sum_b dZ[z][b][o].  Block = 64 columns x 4 row phases: thread (c, q) adds rows
// q, q+4, ... in ascending order, the four partial sums are then added in the order q = 0..3.
template <typename T>
__global__ __launch_bounds__(256) void bias_grad_kernel(const T* dz, int rows, int cols, int64_t dz_bs,
                                                        float* db, int64_t db_bs) {
  __shared__ float part[4][64];
  const int c = threadIdx.x & 63, q = threadIdx.x >> 6;
  const int o = blockIdx.x * 64 + c;
  float s = 0.f;
  if (o < cols) {
    const T* p = dz + (int64_t)blockIdx.y * dz_bs + o;
    for (int b = q; b < rows; b += 4) s += as_float(p[(int64_t)b * cols]);
  }
  part[q][c] = s;
  __syncthreads();
  if (q == 0 && o < cols) db[(int64_t)blockIdx.y * db_bs + o] = ((part[0][c] + part[1][c]) + part[2][c]) + part[3][c];
}

// x (fp32) -> bf16, round to nearest even: the input batch as the first GEMM sees it
__global__ __launch_bounds__(256) void to_bf16_kernel(const float* x, uint16_t* y, int64_t n) {
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) put(y + i, x[i]);
}

__device__ __forceinline__ float wave_max(float x) {
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
  return x;
}

// Label smoothing eps of replica r (Remark 1): the value of its channel, or 0 without one.
__device__ __forceinline__ float smoothing_of(const hdet_ctrl* ctrl, int ls_channel, int r) {
  return ls_channel >= 0 ? (float)hdet_channel_value(ctrl, ls_channel, r, 0.0) : 0.f;
}

// One wavefront per row.  With the target q = (1 - eps) onehot + eps / C:
//   loss_b = log(sum exp(z - max)) - (1 - eps) (z_y - max) - eps mean_c (z_c - max),
//   dlogits = (softmax - q) / B.
// 4 rows per 256-thread block.
// grad_rows: the row count the gradient is divided by -- `rows`, or N * rows when the replica mean of the
// gradients is formed downstream as one sum over all replicas' rows (shared-gradient mode).
template <typename T>
__global__ __launch_bounds__(256) void xent_kernel(const float* logits, const int32_t* labels, int rows,
                                                   int classes, T* dlogits, float* row_loss, const hdet_ctrl* ctrl,
                                                   int ls_channel, int grad_rows) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const float eps = smoothing_of(ctrl, ls_channel, blockIdx.y);
  const int64_t gr = (int64_t)blockIdx.y * rows + row;
  const float* z = logits + gr * classes;
  float mx = -INFINITY;
  for (int c = lane; c < classes; c += 64) mx = fmaxf(mx, z[c]);
  mx = wave_max(mx);
  float se = 0.f, sz = 0.f;
  for (int c = lane; c < classes; c += 64) { se += expf(z[c] - mx); sz += z[c] - mx; }
  se = wave_sum(se);
  sz = wave_sum(sz);
  const int y = labels[gr];
  const float inv = 1.f / se, invb = 1.f / (float)grad_rows;
  const float hit = 1.f - eps, miss = eps / (float)classes;
  T* d = dlogits + gr * classes;
  for (int c = lane; c < classes; c += 64) put(d + c, (expf(z[c] - mx) * inv - (c == y ? hit : 0.f) - miss) * invb);
  if (lane == 0) row_loss[gr] = logf(se) - hit * (z[y] - mx) - eps * (sz / (float)classes);
}

// Wide rows (2048 <= classes <= 32768, classes % 4 == 0): one block of BS threads per row, the row
// held in registers (thread t owns the 4-element chunks t, t + BS, ...), so the logits are
// read once; logits and their gradient are streamed past the caches.  Same quantities as
// xent_kernel, arranged for few instructions per element: e = exp2(z * log2(e) - max * log2(e)) on the
// hardware's exp2 (relative error about 1e-7), gradient e * (1 / (sum * rows)) - miss / rows with the
// label's entry corrected by its owner, sum of (z - max) as sum of z minus classes * max.
//
// With colsum != nullptr a block takes `rows_per_block` consecutive rows, one after the other with the
// next row's loads in flight, and a thread also adds up, per column it owns, the gradients it stores:
// colsum[(replica * gridDim.x + blockIdx.x) * classes + c] = sum over the block's rows of dlogits as
// stored, rows in ascending order -- stage 1 of the output layer's bias gradient.
constexpr float kLog2e = 1.4426950408889634f;

template <int BS>
__device__ __forceinline__ void xent_block_reduce(float& a, float& b, float* red, float* red2, bool is_max) {
  constexpr int NW = BS / 64;
  const int tid = threadIdx.x;
  if (is_max) a = wave_max(a);
  else { a = wave_sum(a); b = wave_sum(b); }
  if ((tid & 63) == 0) { red[tid >> 6] = a; red2[tid >> 6] = b; }
  __syncthreads();
  a = red[0];
  b = red2[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) {
    if (is_max) a = fmaxf(a, red[w]);
    else { a += red[w]; b += red2[w]; }
  }
  __syncthreads();
}

template <typename T, int BS, int NV, bool SUMS>
__global__ __launch_bounds__(BS, SUMS ? 2 : 4) void xent_row_kernel(const float* logits, const int32_t* labels, int rows, int classes,
                                                      int rows_per_block, T* dlogits, float* row_loss, const hdet_ctrl* ctrl,
                                                      int ls_channel, float* colsum, int grad_rows) {
  constexpr int NW = BS / 64;
  __shared__ float red[NW], red2[NW];
  const int r = blockIdx.y, tid = threadIdx.x, c4 = classes >> 2;
  const float eps = smoothing_of(ctrl, ls_channel, r);
  const float invb = 1.f / (float)grad_rows, hit = 1.f - eps, miss = eps / (float)classes;
  const float hitb = hit * invb, missb = miss * invb;
  const int row0 = blockIdx.x * rows_per_block;
  const int row1 = row0 + rows_per_block < rows ? row0 + rows_per_block : rows;
  hdet_f4 cur[NV], nxt[SUMS ? NV : 1], acc[SUMS ? NV : 1];
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    if (SUMS) {
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i].v[j] = 0.f;
    }
    if (tid + BS * i < c4 && row0 < row1) cur[i] = hdet_ld4_stream(logits + ((int64_t)r * rows + row0) * classes + 4 * (tid + BS * i));
  }
  for (int row = row0; row < row1; ++row) {
    const int64_t gr = (int64_t)r * rows + row;
    if (SUMS && row + 1 < row1) {
#pragma unroll
      for (int i = 0; i < NV; ++i)
        if (tid + BS * i < c4) nxt[i] = hdet_ld4_stream(logits + (gr + 1) * classes + 4 * (tid + BS * i));
    }
    float mx = -INFINITY, sz = 0.f, unused = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i)
      if (tid + BS * i < c4) {
#pragma unroll
        for (int j = 0; j < 4; ++j) { mx = fmaxf(mx, cur[i].v[j]); sz += cur[i].v[j]; }
      }
    xent_block_reduce<BS>(mx, unused, red, red2, true);
    const float mxl = mx * kLog2e;
    float se = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i)
      if (tid + BS * i < c4) {
#pragma unroll
        for (int j = 0; j < 4; ++j) { cur[i].v[j] = __builtin_amdgcn_exp2f(__builtin_fmaf(cur[i].v[j], kLog2e, -mxl)); se += cur[i].v[j]; }
      }
    xent_block_reduce<BS>(se, sz, red, red2, false);
    const int y = __builtin_amdgcn_readfirstlane(labels[gr]);      // the same for the whole block
    const int ych = y >> 2;
    const float a = invb / se;
    T* dl = dlogits + gr * classes;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int ch = tid + BS * i;
      if (ch < c4) {
        hdet_f4 o;
#pragma unroll
        for (int j = 0; j < 4; ++j) o.v[j] = __builtin_fmaf(cur[i].v[j], a, -missb);
        if (ych >= BS * i && ych < BS * (i + 1)) {                  // uniform: the label's chunk is among these
          asm volatile("" ::: "memory");                            // keeps this a branch, taken once per row
#pragma unroll
          for (int j = 0; j < 4; ++j) o.v[j] -= 4 * ch + j == y ? hitb : 0.f;
        }
        hdet_st4_stream(dl + 4 * ch, o);
        if (SUMS) {
          if (sizeof(T) == 2) {
            const unsigned u0 = hdet_bf16_pack(o.v[0], o.v[1]), u1 = hdet_bf16_pack(o.v[2], o.v[3]);
            acc[i].v[0] += __uint_as_float(u0 << 16);
            acc[i].v[1] += __uint_as_float(u0 & 0xffff0000u);
            acc[i].v[2] += __uint_as_float(u1 << 16);
            acc[i].v[3] += __uint_as_float(u1 & 0xffff0000u);
          } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[i].v[j] += o.v[j];
          }
        }
      }
    }
    if (tid == 0) row_loss[gr] = logf(se) - hit * (logits[gr * classes + y] - mx) - eps * (sz / (float)classes - mx);
    if (SUMS) {
#pragma unroll
      for (int i = 0; i < NV; ++i) cur[i] = nxt[i];
    }
  }
  if (SUMS) {
    float* cs = colsum + ((int64_t)r * gridDim.x + blockIdx.x) * classes;
#pragma unroll
    for (int i = 0; i < NV; ++i)
      if (tid + BS * i < c4) *reinterpret_cast<hdet_f4*>(cs + 4 * (tid + BS * i)) = acc[i];
  }
}

// Per-replica mean of the row losses in a fixed tree order (one block per replica), the
// step loss l(theta_r, B_r) of Algorithm 1, and its accumulation into L_acc (Sec. 3.4).
__global__ __launch_bounds__(256) void loss_reduce_kernel(const float* row_loss, int rows, hdet_ctrl* ctrl) {
  __shared__ double part[4];
  const int r = blockIdx.x;
  double s = 0.0;
  for (int b = threadIdx.x; b < rows; b += 256) s += (double)row_loss[(int64_t)r * rows + b];
  for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    const double mean = (part[0] + part[1] + part[2] + part[3]) / (double)rows;
    ctrl->l_step[r] = (float)mean;
    ctrl->l_acc[r] += mean;
  }
}

}  // namespace

struct hdet_mlp_plan {
  hdet_config cfg;
  hdet_buffers buf;
  int n_layers;
  std::vector<int64_t> w_off, b_off;     // offsets inside a parameter plane
  std::vector<void*> act;                // act[i]: input of layer i, fp32 or bf16 by precision
                                         // (fp32: act[0] is the caller's x; bf16: its bf16 copy)
  float* logits;
  void* dz_a; void* dz_b;                // ping-pong activation gradients, fp32 or bf16
  float* row_loss;
  float* colsum_part;                    // bf16: [N][ceil(B / 128)][widest layer] partial column sums of an activation gradient
  bool bf16;
  int ls_channel;                        // label-smoothing channel or -1
};

bool hdet_xent_wide(int classes) { return classes >= 2048 && classes <= 32768 && classes % 4 == 0; }

hipError_t hdet_launch_xent(bool bf16, const float* logits, const int32_t* labels, int rows, int classes, void* dlogits,
                            float* row_loss, int n_replicas, const hdet_ctrl* ctrl, int ls_channel, hipStream_t s,
                            float* colsum, int rows_per_block, int grad_rows) {
  if (grad_rows <= 0) grad_rows = rows;
  if (hdet_xent_wide(classes)) {
    const bool sums = colsum != nullptr && rows_per_block > 0;
    if (!sums) rows_per_block = 1;
    const dim3 grid((rows + rows_per_block - 1) / rows_per_block, n_replicas);
#define HDET_XENT_ROW(T, BS, NV, SUMS) \
  hipLaunchKernelGGL((xent_row_kernel<T, BS, NV, SUMS>), grid, dim3(BS), 0, s, logits, labels, rows, classes, rows_per_block, (T*)dlogits, row_loss, ctrl, ls_channel, colsum, grad_rows)
#define HDET_XENT_ROW_T(BS, NV, SUMS)        \
  do {                                       \
    if (bf16) HDET_XENT_ROW(uint16_t, BS, NV, SUMS); \
    else HDET_XENT_ROW(float, BS, NV, SUMS); \
  } while (0)
    if (classes <= 8192) {
      if (sums) HDET_XENT_ROW_T(256, 8, true);
      else HDET_XENT_ROW_T(256, 8, false);
    } else {
      if (sums) HDET_XENT_ROW_T(512, 16, true);
      else HDET_XENT_ROW_T(512, 16, false);
    }
#undef HDET_XENT_ROW_T
#undef HDET_XENT_ROW
    return hipGetLastError();
  }
  const dim3 grid((rows + 3) / 4, n_replicas);
  if (bf16) hipLaunchKernelGGL(xent_kernel<uint16_t>, grid, dim3(256), 0, s, logits, labels, rows, classes, (uint16_t*)dlogits, row_loss, ctrl, ls_channel, grad_rows);
  else hipLaunchKernelGGL(xent_kernel<float>, grid, dim3(256), 0, s, logits, labels, rows, classes, (float*)dlogits, row_loss, ctrl, ls_channel, grad_rows);
  return hipGetLastError();
}

hipError_t hdet_launch_loss_reduce(const float* row_loss, int rows, hdet_ctrl* ctrl, int n_replicas, hipStream_t s) {
  hipLaunchKernelGGL(loss_reduce_kernel, dim3(n_replicas), dim3(256), 0, s, row_loss, rows, ctrl);
  return hipGetLastError();
}

static size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

int hdet_mlp_workspace_bytes(const hdet_config& cfg, size_t* bytes, std::string* err) {
  (void)err;
  const size_t n = cfg.n_replicas, b = cfg.dims.batch;
  const int L = cfg.dims.n_layers;
  const bool bf16 = cfg.precision == HDET_BF16_GEMM_FP32_MASTER;
  const size_t esz = bf16 ? sizeof(uint16_t) : sizeof(float);
  size_t total = 0, maxw = 0;
  if (bf16) total += align_up(n * b * (size_t)cfg.dims.widths[0] * esz);      // bf16 copy of x
  for (int i = 1; i <= L; ++i) {                                              // act[1..L-1], logits
    total += align_up(n * b * (size_t)cfg.dims.widths[i] * (i < L ? esz : sizeof(float)));
    if ((size_t)cfg.dims.widths[i] > maxw) maxw = cfg.dims.widths[i];
  }
  for (int i = 0; i < L; ++i) if ((size_t)cfg.dims.widths[i] > maxw) maxw = cfg.dims.widths[i];
  total += 2 * align_up(n * b * maxw * esz);                                  // dz ping-pong
  total += align_up(n * b * sizeof(float));                                   // row losses
  if (bf16) total += align_up(n * ((b + 127) / 128) * maxw * sizeof(float));  // column sums per 128-row chunk
  *bytes = total;
  return HDET_OK;
}

hdet_mlp_plan* hdet_mlp_create(const hdet_config& cfg, const hdet_buffers& buf, int ls_channel, std::string* err) {
  size_t need = 0;
  if (hdet_mlp_workspace_bytes(cfg, &need, err) != HDET_OK) return nullptr;
  if (!buf.workspace_dev || buf.workspace_bytes < need) { *err = "workspace_dev is too small"; return nullptr; }
  hdet_mlp_plan* p = new hdet_mlp_plan();
  p->cfg = cfg; p->buf = buf; p->n_layers = cfg.dims.n_layers;
  p->ls_channel = ls_channel;
  const size_t n = cfg.n_replicas, b = cfg.dims.batch;
  const int L = p->n_layers;
  int64_t off = 0;
  for (int i = 0; i < L; ++i) {
    p->w_off.push_back(off); off += (int64_t)cfg.dims.widths[i + 1] * cfg.dims.widths[i];
    p->b_off.push_back(off); off += cfg.dims.widths[i + 1];
  }
  char* ws = (char*)buf.workspace_dev;
  size_t maxw = 0;
  for (int i = 0; i <= L; ++i) if ((size_t)cfg.dims.widths[i] > maxw) maxw = cfg.dims.widths[i];
  p->bf16 = cfg.precision == HDET_BF16_GEMM_FP32_MASTER;
  const size_t esz = p->bf16 ? sizeof(uint16_t) : sizeof(float);
  p->act.assign(L, nullptr);
  if (p->bf16) { p->act[0] = ws; ws += align_up(n * b * (size_t)cfg.dims.widths[0] * esz); }
  for (int i = 1; i <= L; ++i) {
    void* ptr = ws; ws += align_up(n * b * (size_t)cfg.dims.widths[i] * (i < L ? esz : sizeof(float)));
    if (i < L) p->act[i] = ptr; else p->logits = (float*)ptr;
  }
  p->dz_a = ws; ws += align_up(n * b * maxw * esz);
  p->dz_b = ws; ws += align_up(n * b * maxw * esz);
  p->row_loss = (float*)ws; ws += align_up(n * b * sizeof(float));
  p->colsum_part = p->bf16 ? (float*)ws : nullptr;
  return p;
}

void hdet_mlp_destroy(hdet_mlp_plan* p) { delete p; }

static hipError_t forward_backward_f32(hdet_mlp_plan* p, const void* x, const int32_t* y, hdet_ctrl* ctrl,
                                       hipStream_t s) {
  const hdet_config& c = p->cfg;
  const int N = c.n_replicas, B = c.dims.batch, L = p->n_layers;
  const int* w = c.dims.widths;
  const int64_t ps = p->buf.plane_stride;
  const float* theta = p->buf.params_dev;
  float* grads = p->buf.grads_dev;
  p->act[0] = const_cast<void*>(x);
  // Shared-gradient mode (Algorithm 1, "AllReduce gradients"): every replica applies the replica mean, so only the sum of
  // the replicas' gradients is formed -- the N batches are rows of one matrix, a weight gradient is one product over
  // K = N B rows -- in plane 0 of the gradient buffer; the update kernel multiplies by 1 / N.
  const bool shared = c.grad_mode == HDET_GRAD_SHARED;

  // forward: Y = act(X W^T + b)
  for (int i = 0; i < L; ++i) {
    hdet_sgemm_args g = {};
    g.a = (const float*)p->act[i]; g.a_rs = w[i]; g.a_cs = 1; g.a_s[0] = (int64_t)B * w[i];
    g.b = theta + p->w_off[i]; g.b_rs = 1; g.b_cs = w[i]; g.b_s[0] = ps;      // B(k,n) = W[n][k]
    g.c = i + 1 < L ? (float*)p->act[i + 1] : p->logits; g.c_rs = w[i + 1]; g.c_s[0] = (int64_t)B * w[i + 1];
    g.m = B; g.n = w[i + 1]; g.k = w[i];
    g.bias = theta + p->b_off[i]; g.bias_bs = ps;
    if (hipError_t e = hdet_launch_sgemm(g, i + 1 < L ? HDET_SEPI_BIAS_RELU : HDET_SEPI_BIAS, N, s)) return e;
  }
  // loss and dlogits
  float* dz = (float*)p->dz_a; float* dz_next = (float*)p->dz_b;
  if (hipError_t e = hdet_launch_xent(false, p->logits, y, B, w[L], dz, p->row_loss, N, ctrl, p->ls_channel, s, nullptr, 0, B)) return e;
  hipLaunchKernelGGL(loss_reduce_kernel, dim3(N), dim3(256), 0, s, p->row_loss, B, ctrl);
  // backward
  for (int i = L - 1; i >= 0; --i) {
    // dW = dZ^T X
    hdet_sgemm_args g = {};
    g.a = dz; g.a_rs = 1; g.a_cs = w[i + 1]; g.a_s[0] = (int64_t)B * w[i + 1];     // A(o,b) = dZ[b][o]
    g.b = (const float*)p->act[i]; g.b_rs = w[i]; g.b_cs = 1; g.b_s[0] = (int64_t)B * w[i];   // B(b,k) = X[b][k]
    g.c = grads + p->w_off[i]; g.c_rs = w[i]; g.c_s[0] = ps;
    g.m = w[i + 1]; g.n = w[i]; g.k = shared ? N * B : B;
    if (hipError_t e = hdet_launch_sgemm(g, HDET_SEPI_NONE, shared ? 1 : N, s)) return e;
    hipLaunchKernelGGL(bias_grad_kernel<float>, dim3((w[i + 1] + 63) / 64, shared ? 1 : N), dim3(256), 0, s, dz, shared ? N * B : B, w[i + 1],
                       (int64_t)B * w[i + 1], grads + p->b_off[i], ps);
    if (i > 0) {
      // dX = dZ W, masked by the ReLU of the layer below
      hdet_sgemm_args d = {};
      d.a = dz; d.a_rs = w[i + 1]; d.a_cs = 1; d.a_s[0] = (int64_t)B * w[i + 1];
      d.b = theta + p->w_off[i]; d.b_rs = w[i]; d.b_cs = 1; d.b_s[0] = ps;         // B(o,k) = W[o][k]
      d.c = dz_next; d.c_rs = w[i]; d.c_s[0] = (int64_t)B * w[i];
      d.m = B; d.n = w[i]; d.k = w[i + 1];
      d.mask = (const float*)p->act[i]; d.mask_rs = w[i]; d.mask_bs = (int64_t)B * w[i];
      if (hipError_t e = hdet_launch_sgemm(d, HDET_SEPI_MASK, N, s)) return e;
      float* t = dz; dz = dz_next; dz_next = t;
    }
  }
  return hipGetLastError();
}

static hipError_t forward_backward_bf16(hdet_mlp_plan* p, const void* x, const int32_t* y, hdet_ctrl* ctrl,
                                        hipStream_t s, const hdet_update_args* fuse, hdet_slices* fused) {
  const hdet_config& c = p->cfg;
  const int N = c.n_replicas, B = c.dims.batch, L = p->n_layers;
  const int* w = c.dims.widths;
  const int64_t ps = p->buf.plane_stride;
  const float* theta = p->buf.params_dev;           // biases (fp32)
  const uint16_t* wbf = p->buf.params_bf16_dev;     // weights as the GEMMs see them
  float* grads = p->buf.grads_dev;
  hipError_t e;
  const bool shared = c.grad_mode == HDET_GRAD_SHARED;      // one gradient plane: see forward_backward_f32

  const int64_t nx = (int64_t)N * B * w[0];
  int cb = (int)((nx + 255) / 256); if (cb > 4096) cb = 4096;
  hipLaunchKernelGGL(to_bf16_kernel, dim3(cb), dim3(256), 0, s, (const float*)x, (uint16_t*)p->act[0], nx);

  for (int i = 0; i < L; ++i) {                      // forward: Y = act(X W^T + b)
    hdet_bgemm_args g = {};
    g.a = (const uint16_t*)p->act[i]; g.lda = w[i]; g.a_s[0] = (int64_t)B * w[i];
    g.b = wbf + p->w_off[i]; g.ldb = w[i]; g.b_s[0] = ps;
    g.c = i + 1 < L ? p->act[i + 1] : (void*)p->logits; g.ldc = w[i + 1]; g.c_s[0] = (int64_t)B * w[i + 1];
    g.m = B; g.n = w[i + 1]; g.k = w[i];
    g.bias = theta + p->b_off[i]; g.bias_bs = ps;
    e = hdet_launch_bgemm(g, true, true, i + 1 < L ? HDET_EPI_BIAS_RELU_BF16 : HDET_EPI_BIAS_F32, N, s);
    if (e != hipSuccess) return e;
  }
  uint16_t* dz = (uint16_t*)p->dz_a; uint16_t* dz_next = (uint16_t*)p->dz_b;
  const int nchunks = (B + 127) / 128;
  bool have_part = false;
  if (hipError_t e = hdet_launch_xent(true, p->logits, y, B, w[L], dz, p->row_loss, N, ctrl, p->ls_channel, s, nullptr, 0, B)) return e;
  hipLaunchKernelGGL(loss_reduce_kernel, dim3(N), dim3(256), 0, s, p->row_loss, B, ctrl);
  for (int i = L - 1; i >= 0; --i) {
    // db = column sums of dZ: from the 128-row partial sums when the product that formed dZ left them, else from dZ itself
    if (have_part)
      hipLaunchKernelGGL(bias_grad_kernel<float>, dim3((w[i + 1] + 63) / 64, shared ? 1 : N), dim3(256), 0, s, p->colsum_part,
                         shared ? N * nchunks : nchunks, w[i + 1], (int64_t)nchunks * w[i + 1], grads + p->b_off[i], ps);
    else
      hipLaunchKernelGGL(bias_grad_kernel<uint16_t>, dim3((w[i + 1] + 63) / 64, shared ? 1 : N), dim3(256), 0, s, dz, shared ? N * B : B, w[i + 1],
                         (int64_t)B * w[i + 1], grads + p->b_off[i], ps);
    have_part = false;
    const uint16_t* dz_cur = dz;
    if (i > 0) {                                     // dX = dZ W, through the ReLU below (before W is touched by a fused update)
      hdet_bgemm_args d = {};
      d.a = dz; d.lda = w[i + 1]; d.a_s[0] = (int64_t)B * w[i + 1];
      d.b = wbf + p->w_off[i]; d.ldb = w[i]; d.b_s[0] = ps;                       // B(o,k) = W[o][k]
      d.c = dz_next; d.ldc = w[i]; d.c_s[0] = (int64_t)B * w[i];
      d.m = B; d.n = w[i]; d.k = w[i + 1];
      d.mask = (const uint16_t*)p->act[i]; d.mask_ld = w[i]; d.mask_bs = (int64_t)B * w[i];
      d.n1 = d.n2 = 1;
      if (hdet_bgemm_dma_eligible(d, true, false, HDET_EPI_MASK_BF16)) {       // that kernel also leaves the column sums of dX
        d.colsum = p->colsum_part;
        have_part = true;
      }
      e = hdet_launch_bgemm(d, true, false, HDET_EPI_MASK_BF16, N, s);
      if (e != hipSuccess) return e;
      uint16_t* t = dz; dz = dz_next; dz_next = t;
    }
    hdet_bgemm_args g = {};                          // dW = dZ^T X
    g.a = dz_cur; g.lda = w[i + 1]; g.a_s[0] = (int64_t)B * w[i + 1];           // A(o,b) = dZ[b][o]
    g.b = (const uint16_t*)p->act[i]; g.ldb = w[i]; g.b_s[0] = (int64_t)B * w[i];   // B(b,k) = X[b][k]
    g.c = grads + p->w_off[i]; g.ldc = w[i]; g.c_s[0] = ps;
    g.m = w[i + 1]; g.n = w[i]; g.k = shared ? N * B : B;
    g.n1 = g.n2 = 1;
    const int64_t wlen = (int64_t)w[i + 1] * w[i];
    // the update of W applied by the product that forms its gradient (Eq. 2): dW never goes to memory
    if (fuse && !shared && hdet_fuse_args_for(c, *fuse, p->w_off[i], w[i + 1], w[i], &g.upd) &&
        hdet_bgemm_dma_eligible(g, false, false, HDET_EPI_ADAMW)) {
      e = hdet_launch_bgemm_dma(g, false, false, HDET_EPI_ADAMW, N, s);
      if (e != hipSuccess) return e;
      fused->push_back({p->w_off[i], wlen});
      continue;
    }
    e = hdet_launch_bgemm(g, false, false, HDET_EPI_F32, shared ? 1 : N, s);
    if (e != hipSuccess) return e;
  }
  return hipGetLastError();
}

hipError_t hdet_mlp_forward_backward(hdet_mlp_plan* p, const void* x, const int32_t* y, hdet_ctrl* ctrl,
                                     hipStream_t s, const hdet_update_args* fuse, hdet_slices* fused) {
  return p->bf16 ? forward_backward_bf16(p, x, y, ctrl, s, fused ? fuse : nullptr, fused) : forward_backward_f32(p, x, y, ctrl, s);
}

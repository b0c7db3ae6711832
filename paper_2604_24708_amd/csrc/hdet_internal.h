// Internal declarations shared by the translation units of libhdet.so.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <utility>
#include <vector>

#include "hdet.h"

typedef std::vector<std::pair<int64_t, int64_t>> hdet_slices;    // (offset, length) slices of a parameter plane

// ---------------------------------------------------------------------------------------
// Device-resident schedule / controller state (one per handle).  Kernels read the rates
// from here, so no step needs a host round trip: the host only knows t.
// ---------------------------------------------------------------------------------------
struct hdet_ctrl {
  double base[HDET_MAX_CH];                       // h_bar_j (Eq. 7); [0] valid once active
  double vel[HDET_MAX_CH];                        // v_j
  double delta[HDET_MAX_CH];                      // last Delta_j (Eq. 6)
  double rho[HDET_MAX_CH][HDET_MAX_REPLICAS];     // Eq. 1 per channel
  double w[HDET_MAX_REPLICAS];                    // last softmax weights (Eq. 4)
  double l_acc[HDET_MAX_REPLICAS];                // running loss sum of the interval
  double l_last[HDET_MAX_REPLICAS];               // L_r of the last sync step
  float l_step[HDET_MAX_REPLICAS];                // losses of the last forward
  float lr_used[HDET_MAX_REPLICAS];               // rates of the last update
  int32_t perm[HDET_MAX_CH][HDET_MAX_REPLICAS];   // pi_j
  long long k;                                    // controller updates done
  int32_t controller_active;
  int32_t nonfinite;
  int32_t n_lr;                                   // channels 0..n_lr-1 are learning rates (one per group)
  int32_t pad_;
  double warm_sumsq;                              // ||theta0||^2 of the warm initialisation
  double warm_partial[1024];                      // its per-block partial sums
};
#define HDET_WARM_PARTIALS 1024

// h_{j,r} = h_bar_j * rho_{j, pi_j(r)} in fp64.  The learning-rate channels follow the host's
// one-cycle value `eta_sched` until the controller has taken over.
__device__ __forceinline__ double hdet_channel_value(const hdet_ctrl* c, int j, int r,
                                                     double eta_sched) {
  const double b = (j < c->n_lr && !c->controller_active) ? eta_sched : c->base[j];
  return b * c->rho[j][c->perm[j][r]];
}

// ---------------------------------------------------------------------------------------
// Kernel launch parameters
// ---------------------------------------------------------------------------------------
struct hdet_update_args {
  float* theta;
  const float* grad;
  float* m;
  float* v;
  uint16_t* shadow;        // bf16 copy of theta or nullptr
  const hdet_ctrl* ctrl;
  hdet_ctrl* ctrl_out;     // same block, for lr_used
  int64_t n_params;        // P
  int64_t stride;          // plane stride in elements
  int64_t grad_stride;     // plane stride of `grad`: `stride`, or 0 when every replica applies the one plane at `grad`
                           // times grad_scale (a model path in shared-gradient mode has summed the replicas' gradients
                           // there: the replica mean is that sum times 1 / N)
  float grad_scale;
  int32_t n_replicas;
  int32_t lr_channel;      // learning-rate channel of the parameter group being updated
  int32_t wd_channel;      // channel index of a weight-decay channel or -1
  int32_t first_step;      // SGDM: buf <- g'
  int32_t shared_state;    // AdamW on the mean gradient: m, v are one plane, not one per replica
  double eta_sched;        // one-cycle value of this step
  double wd_const;
  double inv_bc1;          // 1 / (1 - beta1^t)
  float inv_sqrt_bc2;      // 1 / sqrt(1 - beta2^t)
  float beta1, beta2, one_m_beta1, one_m_beta2, eps, momentum;
  int32_t fuse_min_tiles;  // host only: a weight-gradient product carries the update if it has at least this many 256 x 256 tiles
};

struct hdet_converge_args {
  float* theta;
  uint16_t* shadow;
  int64_t n_params;
  int64_t stride;
  int32_t n_replicas;
  int32_t tail_only;       // loop kernel: only the P mod 4 trailing parameters
};

struct hdet_controller_args {
  hdet_ctrl* ctrl;
  double injected[HDET_MAX_REPLICAS];  // interval losses given by the caller
  int32_t use_injected;
  int32_t run_controller;              // enabled and t >= S_warm
  int32_t n_replicas, n_channels;
  int32_t n_lr;                        // learning-rate channels come first
  int32_t sync_interval;
  int32_t reshuffle;                   // new permutations at every sync step, numbered by it
  uint32_t sync_index;                 // t / T of this sync step
  double eta_sched;                    // one-cycle value of the sync step (hand-over)
  double sigma, beta, gamma;
  double lambda[HDET_MAX_CH], lo[HDET_MAX_CH], hi[HDET_MAX_CH];
  uint32_t seed_lo, seed_hi;
};

// variant 0: fastest kernel for the case; 1: the general loop kernel for everything
hipError_t hdet_launch_update(const hdet_update_args& a, int optimizer, bool shared, bool fuse_converge,
                              int variant, int blocks, hipStream_t stream);
hipError_t hdet_launch_converge(const hdet_converge_args& a, int variant, int blocks, hipStream_t stream);
hipError_t hdet_launch_shadow(const float* theta, uint16_t* shadow, int64_t n_params, int64_t stride,
                              int n_replicas, int blocks, hipStream_t stream);
hipError_t hdet_launch_controller(const hdet_controller_args& a, hipStream_t stream);
hipError_t hdet_launch_warm_init(const float* theta0, float* theta, int64_t n_params, int64_t stride, int n_replicas,
                                 double* partial, double* sumsq, double nu, uint64_t seed, hipStream_t stream);
// the noise generator numbers blocks of four parameters with a 32-bit counter word
#define HDET_WARM_MAX_PARAMS ((int64_t)1 << 34)
// message that hdet_last_error(NULL) returns (entry points without a handle)
void hdet_set_global_error(const std::string& msg);

// ---------------------------------------------------------------------------------------
// Replica-batched GEMMs.  The batch index z of a launch is split into up to three levels,
//   z = (z0 * n1 + z1) * n2 + z2      (z0: replica; z1, z2: e.g. sequence and head),
// and an operand's base offset is z0*s[0] + z1*s[1] + z2*s[2] elements.
// ---------------------------------------------------------------------------------------
struct hdet_batch_index { int z0, z1, z2; };
__host__ __device__ __forceinline__ hdet_batch_index hdet_split_batch(int z, int n1, int n2) {
  hdet_batch_index b;
  b.z2 = z % n2;
  const int t = z / n2;
  b.z1 = t % n1;
  b.z0 = t / n1;
  return b;
}
__host__ __device__ __forceinline__ int64_t hdet_batch_offset(const hdet_batch_index& b, const int64_t* s) {
  return (int64_t)b.z0 * s[0] + (int64_t)b.z1 * s[1] + (int64_t)b.z2 * s[2];
}

// fp32 GEMM with element strides (hdet_gemm_f32.hip): C(m,n) = sum_k A(m,k) B(k,n)
enum { HDET_SEPI_NONE = 0, HDET_SEPI_BIAS = 1, HDET_SEPI_BIAS_RELU = 2, HDET_SEPI_MASK = 3 };
struct hdet_sgemm_args {
  const float* a; const float* b; float* c;
  int m, n, k;
  int n1, n2;                   // batch split (0 is read as 1)
  int64_t a_rs, a_cs, a_s[3];   // A(m,k) = a[batch + m*a_rs + k*a_cs]
  int64_t b_rs, b_cs, b_s[3];   // B(k,n) = b[batch + k*b_rs + n*b_cs]
  int64_t c_rs, c_s[3];         // C(m,n) = c[batch + m*c_rs + n]
  const float* bias; int64_t bias_bs;            // + bias[z0*bias_bs + n]
  const float* mask; int64_t mask_rs, mask_bs;   // * (mask[z0*mask_bs + m*mask_rs + n] > 0)
};
hipError_t hdet_launch_sgemm(const hdet_sgemm_args& g, int epi, int batch, hipStream_t stream);

// bf16 GEMM on the matrix cores (hdet_gemm_bf16.hip)
enum { HDET_EPI_F32 = 0, HDET_EPI_BIAS_F32 = 1, HDET_EPI_BIAS_RELU_BF16 = 2, HDET_EPI_MASK_BF16 = 3,
       HDET_EPI_BF16 = 4, HDET_EPI_BIAS_BF16 = 5,
       // LDS-direct kernel only (the caller checks hdet_bgemm_dma_eligible first):
       HDET_EPI_BIAS_GELU_BF16 = 6,   // c = bf16(acc + bias), c2 = bf16(gelu(c)): pre-activation and activation
       HDET_EPI_GELUGRAD_BF16 = 7,    // c = bf16(bf16(acc) * gelu'(mask)): gradient through the GELU at pre-activation `mask`
       HDET_EPI_BIAS_RESID_BF16 = 8,  // c = bf16(mask + bf16(acc + bias)): a Linear layer added to its residual stream `mask`
       HDET_EPI_BIAS_DROP_RESID_BF16 = 9,     // the same with dropout of the layer's output before the sum
       HDET_EPI_ADAMW = 10 };         // weight gradient that is applied at once: the AdamW update of `upd` on the tile (c is not written)

struct hdet_bgemm_args {
  const uint16_t* a;       // bf16
  const uint16_t* b;       // bf16
  void* c;                 // fp32 or bf16, row-major [m][ldc]
  void* c2;                // second bf16 output in c's layout (HDET_EPI_BIAS_GELU_BF16) or nullptr
  int m, n, k;
  int n1, n2;              // batch split (0 is read as 1)
  int64_t lda, ldb, ldc;   // leading dimensions in elements
  int64_t a_s[3], b_s[3], c_s[3];      // batch strides in elements
  const float* bias; int64_t bias_bs;  // bias[z0*bias_bs + n]
  const uint16_t* mask; int64_t mask_ld, mask_bs;   // bf16 activations gating the gradient (per replica)
  // HDET_EPI_BIAS_DROP_RESID_BF16: inverted dropout of the layer's output at the replica's rate (value of
  // channel drop_channel), masks from Philox-4x32-10 with counter (element / 4, drop_step,
  // replica * 65536 + drop_site, drop_stream) and key drop_seed; element = row * ldc + column
  const hdet_ctrl* drop_ctrl; int drop_channel;
  uint32_t drop_step, drop_site, drop_stream, drop_seed_lo, drop_seed_hi;
  // HDET_EPI_GELUGRAD_BF16 and HDET_EPI_MASK_BF16 on the LDS-direct kernel, optional (n1 = n2 = 1): colsum[(replica * ceil(m / 128) + m / 128) * n + column] receives the
  // sum of C as stored over that 128-row block of the column (stage 1 of the bias gradient of the layer whose
  // pre-activation gradient C is); colsum_bs is unused padding for alignment
  float* colsum;
  int tile_group;          // LDS-direct kernel: consecutive blocks walk groups of this many tile rows column by column (0, 1: row by row)
  // HDET_EPI_ADAMW (n1 = n2 = 1, batch item = replica): the product is the replica's gradient of a weight matrix;
  // element (row, col) updates theta / m / v / shadow at [replica * c_s[0] + row * ldc + col] of upd's pointers,
  // which point at the matrix inside plane 0, with the scalars of upd (Eq. 2; per-replica rate from upd.ctrl)
  hdet_update_args upd;
};

// Parameter group that holds the slice [off, off + len) of a plane, or -1 if it lies in more than one.
inline int hdet_group_of_slice(const hdet_config& c, int64_t off, int64_t len) {
  if (c.n_groups <= 1) return 0;
  int64_t begin = 0;
  for (int g = 0; g < c.n_groups; ++g) {
    if (off >= begin && off + len <= c.group_end[g]) return g;
    begin = c.group_end[g];
  }
  return -1;
}

// A weight matrix [rows][cols] at `off` whose update a model path may apply inside the weight-gradient product: `fuse`
// with its pointers moved to the matrix and the matrix's rate channel; false if the matrix spans parameter groups or
// the product (one per replica) has too few tiles to keep the chip's memory system busy during its epilogues -- a small
// product's update is faster as part of the plane-wide update launch.
inline bool hdet_fuse_args_for(const hdet_config& c, const hdet_update_args& fuse, int64_t off, int rows, int cols, hdet_update_args* out) {
  const int64_t len = (int64_t)rows * cols;
  const int grp = hdet_group_of_slice(c, off, len);
  if (grp < 0) return false;
  if ((int64_t)((rows + 255) / 256) * ((cols + 255) / 256) * c.n_replicas < fuse.fuse_min_tiles) return false;
  *out = fuse;
  out->theta += off; out->m += off; out->v += off;
  if (out->shadow) out->shadow += off;
  out->n_params = len;
  out->lr_channel = grp;
  return true;
}

// a_kmajor: A(m,k) at a[m*lda + k], else at a[k*lda + m]; b_kmajor: B(k,n) at b[n*ldb + k], else
// at b[k*ldb + n].  (true,true) forward, (true,false) dgrad, (false,false) wgrad.
hipError_t hdet_launch_bgemm(const hdet_bgemm_args& g, bool a_kmajor, bool b_kmajor, int epi, int batch,
                             hipStream_t stream);
// LDS-direct fast path (hdet_gemm_bf16_dma.hip): taken by hdet_launch_bgemm when `eligible` (operands of
// whole, 16-byte aligned chunks; C, bias and mask addressable 4 columns at a time; batch-item extents
// below 2 GiB); n1, n2 >= 1 on entry.
bool hdet_bgemm_dma_eligible(const hdet_bgemm_args& g, bool a_kmajor, bool b_kmajor, int epi);
int hdet_compute_units();     // compute units of the current device (queried once per device; 256 on MI355X)
hipError_t hdet_launch_bgemm_dma(const hdet_bgemm_args& g, bool a_kmajor, bool b_kmajor, int epi, int batch,
                                 hipStream_t stream);

// ---------------------------------------------------------------------------------------
// MLP forward/backward (hdet_mlp.hip)
// ---------------------------------------------------------------------------------------
struct hdet_mlp_plan;
int hdet_mlp_workspace_bytes(const hdet_config& cfg, size_t* bytes, std::string* err);
hdet_mlp_plan* hdet_mlp_create(const hdet_config& cfg, const hdet_buffers& buf, int ls_channel, std::string* err);
void hdet_mlp_destroy(hdet_mlp_plan* p);
// fuse != nullptr (mixed precision, AdamW, per-replica gradients and moments): the update described by *fuse (pointers at
// plane 0, scalars of this step) is applied to a weight matrix inside the product that forms its gradient where
// that product can; the slices (offset, length) updated that way are appended to *fused and their gradients are not
// written.
hipError_t hdet_mlp_forward_backward(hdet_mlp_plan* p, const void* x, const int32_t* y, hdet_ctrl* ctrl,
                                     hipStream_t stream, const hdet_update_args* fuse = nullptr, hdet_slices* fused = nullptr);

// ---------------------------------------------------------------------------------------
// Transformer forward/backward (hdet_transformer.hip)
// ---------------------------------------------------------------------------------------
struct hdet_tf_plan;
int64_t hdet_tf_param_count(const hdet_config& cfg);
int hdet_tf_validate(const hdet_config& cfg, std::string* err);
int hdet_tf_workspace_bytes(const hdet_config& cfg, size_t* bytes, std::string* err);
// drop_channel, ls_channel, temp_channel: channel indices of Remark 1's scalars read by the model, or -1
hdet_tf_plan* hdet_tf_create(const hdet_config& cfg, const hdet_buffers& buf, int drop_channel, int ls_channel,
                             int temp_channel, std::string* err);
void hdet_tf_destroy(hdet_tf_plan* p);
void hdet_tf_set_fused_attention(hdet_tf_plan* p, bool on);   // on by default where the fused kernels apply
// Shared-gradient mode: the slices (offset, length) of a parameter plane whose gradient the pass leaves as ONE plane, the
// sum over the replicas in plane 0 of the gradient buffer; everywhere else it leaves one gradient plane per replica.
void hdet_tf_summed_slices(const hdet_tf_plan* p, std::vector<std::pair<int64_t, int64_t>>* out);
// `step`: the update this gradient is for (keys the dropout masks)
// fuse, fused: as for hdet_mlp_forward_backward
hipError_t hdet_tf_forward_backward(hdet_tf_plan* p, const int32_t* ids, const int32_t* targets, hdet_ctrl* ctrl,
                                    uint32_t step, hipStream_t stream, const hdet_update_args* fuse = nullptr,
                                    hdet_slices* fused = nullptr);

// ---------------------------------------------------------------------------------------
// Fused causal attention, bf16 (hdet_attention.hip)
// ---------------------------------------------------------------------------------------
struct hdet_attn_desc {
  const uint16_t* qkv;      // [N][B][S][3 d_model]: q | k | v, head h in columns h*64..
  uint16_t* a;              // forward output [N][B][S][d_model]
  const uint16_t* da;       // backward: gradient at a
  uint16_t* dqkv;           // backward output, layout of qkv
  float* row_max;           // [N][B][heads][S] row statistics, written by the forward
  float* row_inv;
  float* row_dot;           // scratch of the backward, same shape
  const hdet_ctrl* ctrl;
  int temp_channel;         // attention-temperature channel or -1
  float scale;              // 1 / sqrt(d_head)
  int n_replicas, batch, seq_len, heads, d_model;
};
bool hdet_attn_fusable(int seq_len, int d_model, int heads, int batch);     // head size 64, S a multiple of 64
hipError_t hdet_launch_attn_fwd(const hdet_attn_desc& a, hipStream_t stream);
hipError_t hdet_launch_attn_bwd(const hdet_attn_desc& a, hipStream_t stream);

// ---------------------------------------------------------------------------------------
// Host handle
// ---------------------------------------------------------------------------------------
struct hdet_handle {
  hdet_config cfg;
  hdet_buffers buf;
  hipStream_t stream;
  hdet_ctrl* ctrl_dev;
  int device;
  int64_t t;
  int64_t last_autolr_t;     // sync step already processed by hdet_autolr_update
  int64_t converged_at_t;    // t whose parameters are already averaged
  double gamma;
  int n_channels;
  int n_lr;                             // learning-rate channels (parameter groups) come first
  hdet_channel channels[HDET_MAX_CH];
  int wd_channel;
  int32_t tune_variant, tune_blocks;
  bool fuse_everything;       // hdet_train_step: also small weight-gradient products carry their update
  int n_cu;
  hdet_mlp_plan* mlp;
  hdet_tf_plan* tf;
  int drop_channel;
  int ls_channel;                       // label-smoothing channel or -1
  int temp_channel;                     // attention-temperature channel or -1
  std::string err;
};

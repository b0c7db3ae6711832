/*
 * hdet.h -- C ABI of the HDET (Hyperparameter-Divergent Ensemble Training) step for one
 * AMD MI355X (gfx950).
 *
 * The N data-parallel replicas of the paper live as a replica axis in one GPU's memory:
 * every per-replica tensor is an array of N planes, plane r starting `plane_stride`
 * elements after plane r-1.  The paper's AllReduce calls become reductions along that axis.
 *
 * One training step is (Algorithm 1 of the paper):
 *     hdet_forward_backward   loss and gradient of every replica          (model modes only)
 *     hdet_fanout_step        update t with per-replica rate eta_r        (Sec. 3.2, Eq. 1-2)
 *   (or hdet_train_step for both in one call, which lets the library fuse them)
 *   and, when t mod T == 0,
 *     hdet_converge           replica mean of the parameters              (Sec. 3.3, Eq. 3)
 *     hdet_autolr_update      controller on the interval losses           (Sec. 3.4, Eq. 4-9)
 *
 * General rules
 *   - Every pointer named *_dev is DEVICE memory, owned by the caller and borrowed for the
 *     lifetime of the handle; pointers named *_host are host memory read or written during
 *     the call only.  The library allocates one small device control block per handle
 *     (a few KiB) and nothing else on the device.
 *   - All device work is enqueued on the HIP stream given at creation; calls return without
 *     waiting for it unless stated otherwise.  Calls on one handle must not overlap.
 *   - Every function returns 0 (HDET_OK) or a negative HDET_E* code; after a failure
 *     hdet_last_error() gives a message.  No C++ exception crosses this boundary.
 *   - There is no CPU fallback: without a HIP device hdet_create fails with HDET_EHIP.
 */
#ifndef HDET_H
#define HDET_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HDET_MAX_REPLICAS 64   /* one wavefront holds one replica per lane in the controller */
#define HDET_MAX_CH       8    /* explored hyperparameter channels (Remark 1)                */
#define HDET_MAX_GROUPS   4    /* parameter groups with a learning-rate channel each        */
#define HDET_MAX_LAYERS   16

enum { HDET_OK = 0, HDET_EINVAL = -1, HDET_ESTATE = -2, HDET_EHIP = -3,
       HDET_ENONFINITE = -4 };   /* an interval loss handed to hdet_autolr_update is not finite */

enum { HDET_SGDM = 0, HDET_ADAMW = 1 };                       /* optimizer                   */
enum { HDET_GRAD_SHARED = 0, HDET_GRAD_PER_REPLICA = 1 };     /* gradient exchange           */
enum { HDET_FP32 = 0, HDET_BF16_GEMM_FP32_MASTER = 1 };       /* precision of the model GEMMs */
enum { HDET_FLAT = 0, HDET_MLP = 1, HDET_TRANSFORMER = 2 };   /* model kind                  */
enum { HDET_CH_LR = 0, HDET_CH_DROPOUT = 1, HDET_CH_WD = 2,      /* channel kinds (Remark 1)   */
       HDET_CH_LABEL_SMOOTH = 3, HDET_CH_ATTN_TEMP = 4 };

/* flags of hdet_fanout_step and hdet_train_step */
#define HDET_FUSE_CONVERGE 1u  /* on a sync step, average inside the update kernel (Eq. 3)   */

typedef struct hdet_handle hdet_handle;

/* One explored scalar hyperparameter beside the learning rate (Remark 1): replica r uses
 * base * rho_{pi(r)} with rho from Eq. 1 at this channel's alpha and its own permutation. */
typedef struct {
  int32_t kind;        /* HDET_CH_DROPOUT, HDET_CH_WD, HDET_CH_LABEL_SMOOTH or HDET_CH_ATTN_TEMP */
  int32_t reserved;
  double  base;        /* initial centre value h_bar                                         */
  double  alpha;       /* spread ratio                                                       */
  double  lambda;      /* step of Eq. 7 for this channel                                     */
  double  lo, hi;      /* the centre value is clamped to [lo, hi] after each controller step.
                          Replica values range over centre * [1 - alpha, 1 + alpha] (Eq. 1), so
                          the whole range must stay meaningful: hi * (1 + alpha) < 1 for a
                          dropout rate, <= 1 for label smoothing, lo * (1 - alpha) > 0 for an
                          attention temperature; lo <= base <= hi.  HDET_EINVAL otherwise.    */
} hdet_channel;

typedef struct {
  int64_t n_params;                        /* HDET_FLAT: P, parameters per replica           */
  int32_t n_layers;                        /* HDET_MLP: number of Linear layers              */
  int32_t widths[HDET_MAX_LAYERS + 1];     /* HDET_MLP: d_in, hidden..., d_out               */
  int32_t batch;                           /* HDET_MLP: rows per replica and step;
                                              HDET_TRANSFORMER: sequences per replica and step */
  /* HDET_TRANSFORMER: decoder-only, pre-LayerNorm, learned positions, tanh-GELU MLP, causal
   * attention, biases on every Linear, untied output head, final LayerNorm (eps 1e-5).      */
  int32_t n_blocks, d_model, n_heads, d_ff, seq_len, vocab;
} hdet_model_dims;

/* Arguments of Algorithm 1 ("Require") plus what the paper leaves to the optimizer. */
typedef struct {
  int32_t  n_replicas;      /* N, 1..HDET_MAX_REPLICAS                                       */
  int32_t  sync_interval;   /* T >= 1                                                        */
  int64_t  total_steps;     /* S >= 1; hdet_fanout_step fails with HDET_ESTATE beyond it     */
  int64_t  warm_steps;      /* S_warm: the controller runs at sync steps with t >= S_warm    */
  double   lr_max;          /* one-cycle peak eta_max                                        */
  double   f_div;           /* initial rate = eta_max / f_div                                */
  double   f_final;         /* final rate   = eta_max / (f_div * f_final)                    */
  double   pct_start;       /* p: fraction of S spent rising                                 */
  int32_t  constant_lr;     /* nonzero: base schedule is eta_max at every step               */
  int32_t  autolr_enabled;  /* nonzero: run the controller of Sec. 3.4                       */
  double   alpha;           /* spread ratio of the learning rate (Eq. 1)                     */
  double   beta;            /* velocity momentum (Eq. 7)                                     */
  double   sigma;           /* softmax temperature (Eq. 4)                                   */
  double   lambda;          /* step of Eq. 7 for the learning rate                           */
  double   gamma_override;  /* >= 0 replaces the decay of Eq. 8; < 0 computes it             */
  int32_t  optimizer;       /* HDET_SGDM or HDET_ADAMW                                       */
  int32_t  grad_mode;       /* HDET_GRAD_SHARED: every replica applies the replica mean of
                               the gradients (the paper's gradient AllReduce);
                               HDET_GRAD_PER_REPLICA: replica r applies its own gradient    */
  int32_t  shared_opt_state;       /* 1 (HDET_ADAMW with HDET_GRAD_SHARED only): the moments
                               depend on the mean gradient alone, so they are the same for every
                               replica and are kept once: opt_m_dev and opt_v_dev are
                               [plane_stride] instead of [N][plane_stride], and a step moves
                               12 N + 16 bytes per element instead of 28 N                   */
  int32_t  reshuffle_every_sync;   /* 0: new permutations only when the controller runs
                               (Algorithm 1), numbered by the controller update k; 1: at every
                               sync step, also before warm_steps or with the controller off
                               (the caption of Fig. 1), numbered by the sync step t / T      */
  double   momentum;        /* SGDM                                                          */
  double   beta1, beta2, eps;      /* AdamW                                                  */
  double   weight_decay;    /* used by all replicas unless a HDET_CH_WD channel exists       */
  int32_t  precision;       /* HDET_FP32 or HDET_BF16_GEMM_FP32_MASTER                       */
  int32_t  model_kind;      /* HDET_FLAT, HDET_MLP or HDET_TRANSFORMER                       */
  hdet_model_dims dims;
  int32_t  n_extra_channels;           /* 0..HDET_MAX_CH - max(n_groups, 1)                  */
  int32_t  n_groups;        /* 0 or 1: one learning-rate channel for all parameters; G > 1:
                               parameter groups with a rate channel each (Sec. 3.4, "random
                               reassignment across hyperparameters": own base rate, velocity
                               and permutation per group, the same one-cycle until hand-over) */
  int64_t  group_end[HDET_MAX_GROUPS]; /* group g is the slice [group_end[g-1], group_end[g]) of a
                               parameter plane; ascending, multiples of 4, the last equals P  */
  hdet_channel extra[HDET_MAX_CH - 1];
  uint64_t seed;            /* keys the permutations of Eq. 9                                */
  void*    stream;          /* hipStream_t, borrowed; NULL = the default stream              */
} hdet_config;

/* Caller-owned device buffers.  Planes are `plane_stride` elements apart; plane_stride >= P
 * and a multiple of 4, every pointer 16-byte aligned (a stride that is a multiple of 64
 * elements and 256-byte aligned pointers put every plane on a cache-line boundary, which the
 * update stream rewards with about 8 % more bandwidth).  Parameter layout inside a plane for
 * HDET_MLP: [W_1 (d_out x d_in, row-major), b_1, W_2, b_2, ...].  For HDET_TRANSFORMER (all
 * row-major): tok_emb [V][d], pos_emb [S][d], then per block ln1_g, ln1_b [d], w_qkv [3d][d],
 * b_qkv [3d], w_o [d][d], b_o [d], ln2_g, ln2_b [d], w_1 [ff][d], b_1 [ff], w_2 [d][ff],
 * b_2 [d], then lnf_g, lnf_b [d], w_head [V][d], b_head [V]; rows 0..d-1 of w_qkv give q,
 * d..2d-1 k, 2d..3d-1 v and head h owns columns h*d/heads .. of each.                       */
typedef struct {
  float*    params_dev;       /* [N][plane_stride] fp32 master parameters, updated in place  */
  float*    grads_dev;        /* [N][plane_stride] fp32; written by hdet_forward_backward;
                                 may be NULL for HDET_FLAT (gradients are passed per step)   */
  float*    opt_m_dev;        /* [N][plane_stride] AdamW first moment / SGD momentum buffer;
                                 must be zero at t = 0 ([plane_stride] with shared_opt_state) */
  float*    opt_v_dev;        /* [N][plane_stride] AdamW second moment; NULL for HDET_SGDM
                                 ([plane_stride] with shared_opt_state)                      */
  uint16_t* params_bf16_dev;  /* [N][plane_stride] bfloat16 copy of the parameters, kept in
                                 step by the update and converge kernels; NULL unless
                                 precision == HDET_BF16_GEMM_FP32_MASTER                     */
  void*     workspace_dev;    /* activations and scratch for hdet_forward_backward           */
  size_t    workspace_bytes;
  int64_t   plane_stride;
} hdet_buffers;

/* Host-side snapshot of the schedule and controller state. */
typedef struct {
  int64_t t;                  /* updates done                                                */
  int64_t k;                  /* controller updates done                                     */
  int32_t controller_active;  /* the controller has taken the base rate over                 */
  int32_t nonfinite;          /* controller calls skipped because a loss was not finite      */
  int32_t n_replicas, n_channels;
  int32_t autolr_done;        /* t is a sync step and hdet_autolr_update has already run on it:
                                 a state saved between hdet_fanout_step and hdet_autolr_update
                                 has 0 here, and the resumed handle still accepts that call     */
  int32_t reserved;
  double  gamma;              /* decay in use for the learning-rate channel                  */
  double  base[HDET_MAX_CH];  /* centre value per channel (rate channels of the groups first,
                                 then the extra channels); rates are meaningful once active  */
  double  vel[HDET_MAX_CH];   /* velocity v of Eq. 7                                         */
  double  delta[HDET_MAX_CH]; /* last hypergradient (Eq. 6)                                  */
  double  w[HDET_MAX_REPLICAS];        /* last softmax weights (Eq. 4)                       */
  double  l_acc[HDET_MAX_REPLICAS];    /* loss accumulated since the last sync step          */
  double  l_last[HDET_MAX_REPLICAS];   /* interval losses L_r seen by the last sync step     */
  float   l_step[HDET_MAX_REPLICAS];   /* losses of the last hdet_forward_backward           */
  float   lr[HDET_MAX_REPLICAS];       /* rates used by the last hdet_fanout_step            */
  double  rho[HDET_MAX_CH][HDET_MAX_REPLICAS];   /* multipliers of Eq. 1 per channel         */
  int32_t perm[HDET_MAX_CH][HDET_MAX_REPLICAS];  /* pi_j(r): replica r uses rho_j[perm]      */
} hdet_state;

/* Bytes the caller must provide: one plane set (N * plane_stride elements) of fp32 for each
 * of params / grads / opt_m / opt_v, of bf16 for the shadow, and the workspace.  Any out
 * pointer may be NULL.  Returns HDET_EINVAL for an invalid configuration.                   */
int hdet_workspace_bytes(const hdet_config* cfg, int64_t plane_stride, size_t* plane_set_bytes,
                         size_t* shadow_bytes, size_t* workspace_bytes);

/* Validates the configuration, computes rho (Eq. 1) and gamma (Eq. 8), sets pi = identity,
 * v = 0, L_acc = 0, t = k = 0 (Algorithm 1, initialisation) and allocates the control block.
 * With HDET_BF16_GEMM_FP32_MASTER the bf16 copy of the parameters is (re)written from
 * params_dev.  Errors: HDET_EINVAL (bad argument, misaligned pointer), HDET_EHIP.           */
int hdet_create(const hdet_config* cfg, const hdet_buffers* buffers, hdet_handle** out);

/* Warm noisy initialisation (Sec. 3.5, Eq. 10): params_dev[r] <- theta0 + eps_r for every
 * replica r, eps_r ~ N(0, nu^2 ||theta0||^2 / P) independently per replica and element (the
 * paper uses nu = 0.01).  theta0_dev: [P] fp32 checkpoint in device memory, 16-byte aligned,
 * not overlapping params_dev.  The noise is a pure function of (seed, replica, index)
 * (Philox-4x32-10 + Box-Muller); the bf16 copy is refreshed.  Only before the first update:
 * HDET_ESTATE once t > 0.                                                                   */
int hdet_warm_init(hdet_handle* h, const float* theta0_dev, double nu, uint64_t seed);

/* For callers that cannot allocate device memory -- code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc: the initialisation of hdet_warm_init without a handle
 * (hdet_create allocates the control block that holds hdet_warm_init's partial sums).  Writes
 * params_dev[r][0..n_params) = theta0 + eps_r for r < n_replicas exactly as hdet_warm_init does
 * for the same (theta0, nu, seed), and, if params_bf16_dev is not NULL, the bfloat16 copy in the
 * same layout.  All pointers are device memory owned by the caller, 16-byte aligned, planes
 * plane_stride elements apart (>= n_params, a multiple of 4); theta0_dev [n_params] must not
 * overlap params_dev; stream: hipStream_t or NULL.  The partial sums of ||theta0||^2 live in a
 * fixed array of 8200 bytes inside the library, one copy per GPU for the life of the process;
 * the call allocates and frees nothing and does not wait for the stream.  Every entry of that
 * array that a call reads it has written before, so nothing carries over from one call to the
 * next; but all calls on one GPU share the array: calls that overlap in time on the same GPU
 * (different streams or threads) race and must be serialised by the caller.
 * Limits: 1 <= n_params <= 2^34, 1 <= n_replicas <= HDET_MAX_REPLICAS; beyond them HDET_EINVAL.
 * Errors: HDET_EINVAL, HDET_EHIP; the message is that of hdet_last_error(NULL).              */
int hdet_warm_init_noalloc(const float* theta0_dev, float* params_dev, uint16_t* params_bf16_dev,
                           int64_t n_params, int64_t plane_stride, int32_t n_replicas, double nu,
                           uint64_t seed, void* stream);

/* Forward, mean cross-entropy and backward of all N replicas on x_dev [N][B][d_in]
 * (fp32; rounded to bf16 on load in bf16 precision) and labels y_dev [N][B] int32 -- for
 * HDET_TRANSFORMER x_dev is token ids [N][B][S] int32 and y_dev the next-token targets
 * [N][B][S] int32, the loss being the mean over the B*S positions
 * ("Forward + backward" of Algorithm 1; the loss is the one that Sec. 3.4 averages into
 * L_r).  With a HDET_CH_DROPOUT channel (Remark 1) replica r drops the two residual
 * branches of every transformer block at its own rate; the mask is a pure function of
 * (seed, step, replica, site, element) from Philox-4x32-10.  With a HDET_CH_LABEL_SMOOTH
 * channel replica r's targets are (1 - eps_r) onehot + eps_r / C (MLP and transformer); with
 * a HDET_CH_ATTN_TEMP channel its attention scores are q.k / (sqrt(d_head) tau_r).  Writes grads_dev, the per-replica losses of this step and adds them to L_acc.
 * If losses_host is not NULL the call waits for the stream and copies the N losses there.
 * HDET_ESTATE for HDET_FLAT handles.                                                        */
int hdet_forward_backward(hdet_handle* h, const void* x_dev, const int32_t* y_dev,
                          float* losses_host);

/* Update t <- t+1 of every replica (Eq. 2 generalised to SGD-momentum / AdamW) with
 * eta_r = eta_bar * rho_{pi(r)} (Eq. 1, Eq. 9), eta_bar being the one-cycle value of
 * schedule index t-1 until the controller has taken over and the controller's base
 * afterwards.  grads_dev: [N][plane_stride] fp32 gradients, or NULL to use the buffer given
 * at creation.  In shared mode the replica mean of the gradients is formed inside the same
 * kernel.  With HDET_FUSE_CONVERGE and t mod T == 0 the replica mean of the updated
 * parameters (Eq. 3) is written to all replicas by the same kernel, and the following
 * hdet_converge is a no-op.  HDET_ESTATE once t == total_steps.                             */
int hdet_fanout_step(hdet_handle* h, const float* grads_dev, uint32_t flags);

/* One whole step of Algorithm 1's inner loop in a single call: forward, loss and backward on
 * (x_dev, y_dev) as hdet_forward_backward does, then update t <- t+1 (Sec. 3.2, Eq. 1-2) as
 * hdet_fanout_step(h, NULL, flags) does.  Parameters, optimizer state, bfloat16 copy, losses and
 * schedule state after the call are those of the two separate calls, bit for bit.  The gradient
 * buffer given at creation is still required but is NOT a defined output of this call: with
 * HDET_BF16_GEMM_FP32_MASTER, HDET_ADAMW, HDET_GRAD_PER_REPLICA and per-replica moments the
 * update of a weight matrix is applied inside the product that forms its gradient (every
 * replica's tile of dW is complete in one block, so Eq. 2 can be applied to it at once), and
 * that gradient is never written to memory: 26 instead of 30 + 4 bytes per weight and replica.
 * Biases, LayerNorm parameters, embeddings and matrices too small for this to pay (see
 * hdet_set_launch_shape), and every configuration outside the one named, take the ordinary
 * update.  With HDET_FUSE_CONVERGE on a sync step the replica mean of Eq. 3
 * is formed after all updates (by the update kernel, or by the converge kernel when some
 * updates were applied inside products), and the following hdet_converge is a no-op.
 * losses_host as for hdet_forward_backward.  HDET_ESTATE for HDET_FLAT handles and once
 * t == total_steps.                                                                          */
int hdet_train_step(hdet_handle* h, const void* x_dev, const int32_t* y_dev, uint32_t flags,
                    float* losses_host);

/* theta_r <- (1/N) sum_r' theta_r' for all r (Eq. 3), summed in the order r' = 0..N-1;
 * optimizer state is left per replica.  May be called at any t (Algorithm 1 calls it when
 * t mod T == 0; a caller whose S is not a multiple of T ends with one more call).           */
int hdet_converge(hdet_handle* h);

/* Sync-step bookkeeping (Algorithm 1, inside "t mod T = 0"): L_r = L_acc / T -- or the N
 * host values given in interval_losses_host -- then L_acc <- 0; if the controller is
 * enabled and t >= S_warm: weights (Eq. 4), hypergradient per channel (Eq. 5-6), velocity
 * and base (Eq. 7-8), fresh permutations (Eq. 9).  Runs on the device in one wavefront.
 * A non-finite loss leaves the controller state untouched (L_acc is still reset, the sync
 * step still counts as processed) and increments hdet_state.nonfinite.  When the losses come
 * from the host (interval_losses_host != NULL, N doubles) and the controller was due, the
 * call then returns HDET_ENONFINITE; with device-accumulated losses the call does not wait
 * for the stream, so it returns HDET_OK and the caller sees the event in the counter of the
 * next hdet_get_state.  HDET_ESTATE off a sync step or twice on the same one.               */
int hdet_autolr_update(hdet_handle* h, const double* interval_losses_host);

/* Waits for the stream and copies the state out / overwrites it (resume).                   */
int hdet_get_state(hdet_handle* h, hdet_state* out);
int hdet_set_state(hdet_handle* h, const hdet_state* in);

/* Kernel selection, for measurements and tests.  variant 0 (default): the fastest update
 * kernel for the case (one thread per replica column, or -- when gradients or parameters
 * must cross the replica axis and N <= 16 -- one wavefront per replica with an LDS
 * exchange); variant 1: the general kernel in which one thread walks the replica axis (any
 * N).  `blocks` > 0 sets the grid of the grid-stride kernels (0: library default).
 * variant | 2: the transformer's attention runs as separate batched GEMMs and softmax
 * kernels (scores and probabilities in device memory) also where the fused kernels apply.
 * variant | 4: hdet_train_step applies the update inside every weight-gradient product that
 * can carry it; by default only inside products with at least one 256 x 256 tile per
 * compute unit (the update of a smaller matrix is faster as part of the plane-wide launch).  */
int hdet_set_launch_shape(hdet_handle* h, int32_t variant, int32_t blocks);

/* Message of the last failure on this handle (or of the last failed hdet_create if h is
 * NULL); owned by the library.                                                              */
const char* hdet_last_error(hdet_handle* h);

/* Releases the control block and the handle.  hdet_destroy(NULL) is a no-op.                */
int hdet_destroy(hdet_handle* h);

#ifdef __cplusplus
}
#endif
#endif /* HDET_H */

// C-ABI entry points of libhdet.so and the host-side part of Algorithm 1: argument
// validation, the step counter, the one-cycle base schedule, Eq. 1 and Eq. 8.
// Everything that touches the N*P parameter planes or the controller state runs in the
// kernels of hdet_update.hip / hdet_controller.hip / hdet_mlp.hip.

#include <math.h>
#include <string.h>

#include <algorithm>
#include <cmath>

#include <new>

#include "hdet_internal.h"

namespace {

thread_local std::string g_create_error;

int fail(hdet_handle* h, int code, const std::string& msg) {
  if (h) h->err = msg; else g_create_error = msg;
  return code;
}

int hip_fail(hdet_handle* h, hipError_t e, const char* what) {
  return fail(h, HDET_EHIP, std::string(what) + ": " + hipGetErrorString(e));
}

// Two-phase cosine one-cycle policy with parameters (eta_max, f_div, f_final, p)
// (Algorithm 1, Require): eta rises from eta_max/f_div to eta_max over schedule indices
// 0 .. p*S-1 and falls to eta_max/(f_div*f_final) at index S-1.
double onecycle(const hdet_config& c, int64_t idx) {
  if (c.constant_lr) return c.lr_max;
  const double lr_init = c.lr_max / c.f_div;
  const double lr_min = lr_init / c.f_final;
  const double end1 = c.pct_start * (double)c.total_steps - 1.0;
  const double end2 = (double)c.total_steps - 1.0;
  const double x = (double)idx;
  double start, end, pct;
  if (x <= end1) {
    start = lr_init; end = c.lr_max;
    pct = end1 > 0.0 ? x / end1 : 1.0;
  } else {
    start = c.lr_max; end = lr_min;
    const double span = end2 - end1;
    pct = span > 0.0 ? (x - end1) / span : 1.0;
  }
  return end + (start - end) / 2.0 * (1.0 + cos(M_PI * pct));
}

// Eq. 8, read so that K = (S - S_warm)/T controller updates take eta_max down to the
// one-cycle floor: (1 - gamma)^K = 1 / (f_div * f_final).
double decay_gamma(const hdet_config& c) {
  if (c.gamma_override >= 0.0) return c.gamma_override;
  const double k_sync = (double)(c.total_steps - c.warm_steps) / (double)c.sync_interval;
  if (k_sync <= 0.0) return 0.0;
  return 1.0 - exp(-log(c.f_div * c.f_final) / k_sync);
}

// Eq. 1
void spread(int n, double alpha, double* rho) {
  const double centre = (n - 1) / 2.0;
  const double delta = centre > 0.5 ? centre : 0.5;
  for (int r = 0; r < n; ++r) rho[r] = 1.0 + alpha * (((double)r - centre) / delta);
}

int64_t param_count(const hdet_config& c) {
  if (c.model_kind == HDET_FLAT) return c.dims.n_params;
  if (c.model_kind == HDET_TRANSFORMER) return hdet_tf_param_count(c);
  int64_t p = 0;
  for (int i = 0; i < c.dims.n_layers; ++i)
    p += (int64_t)c.dims.widths[i + 1] * c.dims.widths[i] + c.dims.widths[i + 1];
  return p;
}

int validate(const hdet_config* c, std::string* why) {
  auto bad = [&](const char* m) { *why = m; return HDET_EINVAL; };
  if (!c) return bad("config is NULL");
  if (c->n_replicas < 1 || c->n_replicas > HDET_MAX_REPLICAS) return bad("n_replicas out of range");
  if (c->sync_interval < 1) return bad("sync_interval must be >= 1");
  if (c->total_steps < 1) return bad("total_steps must be >= 1");
  if (c->warm_steps < 0) return bad("warm_steps must be >= 0");
  if (!(c->lr_max > 0.0) || !(c->f_div > 0.0) || !(c->f_final > 0.0)) return bad("lr_max, f_div, f_final must be > 0");
  if (!(c->pct_start > 0.0 && c->pct_start <= 1.0)) return bad("pct_start must be in (0, 1]");
  if (!(c->alpha >= 0.0 && c->alpha <= 1.0)) return bad("alpha must be in [0, 1]");
  if (c->autolr_enabled && (!(c->sigma > 0.0) || !(c->beta >= 0.0 && c->beta < 1.0))) return bad("sigma must be > 0 and beta in [0, 1)");
  if (c->optimizer != HDET_SGDM && c->optimizer != HDET_ADAMW) return bad("unknown optimizer");
  if (c->grad_mode != HDET_GRAD_SHARED && c->grad_mode != HDET_GRAD_PER_REPLICA) return bad("unknown grad_mode");
  if (c->precision != HDET_FP32 && c->precision != HDET_BF16_GEMM_FP32_MASTER) return bad("unknown precision");
  if (c->optimizer == HDET_ADAMW && (!(c->beta1 >= 0.0 && c->beta1 < 1.0) || !(c->beta2 >= 0.0 && c->beta2 < 1.0) || !(c->eps > 0.0)))
    return bad("AdamW needs beta1, beta2 in [0, 1) and eps > 0");
  if (c->model_kind == HDET_FLAT) {
    if (c->dims.n_params < 1) return bad("n_params must be >= 1");
  } else if (c->model_kind == HDET_MLP) {
    if (c->dims.n_layers < 1 || c->dims.n_layers > HDET_MAX_LAYERS) return bad("n_layers out of range");
    if (c->dims.batch < 1) return bad("batch must be >= 1");
    for (int i = 0; i <= c->dims.n_layers; ++i)
      if (c->dims.widths[i] < 1) return bad("layer widths must be >= 1");
  } else if (c->model_kind == HDET_TRANSFORMER) {
    const int rc = hdet_tf_validate(*c, why);
    if (rc != HDET_OK) return rc;
  } else {
    return bad("unknown model_kind");
  }
  if (c->n_groups < 0 || c->n_groups > HDET_MAX_GROUPS) return bad("n_groups out of range");
  const int n_lr = c->n_groups > 1 ? c->n_groups : 1;
  if (c->n_extra_channels < 0 || c->n_extra_channels > HDET_MAX_CH - n_lr) return bad("n_extra_channels out of range");
  if (c->n_groups > 1) {
    const int64_t p = param_count(*c);
    int64_t prev = 0;
    for (int g = 0; g < c->n_groups; ++g) {
      const int64_t e = c->group_end[g];
      if (e <= prev || e > p || (g + 1 < c->n_groups && (e & 3))) return bad("group_end must ascend in multiples of 4 up to P");
      prev = e;
    }
    if (prev != p) return bad("the last group_end must equal P");
  }
  int seen[5] = {0, 0, 0, 0, 0};
  for (int j = 0; j < c->n_extra_channels; ++j) {
    const hdet_channel& ch = c->extra[j];
    if (ch.kind != HDET_CH_WD && ch.kind != HDET_CH_DROPOUT && ch.kind != HDET_CH_LABEL_SMOOTH && ch.kind != HDET_CH_ATTN_TEMP)
      return bad("extra channel kind must be HDET_CH_DROPOUT, HDET_CH_WD, HDET_CH_LABEL_SMOOTH or HDET_CH_ATTN_TEMP");
    if (++seen[ch.kind] > 1) return bad("at most one channel per kind");
    if (!(ch.alpha >= 0.0 && ch.alpha <= 1.0) || !(ch.lo >= 0.0) || !(ch.lo <= ch.base && ch.base <= ch.hi))
      return bad("extra channel needs alpha in [0, 1] and 0 <= lo <= base <= hi");
    // the controller clamps the centre value to [lo, hi] (Eq. 7); replica r then uses centre * rho_pi(r) with rho in
    // [1 - alpha, 1 + alpha] (Eq. 1, Eq. 9), so the bounds below hold for every value a kernel can read
    if (ch.kind == HDET_CH_DROPOUT && !(ch.hi * (1.0 + ch.alpha) < 1.0))
      return bad("dropout needs hi * (1 + alpha) < 1");
    if (ch.kind == HDET_CH_LABEL_SMOOTH && (c->model_kind == HDET_FLAT || !(ch.hi * (1.0 + ch.alpha) <= 1.0)))
      return bad("label smoothing needs a model and hi * (1 + alpha) <= 1");
    if (ch.kind == HDET_CH_ATTN_TEMP && (c->model_kind != HDET_TRANSFORMER || !(ch.lo * (1.0 - ch.alpha) > 0.0)))
      return bad("attention temperature needs a transformer and lo * (1 - alpha) > 0");
  }
  if (c->shared_opt_state != 0 && c->shared_opt_state != 1) return bad("shared_opt_state must be 0 or 1");
  if (c->shared_opt_state && (c->optimizer != HDET_ADAMW || c->grad_mode != HDET_GRAD_SHARED))
    return bad("shared_opt_state needs HDET_ADAMW with HDET_GRAD_SHARED");
  if (c->reshuffle_every_sync != 0 && c->reshuffle_every_sync != 1) return bad("reshuffle_every_sync must be 0 or 1");
  return HDET_OK;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int default_blocks(const hdet_handle* h) { return h->tune_blocks > 0 ? h->tune_blocks : h->n_cu * 16; }

void fill_ctrl_initial(const hdet_handle* h, hdet_ctrl* c) {
  memset(c, 0, sizeof(*c));
  const int n = h->cfg.n_replicas;
  for (int j = 0; j < h->n_channels; ++j) {
    spread(n, h->channels[j].alpha, c->rho[j]);
    c->base[j] = h->channels[j].base;
    for (int r = 0; r < n; ++r) c->perm[j][r] = r;
  }
  for (int r = 0; r < n; ++r) c->w[r] = 1.0 / n;
  c->n_lr = h->n_lr;
}

int upload_ctrl(hdet_handle* h, const hdet_ctrl& c) {
  hipError_t e = hipMemcpyAsync(h->ctrl_dev, &c, sizeof(c), hipMemcpyHostToDevice, h->stream);
  if (e != hipSuccess) return hip_fail(h, e, "hipMemcpyAsync(control block)");
  e = hipStreamSynchronize(h->stream);
  if (e != hipSuccess) return hip_fail(h, e, "hipStreamSynchronize");
  return HDET_OK;
}

int write_shadow(hdet_handle* h) {
  if (h->cfg.precision != HDET_BF16_GEMM_FP32_MASTER) return HDET_OK;
  hipError_t e = hdet_launch_shadow(h->buf.params_dev, h->buf.params_bf16_dev, param_count(h->cfg),
                                    h->buf.plane_stride, h->cfg.n_replicas, default_blocks(h), h->stream);
  if (e != hipSuccess) return hip_fail(h, e, "bf16 copy kernel");
  return HDET_OK;
}

}  // namespace

void hdet_set_global_error(const std::string& msg) { g_create_error = msg; }

extern "C" {

int hdet_workspace_bytes(const hdet_config* cfg, int64_t plane_stride, size_t* plane_set_bytes,
                         size_t* shadow_bytes, size_t* workspace_bytes) {
  std::string why;
  int rc = validate(cfg, &why);
  if (rc != HDET_OK) return fail(nullptr, rc, why);
  const int64_t p = param_count(*cfg);
  if (plane_stride < p || (plane_stride & 3)) return fail(nullptr, HDET_EINVAL, "plane_stride must be >= P and a multiple of 4");
  const size_t elems = (size_t)cfg->n_replicas * (size_t)plane_stride;
  if (plane_set_bytes) *plane_set_bytes = elems * sizeof(float);
  if (shadow_bytes) *shadow_bytes = cfg->precision == HDET_BF16_GEMM_FP32_MASTER ? elems * sizeof(uint16_t) : 0;
  size_t ws = 0;
  if (cfg->model_kind == HDET_MLP) rc = hdet_mlp_workspace_bytes(*cfg, &ws, &why);
  if (cfg->model_kind == HDET_TRANSFORMER) rc = hdet_tf_workspace_bytes(*cfg, &ws, &why);
  if (rc != HDET_OK) return fail(nullptr, rc, why);
  if (workspace_bytes) *workspace_bytes = ws;
  return HDET_OK;
}

int hdet_create(const hdet_config* cfg, const hdet_buffers* b, hdet_handle** out) {
  if (!out) return fail(nullptr, HDET_EINVAL, "out is NULL");
  *out = nullptr;
  std::string why;
  int rc = validate(cfg, &why);
  if (rc != HDET_OK) return fail(nullptr, rc, why);
  if (!b) return fail(nullptr, HDET_EINVAL, "buffers is NULL");
  const int64_t p = param_count(*cfg);
  if (b->plane_stride < p || (b->plane_stride & 3)) return fail(nullptr, HDET_EINVAL, "plane_stride must be >= P and a multiple of 4");
  if (!b->params_dev || !b->opt_m_dev) return fail(nullptr, HDET_EINVAL, "params_dev and opt_m_dev are required");
  if (cfg->optimizer == HDET_ADAMW && !b->opt_v_dev) return fail(nullptr, HDET_EINVAL, "opt_v_dev is required for AdamW");
  if (cfg->precision == HDET_BF16_GEMM_FP32_MASTER && !b->params_bf16_dev) return fail(nullptr, HDET_EINVAL, "params_bf16_dev is required in bf16 precision");
  if (cfg->model_kind != HDET_FLAT && !b->grads_dev) return fail(nullptr, HDET_EINVAL, "grads_dev is required for model handles");
  if (!aligned16(b->params_dev) || !aligned16(b->opt_m_dev) || !aligned16(b->opt_v_dev) ||
      !aligned16(b->grads_dev) || !aligned16(b->params_bf16_dev) || !aligned16(b->workspace_dev))
    return fail(nullptr, HDET_EINVAL, "device pointers must be 16-byte aligned");

  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(nullptr, e, "hipGetDevice (no HIP device: there is no CPU fallback)");
  hipDeviceProp_t prop;
  e = hipGetDeviceProperties(&prop, dev);
  if (e != hipSuccess) return hip_fail(nullptr, e, "hipGetDeviceProperties");

  hdet_handle* h = new (std::nothrow) hdet_handle();
  if (!h) return fail(nullptr, HDET_EINVAL, "out of host memory");
  h->cfg = *cfg;
  h->buf = *b;
  h->stream = (hipStream_t)cfg->stream;
  h->device = dev;
  h->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  h->t = 0;
  h->last_autolr_t = 0;
  h->converged_at_t = -1;
  h->gamma = decay_gamma(*cfg);
  h->tune_variant = 0;
  h->fuse_everything = false;
  h->tune_blocks = 0;
  h->mlp = nullptr;
  h->tf = nullptr;
  h->drop_channel = -1;
  h->ls_channel = -1;
  h->temp_channel = -1;
  h->ctrl_dev = nullptr;
  h->n_lr = cfg->n_groups > 1 ? cfg->n_groups : 1;
  h->n_channels = h->n_lr + cfg->n_extra_channels;
  h->wd_channel = -1;
  memset(h->channels, 0, sizeof(h->channels));
  for (int g = 0; g < h->n_lr; ++g) {
    h->channels[g].kind = HDET_CH_LR;
    h->channels[g].base = cfg->lr_max;
    h->channels[g].alpha = cfg->alpha;
    h->channels[g].lambda = cfg->lambda;
    h->channels[g].lo = 0.0;
    h->channels[g].hi = INFINITY;
  }
  for (int j = 0; j < cfg->n_extra_channels; ++j) {
    h->channels[h->n_lr + j] = cfg->extra[j];
    if (cfg->extra[j].kind == HDET_CH_WD) h->wd_channel = h->n_lr + j;
    if (cfg->extra[j].kind == HDET_CH_DROPOUT) h->drop_channel = h->n_lr + j;
    if (cfg->extra[j].kind == HDET_CH_LABEL_SMOOTH) h->ls_channel = h->n_lr + j;
    if (cfg->extra[j].kind == HDET_CH_ATTN_TEMP) h->temp_channel = h->n_lr + j;
  }

  e = hipMalloc((void**)&h->ctrl_dev, sizeof(hdet_ctrl));
  if (e != hipSuccess) { rc = hip_fail(nullptr, e, "hipMalloc(control block)"); delete h; return rc; }
  hdet_ctrl c;
  fill_ctrl_initial(h, &c);
  rc = upload_ctrl(h, c);
  if (rc == HDET_OK) rc = write_shadow(h);
  if (rc == HDET_OK && cfg->model_kind == HDET_MLP) {
    h->mlp = hdet_mlp_create(h->cfg, h->buf, h->ls_channel, &why);
    if (!h->mlp) { h->err = why; rc = HDET_EINVAL; }
  }
  if (rc == HDET_OK && cfg->model_kind == HDET_TRANSFORMER) {
    h->tf = hdet_tf_create(h->cfg, h->buf, h->drop_channel, h->ls_channel, h->temp_channel, &why);
    if (!h->tf) { h->err = why; rc = HDET_EINVAL; }
  }
  if (rc != HDET_OK) {
    g_create_error = h->err;
    (void)hipFree(h->ctrl_dev);
    delete h;
    return rc;
  }
  *out = h;
  return HDET_OK;
}

int hdet_forward_backward(hdet_handle* h, const void* x_dev, const int32_t* y_dev, float* losses_host) {
  if (!h) return fail(nullptr, HDET_EINVAL, "handle is NULL");
  if (h->cfg.model_kind == HDET_FLAT || (!h->mlp && !h->tf)) return fail(h, HDET_ESTATE, "flat handles have no forward/backward");
  if (!x_dev || !y_dev) return fail(h, HDET_EINVAL, "x_dev and y_dev are required");
  if (!aligned16(x_dev)) return fail(h, HDET_EINVAL, "x_dev must be 16-byte aligned");
  hipError_t e = h->tf ? hdet_tf_forward_backward(h->tf, (const int32_t*)x_dev, y_dev, h->ctrl_dev, (uint32_t)(h->t + 1), h->stream)
                       : hdet_mlp_forward_backward(h->mlp, x_dev, y_dev, h->ctrl_dev, h->stream);
  if (e != hipSuccess) return hip_fail(h, e, "forward/backward kernels");
  if (losses_host) {
    e = hipMemcpyAsync(losses_host, h->ctrl_dev->l_step, sizeof(float) * h->cfg.n_replicas,
                       hipMemcpyDeviceToHost, h->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(h->stream);
    if (e != hipSuccess) return hip_fail(h, e, "copy of the step losses");
  }
  return HDET_OK;
}

int hdet_warm_init(hdet_handle* h, const float* theta0_dev, double nu, uint64_t seed) {
  if (!h) return fail(nullptr, HDET_EINVAL, "handle is NULL");
  if (h->t != 0) return fail(h, HDET_ESTATE, "hdet_warm_init is only allowed before the first update");
  if (!theta0_dev || !aligned16(theta0_dev)) return fail(h, HDET_EINVAL, "theta0_dev must be a 16-byte aligned device pointer");
  if (!(nu >= 0.0)) return fail(h, HDET_EINVAL, "nu must be >= 0");
  const int64_t p = param_count(h->cfg);
  const float* lo = h->buf.params_dev;
  const float* hi = lo + (int64_t)h->cfg.n_replicas * h->buf.plane_stride;
  if (theta0_dev + p > lo && theta0_dev < hi) return fail(h, HDET_EINVAL, "theta0_dev must not overlap params_dev");
  if (p > HDET_WARM_MAX_PARAMS) return fail(h, HDET_EINVAL, "hdet_warm_init takes at most 2^34 parameters per replica");
  hipError_t e = hdet_launch_warm_init(theta0_dev, h->buf.params_dev, p, h->buf.plane_stride, h->cfg.n_replicas,
                                       h->ctrl_dev->warm_partial, &h->ctrl_dev->warm_sumsq, nu, seed, h->stream);
  if (e != hipSuccess) return hip_fail(h, e, "warm initialisation kernels");
  return write_shadow(h);
}

namespace {

// Arguments of update t (1-based) over the whole plane, with the gradients at g.
void fill_update_args(const hdet_handle* h, int64_t t, const float* g, hdet_update_args* out) {
  const hdet_config& c = h->cfg;
  hdet_update_args a;
  memset(&a, 0, sizeof(a));
  a.theta = h->buf.params_dev;
  a.grad = g;
  a.m = h->buf.opt_m_dev;
  a.v = h->buf.opt_v_dev;
  a.shadow = c.precision == HDET_BF16_GEMM_FP32_MASTER ? h->buf.params_bf16_dev : nullptr;
  a.ctrl = h->ctrl_dev;
  a.ctrl_out = h->ctrl_dev;
  a.n_params = param_count(c);
  a.stride = h->buf.plane_stride;
  a.grad_stride = a.stride;
  a.grad_scale = 1.f;
  a.n_replicas = c.n_replicas;
  a.wd_channel = h->wd_channel;
  a.first_step = t == 1;
  a.shared_state = c.shared_opt_state;
  a.eta_sched = onecycle(c, t - 1);        // update t uses schedule index t-1
  a.wd_const = c.weight_decay;
  const double bc1 = 1.0 - pow(c.beta1, (double)t);
  const double bc2 = 1.0 - pow(c.beta2, (double)t);
  a.inv_bc1 = c.optimizer == HDET_ADAMW ? 1.0 / bc1 : 1.0;
  a.inv_sqrt_bc2 = c.optimizer == HDET_ADAMW ? (float)(1.0 / sqrt(bc2)) : 1.f;
  a.beta1 = (float)c.beta1;
  a.beta2 = (float)c.beta2;
  a.one_m_beta1 = (float)(1.0 - c.beta1);
  a.one_m_beta2 = (float)(1.0 - c.beta2);
  a.eps = (float)c.eps;
  a.momentum = (float)c.momentum;
  *out = a;
}

enum slice_kind { kSummed, kDone };

// One launch per parameter group and kind of slice: the slice of every plane with the group's rate channel.
// `special` (ascending, disjoint): slices whose gradient is one plane holding the sum over the replicas (kSummed: read
// with plane stride 0 and scaled by 1 / N), or whose update has already been applied (kDone: skipped).
int launch_updates(hdet_handle* h, const hdet_update_args& a, const hdet_slices& special, slice_kind kind, bool fuse_converge) {
  const hdet_config& c = h->cfg;
  const bool shared = c.grad_mode == HDET_GRAD_SHARED;
  int64_t begin = 0;
  size_t si = 0;
  for (int grp = 0; grp < h->n_lr; ++grp) {
    const int64_t gend = h->n_lr > 1 ? c.group_end[grp] : a.n_params;
    while (begin < gend) {
      while (si < special.size() && special[si].first + special[si].second <= begin) ++si;
      const bool in_special = si < special.size() && special[si].first <= begin;
      int64_t end = gend;
      if (in_special) end = std::min(end, special[si].first + special[si].second);
      else if (si < special.size()) end = std::min(end, special[si].first);
      if (!(in_special && kind == kDone)) {
        hdet_update_args ga = a;
        ga.theta += begin; ga.grad += begin; ga.m += begin;
        if (ga.v) ga.v += begin;
        if (ga.shadow) ga.shadow += begin;
        ga.n_params = end - begin;
        ga.lr_channel = grp;
        if (in_special) {
          ga.grad_stride = 0;
          ga.grad_scale = (float)(1.0 / (double)c.n_replicas);
        }
        // identical gradients need no mean over the replicas, except that one set of moments is built on that kernel
        const bool mean = shared && (!in_special || c.shared_opt_state);
        hipError_t e = hdet_launch_update(ga, c.optimizer, mean, fuse_converge, h->tune_variant, default_blocks(h), h->stream);
        if (e != hipSuccess) return hip_fail(h, e, "update kernel");
      }
      begin = end;
    }
  }
  return HDET_OK;
}

int launch_converge(hdet_handle* h) {
  hdet_converge_args a;
  a.theta = h->buf.params_dev;
  a.shadow = h->cfg.precision == HDET_BF16_GEMM_FP32_MASTER ? h->buf.params_bf16_dev : nullptr;
  a.n_params = param_count(h->cfg);
  a.stride = h->buf.plane_stride;
  a.n_replicas = h->cfg.n_replicas;
  a.tail_only = 0;
  hipError_t e = hdet_launch_converge(a, h->tune_variant, default_blocks(h), h->stream);
  if (e != hipSuccess) return hip_fail(h, e, "converge kernel");
  h->converged_at_t = h->t;
  return HDET_OK;
}

}  // namespace

int hdet_fanout_step(hdet_handle* h, const float* grads_dev, uint32_t flags) {
  if (!h) return fail(nullptr, HDET_EINVAL, "handle is NULL");
  if (flags & ~HDET_FUSE_CONVERGE) return fail(h, HDET_EINVAL, "unknown flag");
  const float* g = grads_dev ? grads_dev : h->buf.grads_dev;
  if (!g) return fail(h, HDET_EINVAL, "no gradient buffer");
  if (!aligned16(g)) return fail(h, HDET_EINVAL, "grads_dev must be 16-byte aligned");
  const hdet_config& c = h->cfg;
  if (h->t >= c.total_steps) return fail(h, HDET_ESTATE, "all total_steps updates are done");
  const int64_t t = h->t + 1;
  hdet_update_args a;
  fill_update_args(h, t, g, &a);
  const bool fuse = (flags & HDET_FUSE_CONVERGE) && (t % c.sync_interval == 0);
  // A model handle in shared-gradient mode leaves some slices of the plane as one sum over the replicas (plane 0 of its
  // gradient buffer) and the rest as one gradient per replica; either way the kernel applies the replica mean.
  hdet_slices summed;
  const bool shared = c.grad_mode == HDET_GRAD_SHARED;
  if (!grads_dev && shared && c.model_kind == HDET_MLP) summed.push_back({0, a.n_params});
  if (!grads_dev && shared && c.model_kind == HDET_TRANSFORMER) hdet_tf_summed_slices(h->tf, &summed);
  if (int rc = launch_updates(h, a, summed, kSummed, fuse)) return rc;
  h->t = t;
  if (fuse) h->converged_at_t = t;
  return HDET_OK;
}

int hdet_train_step(hdet_handle* h, const void* x_dev, const int32_t* y_dev, uint32_t flags, float* losses_host) {
  if (!h) return fail(nullptr, HDET_EINVAL, "handle is NULL");
  if (flags & ~HDET_FUSE_CONVERGE) return fail(h, HDET_EINVAL, "unknown flag");
  const hdet_config& c = h->cfg;
  if (c.model_kind == HDET_FLAT || (!h->mlp && !h->tf)) return fail(h, HDET_ESTATE, "flat handles have no forward/backward");
  if (!x_dev || !y_dev) return fail(h, HDET_EINVAL, "x_dev and y_dev are required");
  if (!aligned16(x_dev)) return fail(h, HDET_EINVAL, "x_dev must be 16-byte aligned");
  if (!h->buf.grads_dev) return fail(h, HDET_EINVAL, "no gradient buffer");
  if (h->t >= c.total_steps) return fail(h, HDET_ESTATE, "all total_steps updates are done");
  const int64_t t = h->t + 1;
  hdet_update_args a;
  fill_update_args(h, t, h->buf.grads_dev, &a);
  a.fuse_min_tiles = h->fuse_everything ? 0 : h->n_cu;
  // the weight matrices' updates go into the products that form their gradients where the arithmetic allows it
  const bool can_fuse = c.precision == HDET_BF16_GEMM_FP32_MASTER && c.optimizer == HDET_ADAMW &&
                        c.grad_mode == HDET_GRAD_PER_REPLICA && !c.shared_opt_state;
  hdet_slices done;
  hipError_t e = h->tf ? hdet_tf_forward_backward(h->tf, (const int32_t*)x_dev, y_dev, h->ctrl_dev, (uint32_t)t, h->stream,
                                                  can_fuse ? &a : nullptr, can_fuse ? &done : nullptr)
                       : hdet_mlp_forward_backward(h->mlp, x_dev, y_dev, h->ctrl_dev, h->stream, can_fuse ? &a : nullptr,
                                                   can_fuse ? &done : nullptr);
  if (e != hipSuccess) return hip_fail(h, e, "forward/backward kernels");
  std::sort(done.begin(), done.end());
  const bool sync = (flags & HDET_FUSE_CONVERGE) && (t % c.sync_interval == 0);
  int rc;
  if (done.empty()) {
    hdet_slices summed;
    const bool shared = c.grad_mode == HDET_GRAD_SHARED;
    if (shared && c.model_kind == HDET_MLP) summed.push_back({0, a.n_params});
    if (shared && c.model_kind == HDET_TRANSFORMER) hdet_tf_summed_slices(h->tf, &summed);
    rc = launch_updates(h, a, summed, kSummed, sync);
    if (rc != HDET_OK) return rc;
    h->t = t;
    if (sync) h->converged_at_t = t;
  } else {
    // the rest of the plane; the converge of a sync step then runs over the whole plane on its own
    rc = launch_updates(h, a, done, kDone, false);
    if (rc != HDET_OK) return rc;
    h->t = t;
    if (sync && (rc = launch_converge(h)) != HDET_OK) return rc;
  }
  if (losses_host) {
    e = hipMemcpyAsync(losses_host, h->ctrl_dev->l_step, sizeof(float) * c.n_replicas, hipMemcpyDeviceToHost, h->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(h->stream);
    if (e != hipSuccess) return hip_fail(h, e, "copy of the step losses");
  }
  return HDET_OK;
}

int hdet_converge(hdet_handle* h) {
  if (!h) return fail(nullptr, HDET_EINVAL, "handle is NULL");
  if (h->converged_at_t == h->t) return HDET_OK;     // already averaged by the fused update
  return launch_converge(h);
}

int hdet_autolr_update(hdet_handle* h, const double* interval_losses_host) {
  if (!h) return fail(nullptr, HDET_EINVAL, "handle is NULL");
  const hdet_config& c = h->cfg;
  if (h->t == 0 || h->t % c.sync_interval != 0) return fail(h, HDET_ESTATE, "hdet_autolr_update off a sync step");
  if (h->last_autolr_t == h->t) return fail(h, HDET_ESTATE, "hdet_autolr_update called twice on one sync step");
  hdet_controller_args a;
  memset(&a, 0, sizeof(a));
  a.ctrl = h->ctrl_dev;
  a.use_injected = interval_losses_host != nullptr;
  bool nonfinite = false;
  if (interval_losses_host)
    for (int r = 0; r < c.n_replicas; ++r) {
      a.injected[r] = interval_losses_host[r];
      nonfinite = nonfinite || !std::isfinite(interval_losses_host[r]);
    }
  a.run_controller = c.autolr_enabled && h->t >= c.warm_steps;
  a.n_replicas = c.n_replicas;
  a.n_channels = h->n_channels;
  a.n_lr = h->n_lr;
  a.sync_interval = c.sync_interval;
  a.eta_sched = onecycle(c, h->t - 1);
  a.sigma = c.sigma;
  a.beta = c.beta;
  a.gamma = h->gamma;
  for (int j = 0; j < h->n_channels; ++j) {
    a.lambda[j] = h->channels[j].lambda;
    a.lo[j] = h->channels[j].lo;
    a.hi[j] = h->channels[j].hi;
  }
  a.reshuffle = c.reshuffle_every_sync;
  a.sync_index = (uint32_t)(h->t / c.sync_interval);
  a.seed_lo = (uint32_t)(c.seed & 0xffffffffu);
  a.seed_hi = (uint32_t)(c.seed >> 32);
  hipError_t e = hdet_launch_controller(a, h->stream);
  if (e != hipSuccess) return hip_fail(h, e, "controller kernel");
  h->last_autolr_t = h->t;
  // the kernel has left the controller state untouched and counted the event
  if (nonfinite && a.run_controller) return fail(h, HDET_ENONFINITE, "an interval loss is not finite: controller state left untouched");
  return HDET_OK;
}

int hdet_get_state(hdet_handle* h, hdet_state* out) {
  if (!h) return fail(nullptr, HDET_EINVAL, "handle is NULL");
  if (!out) return fail(h, HDET_EINVAL, "out is NULL");
  hdet_ctrl c;
  hipError_t e = hipMemcpyAsync(&c, h->ctrl_dev, sizeof(c), hipMemcpyDeviceToHost, h->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(h->stream);
  if (e != hipSuccess) return hip_fail(h, e, "copy of the control block");
  memset(out, 0, sizeof(*out));
  out->t = h->t;
  out->k = c.k;
  out->controller_active = c.controller_active;
  out->nonfinite = c.nonfinite;
  out->n_replicas = h->cfg.n_replicas;
  out->n_channels = h->n_channels;
  out->autolr_done = h->t > 0 && h->last_autolr_t == h->t;
  out->gamma = h->gamma;
  memcpy(out->base, c.base, sizeof(c.base));
  memcpy(out->vel, c.vel, sizeof(c.vel));
  memcpy(out->delta, c.delta, sizeof(c.delta));
  memcpy(out->w, c.w, sizeof(c.w));
  memcpy(out->l_acc, c.l_acc, sizeof(c.l_acc));
  memcpy(out->l_last, c.l_last, sizeof(c.l_last));
  memcpy(out->l_step, c.l_step, sizeof(c.l_step));
  memcpy(out->lr, c.lr_used, sizeof(c.lr_used));
  memcpy(out->rho, c.rho, sizeof(c.rho));
  memcpy(out->perm, c.perm, sizeof(c.perm));
  return HDET_OK;
}

int hdet_set_state(hdet_handle* h, const hdet_state* in) {
  if (!h) return fail(nullptr, HDET_EINVAL, "handle is NULL");
  if (!in) return fail(h, HDET_EINVAL, "state is NULL");
  if (in->n_replicas != h->cfg.n_replicas || in->n_channels != h->n_channels) return fail(h, HDET_EINVAL, "state belongs to another configuration");
  if (in->t < 0 || in->t > h->cfg.total_steps || in->k < 0) return fail(h, HDET_EINVAL, "state counters out of range");
  for (int j = 0; j < h->n_channels; ++j) {
    uint64_t seen = 0;
    for (int r = 0; r < in->n_replicas; ++r) {
      const int32_t v = in->perm[j][r];
      if (v < 0 || v >= in->n_replicas || (seen >> v) & 1u) return fail(h, HDET_EINVAL, "perm is not a permutation");
      seen |= 1ull << v;
    }
  }
  hdet_ctrl c;
  fill_ctrl_initial(h, &c);
  c.k = in->k;
  c.controller_active = in->controller_active != 0;
  c.nonfinite = in->nonfinite;
  memcpy(c.base, in->base, sizeof(c.base));
  memcpy(c.vel, in->vel, sizeof(c.vel));
  memcpy(c.delta, in->delta, sizeof(c.delta));
  memcpy(c.w, in->w, sizeof(c.w));
  memcpy(c.l_acc, in->l_acc, sizeof(c.l_acc));
  memcpy(c.l_last, in->l_last, sizeof(c.l_last));
  memcpy(c.l_step, in->l_step, sizeof(c.l_step));
  memcpy(c.lr_used, in->lr, sizeof(c.lr_used));
  memcpy(c.perm, in->perm, sizeof(c.perm));
  int rc = upload_ctrl(h, c);
  if (rc != HDET_OK) return rc;
  h->t = in->t;
  h->last_autolr_t = (in->autolr_done && in->t % h->cfg.sync_interval == 0) ? in->t : 0;
  h->converged_at_t = -1;
  return write_shadow(h);
}

int hdet_set_launch_shape(hdet_handle* h, int32_t variant, int32_t blocks) {
  if (!h) return fail(nullptr, HDET_EINVAL, "handle is NULL");
  if (variant < 0 || variant > 7) return fail(h, HDET_EINVAL, "variant must be 0..7");
  if (blocks < 0) return fail(h, HDET_EINVAL, "negative block count");
  h->tune_variant = variant & 1;
  h->fuse_everything = (variant & 4) != 0;
  h->tune_blocks = blocks;
  if (h->tf) hdet_tf_set_fused_attention(h->tf, (variant & 2) == 0);
  return HDET_OK;
}

const char* hdet_last_error(hdet_handle* h) { return h ? h->err.c_str() : g_create_error.c_str(); }

int hdet_destroy(hdet_handle* h) {
  if (!h) return HDET_OK;
  int rc = HDET_OK;
  hipError_t e = hipStreamSynchronize(h->stream);
  if (e != hipSuccess) rc = HDET_EHIP;
  if (h->mlp) hdet_mlp_destroy(h->mlp);
  if (h->tf) hdet_tf_destroy(h->tf);
  if (h->ctrl_dev && hipFree(h->ctrl_dev) != hipSuccess) rc = HDET_EHIP;
  delete h;
  return rc;
}

}  // extern "C"

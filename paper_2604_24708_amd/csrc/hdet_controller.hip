// Auto-LR controller (Sec. 3.4, Eq. 4-9; Algorithm 1, the branch taken at sync steps) as
// one wavefront: lane r holds replica r.  What the paper does with two AllGathers of N
// scalars and host arithmetic is done here with wavefront shuffles on device-resident
// state, so a sync step needs no host round trip.
//
// All arithmetic is fp64 with sums taken in ascending replica order (each lane reads the
// operands through shuffles in that order), contraction into fused multiply-adds disabled,
// so that the result follows the written formulas operation by operation.

#include "hdet_internal.h"

#pragma clang fp contract(off)

namespace {

// Philox-4x32 with 10 rounds (Salmon et al., SC'11).
struct philox_out { uint32_t x[4]; };

__device__ philox_out philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                    uint32_t k1) {
  for (int rnd = 0; rnd < 10; ++rnd) {
    if (rnd > 0) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n1 = (uint32_t)p1;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    const uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
  }
  philox_out o = {{c0, c1, c2, c3}};
  return o;
}

constexpr uint32_t kPermStream = 0x48444554u;   // "HDET"

// Fresh permutation of Eq. 9 for draw number k (the controller update, or the sync step when
// permutations are redrawn at every sync step) and channel j: Fisher-Yates from the
// top index down on the identity, each draw uniform on [0, i] by rejection from successive
// 32-bit words of philox(counter = (block, k, j, kPermStream), key = seed).
__device__ void draw_permutation(int32_t* pi, int n, uint32_t k, uint32_t j, uint32_t seed_lo,
                                 uint32_t seed_hi) {
  for (int i = 0; i < n; ++i) pi[i] = i;
  uint32_t block = 0;
  int have = 0;
  philox_out words = {{0, 0, 0, 0}};
  for (int i = n - 1; i > 0; --i) {
    const uint32_t bound = (uint32_t)i + 1u;
    const uint64_t limit = 0x100000000ull - (0x100000000ull % bound);
    uint32_t x;
    do {
      if (have == 0) {
        words = philox4x32_10(block++, k, j, kPermStream, seed_lo, seed_hi);
        have = 4;
      }
      x = words.x[4 - have];
      --have;
    } while ((uint64_t)x >= limit);
    const int t = (int)(x % bound);
    const int32_t tmp = pi[i]; pi[i] = pi[t]; pi[t] = tmp;
  }
}

// sum over lanes 0..n-1 in ascending order; every lane gets the result
__device__ __forceinline__ double ordered_sum(double x, int n) {
  double s = 0.0;
  for (int r = 0; r < n; ++r) s += __shfl(x, r);
  return s;
}

__global__ __launch_bounds__(64) void hdet_controller_kernel(const hdet_controller_args a) {
  __shared__ int32_t s_perm[HDET_MAX_CH][HDET_MAX_REPLICAS];
  hdet_ctrl* c = a.ctrl;
  const int lane = threadIdx.x;
  const int n = a.n_replicas;
  const bool mine = lane < n;

  // L_r: mean loss of the interval; the accumulator restarts at every sync step
  double L = 0.0;
  if (mine) {
    L = a.use_injected ? a.injected[lane] : c->l_acc[lane] / (double)a.sync_interval;
    c->l_last[lane] = L;
    c->l_acc[lane] = 0.0;
  }
  if (!a.run_controller) {
    // Fig. 1's reading: a fresh assignment before every cycle, also while the base still follows
    // the one-cycle schedule
    if (a.reshuffle) {
      if (lane < a.n_channels) draw_permutation(s_perm[lane], n, a.sync_index, (uint32_t)lane, a.seed_lo, a.seed_hi);
      __syncthreads();
      if (mine)
        for (int j = 0; j < a.n_channels; ++j) c->perm[j][lane] = s_perm[j][lane];
    }
    return;
  }

  const bool bad = mine && !isfinite(L);
  if (__ballot(bad) != 0ull) {               // no ranking signal: leave the state untouched
    if (lane == 0) c->nonfinite += 1;
    return;
  }

  const bool was_active = c->controller_active != 0;
  const long long k_new = c->k + 1;

  // Eq. 4: s_r = (Lbar - L_r) / sigma, w = softmax(s)
  const double lbar = ordered_sum(L, n) / (double)n;
  const double s = mine ? (lbar - L) / a.sigma : 0.0;
  double smax = __shfl(s, 0);
  for (int r = 1; r < n; ++r) { const double o = __shfl(s, r); smax = o > smax ? o : smax; }
  const double e = mine ? exp(s - smax) : 0.0;
  const double z = ordered_sum(e, n);
  const double w = e / z;
  const double inv_n = 1.0 / (double)n;

  for (int j = 0; j < a.n_channels; ++j) {
    // at hand-over the base is the mean of the rates in effect: the schedule value
    const double b = (j < a.n_lr && !was_active) ? a.eta_sched : c->base[j];
    const double h = mine ? b * c->rho[j][c->perm[j][lane]] : 0.0;
    // Eq. 5-6: Delta = sum_r w_r h_r - (1/N) sum_r h_r = sum_r (w_r - 1/N) h_r
    const double d = ordered_sum(mine ? (w - inv_n) * h : 0.0, n);
    // Eq. 7 (gamma of Eq. 8 for the learning rates only)
    const double gamma = j < a.n_lr ? a.gamma : 0.0;
    const double nv = a.beta * c->vel[j] + (1.0 - a.beta) * d;
    double nb = b * (1.0 - gamma) + nv * a.lambda[j];
    nb = nb < a.lo[j] ? a.lo[j] : nb;
    nb = nb > a.hi[j] ? a.hi[j] : nb;
    __syncthreads();                          // every lane has read vel/base of channel j
    if (lane == 0) { c->vel[j] = nv; c->delta[j] = d; c->base[j] = nb; }
  }
  if (mine) c->w[lane] = w;

  // Eq. 9: one independent permutation per channel
  if (lane < a.n_channels)
    draw_permutation(s_perm[lane], n, a.reshuffle ? a.sync_index : (uint32_t)k_new, (uint32_t)lane, a.seed_lo, a.seed_hi);
  __syncthreads();
  if (mine)
    for (int j = 0; j < a.n_channels; ++j) c->perm[j][lane] = s_perm[j][lane];
  if (lane == 0) { c->k = k_new; c->controller_active = 1; }
}

}  // namespace

hipError_t hdet_launch_controller(const hdet_controller_args& a, hipStream_t stream) {
  hipLaunchKernelGGL(hdet_controller_kernel, dim3(1), dim3(64), 0, stream, a);
  return hipGetLastError();
}

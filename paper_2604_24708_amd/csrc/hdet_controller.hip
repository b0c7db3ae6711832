// Auto-LR controller (Sec. 3.4, Eq. 4-9; Algorithm 1, the branch taken at sync steps) as
// one wavefront: lane r holds replica r.  What the paper does with two AllGathers of N
// scalars and host arithmetic is done here with wavefront shuffles on device-resident
// state, so a sync step needs no host round trip.
//
// All arithmetic is fp64 with sums taken in ascending replica order (each lane reads the
// operands through shuffles in that order), contraction into fused multiply-adds disabled,
// so that the result follows the written formulas operation by operation.

#include "hdet_elem.h"        // Philox-4x32-10, the one device copy
#include "hdet_internal.h"

#pragma clang fp contract(off)

namespace {

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
  hdet_philox4 words = {{0, 0, 0, 0}};
  for (int i = n - 1; i > 0; --i) {
    const uint32_t bound = (uint32_t)i + 1u;
    const uint64_t limit = 0x100000000ull - (0x100000000ull % bound);
    uint32_t x;
    do {
      if (have == 0) {
        words = hdet_philox4x32_10(block++, k, j, kPermStream, seed_lo, seed_hi);
        have = 4;
      }
      x = words.x[4 - have];
      --have;
    } while ((uint64_t)x >= limit);
    const int t = (int)(x % bound);
    const int32_t tmp = pi[i]; pi[i] = pi[t]; pi[t] = tmp;
  }
}

// exp(x) for the softmax of Eq. 4 (x <= 0 there), specified operation by operation so that every
// implementation in IEEE double arithmetic without fused multiply-adds returns the same bits as this
// one, whatever its math library does:
//   x < -708             -> 0                                   (below 2^-1021: treated as no weight)
//   k = rint(x * log2 e),  r = (x - k * LN2_HI) - k * LN2_LO    (LN2_HI has 32 significant bits: k * LN2_HI is exact)
//   p = sum_{i <= 13} r^i / i!  by Horner's rule from i = 13 down, each coefficient the rounded quotient 1 / i!
//   result = p * 2^k                                             (exact scaling, k >= -1021)
// |r| <= 0.347, so the series is cut below 2^-57 and the result is within two units in the last place of exp(x).
__device__ double exp_spec(double x) {
  if (!(x >= -708.0)) return 0.0;
  const double k = __builtin_rint(x * 1.4426950408889634);
  const double r = (x - k * 6.93147180369123816490e-01) - k * 1.90821492927058770002e-10;
  const double c[14] = {1.0, 1.0, 1.0 / 2.0, 1.0 / 6.0, 1.0 / 24.0, 1.0 / 120.0, 1.0 / 720.0, 1.0 / 5040.0, 1.0 / 40320.0,
                        1.0 / 362880.0, 1.0 / 3628800.0, 1.0 / 39916800.0, 1.0 / 479001600.0, 1.0 / 6227020800.0};
  double p = c[13];
#pragma unroll
  for (int i = 12; i >= 0; --i) p = p * r + c[i];
  return p * __builtin_ldexp(1.0, (int)k);
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
  const double e = mine ? exp_spec(s - smax) : 0.0;
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

// Replica-batched bf16 GEMM on the gfx950 matrix cores, fast path: operand tiles go from
// global memory straight into LDS (buffer_load ... lds), several K steps ahead, and never pass
// through registers.  Same contract as the register-staged kernel in hdet_gemm_bf16.hip
// ("Forward + backward" of Algorithm 1 in mixed precision, N independent weight sets):
//
//   C(m,n) = sum_k A(m,k) * B(k,n)          A, B bfloat16; fp32 accumulation; C fp32 or bfloat16
//
// with the three operand orders of a Linear layer (forward NT, dgrad NN, wgrad TN).  The host
// routes a product here when every 8-element chunk of A and B is 16-byte aligned and either whole
// or absent and C can be written 4 columns at a time; everything else takes the other kernel.
//
// Design
//  * Block tile TM x TN, WGM x WGN wavefronts, each owning (TM/WGM) x (TN/WGN) as 32x32 blocks of
//    v_mfma_f32_32x32x16_bf16.  K step TK = 32 or 64, NST LDS stages of one K step each.
//  * LDS-direct loads: one instruction moves 64 lanes x 16 bytes into 1 KiB of consecutive LDS.
//    Which global chunk a lane fetches is chosen so that the tile lands already swizzled:
//      - operand contiguous along k: tile [row][TK], the 16-byte chunks of a row XOR-permuted by
//        a function of the row, so that the 128-bit fragment reads hit disjoint banks;
//      - operand contiguous along the output axis: tile [k][ROWS], chunks XOR-permuted by
//        4 (k mod 4), so that the four k-rows a 16-lane group of the transposing LDS read
//        (ds_read_b64_tr_b16) touches fall on disjoint banks.  No padding anywhere.
//    The loads go through a buffer descriptor whose extent is the operand of this batch item:
//    chunks outside it (ragged m, n, k edges) are given an out-of-range offset and arrive as
//    zeros, so the loop has no edge cases.
//  * Pipeline: the stage NST K steps ahead is requested as soon as its buffer is free.  One
//    barrier per K step, placed before the last MFMA sub-step: by then every wavefront has read
//    the whole current stage into registers, so the stage is refilled at once, and the next
//    stage has landed (s_waitcnt vmcnt leaves the younger stages in flight).  Fragments are
//    double-buffered in registers across sub-steps, LDS reads and load issue are dealt out
//    between the MFMAs, and the order is pinned with sched_barrier.
//  * Epilogue through LDS: accumulators (lane = column, 4 consecutive rows) are transposed via a
//    per-wavefront staging strip so that every global store writes whole rows, 4 columns per
//    lane; bias / ReLU / ReLU-gate / bf16 rounding (hardware round-to-nearest-even) fused.
//  * Launch order is remapped so that each XCD (own L2) works on a contiguous range of tiles, walked in groups
//    of tile rows so that concurrent blocks share operand tiles of both kinds.

#include "hdet_internal.h"
#include "hdet_elem.h"
#include "hdet_update_math.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f16v __attribute__((ext_vector_type(16)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef short s4 __attribute__((ext_vector_type(4)));
typedef short s8 __attribute__((ext_vector_type(8)));
typedef int i4 __attribute__((ext_vector_type(4)));
typedef unsigned short us4 __attribute__((ext_vector_type(4)));

#pragma clang diagnostic ignored "-Winline-asm"

// 64 lanes x 16 bytes from the buffer `rsrc` at byte offsets `voff` (out of range: zeros) to the
// LDS bytes [lds_addr, lds_addr + 1024), lane l at lds_addr + 16 l.  Completion is counted by
// vmcnt.  Written as inline assembly so that the only waits on these loads are the explicit
// ones below (the compiler would otherwise drain all of them before any LDS read).
__device__ __forceinline__ void lds_load16(i4 rsrc, uint32_t lds_addr, uint32_t voff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" ::"s"(lds_addr), "v"(voff), "s"(rsrc)
               : "memory", "m0");
}
// raw buffer descriptor: base, stride 0, extent in bytes, 32-bit untyped data
__device__ __forceinline__ i4 make_rsrc(const void* p, uint32_t bytes) {
  const uint64_t a = (uint64_t)p;
  const i4 r = {(int)(uint32_t)a, (int)(uint32_t)(a >> 32), (int)bytes, 0x00020000};
  return r;
}
__device__ __forceinline__ uint32_t lds_addr_of(const uint16_t* p) {
  return (uint32_t)(size_t)((__attribute__((address_space(3))) const uint16_t*)p);
}
// own LDS-direct loads older than the newest N have landed and own LDS reads are complete; then
// the block meets
template <int N> __device__ __forceinline__ void wait_and_barrier() {
  asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

constexpr uint32_t kAbsent = 0x80000000u;   // offset beyond every extent the host lets through

__device__ __forceinline__ unsigned short f2bf(float x) {      // round to nearest even
  return __builtin_bit_cast(unsigned short, (__bf16)x);
}
__device__ __forceinline__ float bf2f(unsigned short h) { return __uint_as_float((unsigned)h << 16); }

// One operand tile: ROWS rows of the output dimension x TK of the contraction.
// KMAJOR: element (row, k) at src[row * ld + k], LDS tile [row][TK];
// otherwise at src[k * ld + row], LDS tile [k][ROWS].
template <bool KMAJOR, int ROWS, int THREADS, int TK>
struct lds_tile {
  static constexpr int NI = ROWS * TK * 2 / (THREADS * 16);   // load instructions per thread and stage
  static constexpr int RCH = ROWS / 8;                        // chunks per k-row of a [k][ROWS] tile
  static constexpr int CPR = TK / 8;                          // chunks per row of a [row][TK] tile
  static_assert(KMAJOR || ROWS >= 128, "the chunk permutation of a [k][ROWS] tile needs at least 16 chunks per k-row");
  static_assert(TK == 32 || TK == 64, "K step");
  // chunk permutation inside a [row][TK] row: 64-byte rows by row / 4, 128-byte rows by row / 2
  static __device__ __forceinline__ int swz(int r) { return TK == 32 ? (r >> 2) & 3 : (r >> 1) & 7; }
  uint32_t off[NI];     // byte offset of this lane's chunk at K step 0, or kAbsent
  int kofs[NI];         // k index of the chunk inside a K step
  uint32_t kstep;       // bytes per K step
  __device__ __forceinline__ void init(int row0, int rows, int64_t ld, int tid) {
    kstep = KMAJOR ? TK * 2 : (uint32_t)(ld * TK * 2);
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int c = tid + i * THREADS;          // chunk slot in LDS order: LDS byte 16 c
      if (KMAJOR) {
        const int r = c / CPR, cg = (c % CPR) ^ swz(r);
        const int row = row0 + r;
        kofs[i] = cg * 8;
        off[i] = row < rows ? (uint32_t)((row * ld + cg * 8) * 2) : kAbsent;
      } else {
        const int kk = c / RCH, cg = (c % RCH) ^ ((kk & 3) << 2);
        const int row = row0 + cg * 8;
        kofs[i] = kk;
        off[i] = row < rows ? (uint32_t)((kk * ld + row) * 2) : kAbsent;
      }
    }
  }
  __device__ __forceinline__ void issue_one(int i, i4 rsrc, uint32_t tile_addr, int kt, int kdim, int wave) const {
    const uint32_t v = (kt * TK + kofs[i] < kdim) ? off[i] + (uint32_t)kt * kstep : kAbsent;
    lds_load16(rsrc, tile_addr + (i * THREADS + wave * 64) * 16, v);
  }
  // MFMA 32x32x16 operand fragment: lane l gets (row = r0 + l % 32, k = ks + 8 * (l / 32) + 0..7).
  static __device__ __forceinline__ bf16x8 fragment(const uint16_t* tile, int r0, int ks, int lane) {
    if (KMAJOR) {
      const int row = r0 + (lane & 31);
      const int chunk = ((ks >> 3) + (lane >> 5)) ^ swz(row);
      return *reinterpret_cast<const bf16x8*>(tile + row * TK + (chunk << 3));
    }
    // Transposing read: within a 16-lane group, lane p points at the 4 elements
    // (k = kb + p / 4, rows rb + 4 * (p % 4) .. + 3) and lane i receives (k = kb .. kb + 3, row rb + i).
    const int p = lane & 15;
    const int row = r0 + (((lane >> 4) & 1) << 4) + ((p & 3) << 2);
    const int k = ks + ((lane >> 5) << 3) + (p >> 2);
    const uint16_t* q = tile + k * ROWS + (((row >> 3) ^ ((k & 3) << 2)) << 3) + (row & 7);
    const s4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s4 __attribute__((address_space(3)))*)(q));
    const s4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s4 __attribute__((address_space(3)))*)(q + 4 * ROWS));
    const s8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, both);
  }
};

}  // namespace

// Two blocks share a CU when their stages fit twice into the 160 KiB of LDS; the register budget
// follows (second launch-bound argument: wavefronts per SIMD).
template <bool A_KMAJOR, bool B_KMAJOR, int EPI, int TM, int TN, int WGM, int WGN, int NST, int TK>
__global__ __launch_bounds__(64 * WGM * WGN, (NST * (TM + TN) * TK * 2 <= 80 * 1024 ? 2 : 1) * (WGM * WGN / 4))
void hdet_bgemm_dma_kernel(const hdet_bgemm_args g) {
  constexpr int THREADS = 64 * WGM * WGN;
  constexpr int WMT = TM / WGM / 32, WNT = TN / WGN / 32;
  constexpr int STAGE = (TM + TN) * TK;           // elements per stage: A tile then B tile
  __shared__ __attribute__((aligned(1024))) uint16_t S[NST * STAGE];
  typedef lds_tile<A_KMAJOR, TM, THREADS, TK> ta;
  typedef lds_tile<B_KMAJOR, TN, THREADS, TK> tb;
  constexpr int LPT = ta::NI + tb::NI;            // load instructions per thread and stage

  int bx, by, bz;
  {
    // Launch order -> tile: each XCD (own L2; blocks are dealt to the XCDs round-robin) works through a contiguous
    // range of tiles, and inside a batch item consecutive tiles walk groups of tile_group tile rows column by column,
    // so that the blocks an XCD runs at one time share operand tiles of both kinds in its L2.
    const unsigned total = gridDim.x * gridDim.y * gridDim.z;
    unsigned t = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
    {   // XCD x = launch index mod 8 takes the x-th of eight contiguous ranges (the first total mod 8 ranges one tile longer)
      const unsigned x = t & 7u, rem = total & 7u;
      t = x * (total >> 3) + (x < rem ? x : rem) + (t >> 3);
    }
    const unsigned per = gridDim.x * gridDim.y;
    bz = t / per;
    const unsigned r = t - bz * per;
    const unsigned gm = g.tile_group > 1 ? (unsigned)g.tile_group : 1u;
    const unsigned gsz = gm * gridDim.x;
    const unsigned grp = r / gsz, first = grp * gm;
    const unsigned rows = gridDim.y - first < gm ? gridDim.y - first : gm;
    const unsigned q = r - grp * gsz;
    by = first + q % rows;
    bx = q / rows;
  }
  const hdet_batch_index bi = hdet_split_batch(bz, g.n1, g.n2);
  const int z = bi.z0;            // replica: bias and mask are per replica
  const uint16_t* A = g.a + hdet_batch_offset(bi, g.a_s);
  const uint16_t* B = g.b + hdet_batch_offset(bi, g.b_s);
  const int64_t c_base = hdet_batch_offset(bi, g.c_s);
  const int m0 = by * TM, n0 = bx * TN;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = (wave / WGN) * (32 * WMT), wn = (wave % WGN) * (32 * WNT);

  // byte extent of each operand for this batch item: the bound that turns absent chunks into zeros
  const uint32_t a_bytes = (uint32_t)(((int64_t)((A_KMAJOR ? g.m : g.k) - 1) * g.lda + (A_KMAJOR ? g.k : g.m)) * 2);
  const uint32_t b_bytes = (uint32_t)(((int64_t)((B_KMAJOR ? g.n : g.k) - 1) * g.ldb + (B_KMAJOR ? g.k : g.n)) * 2);
  const i4 ra = make_rsrc(A, a_bytes), rb = make_rsrc(B, b_bytes);
  const uint32_t s_addr = lds_addr_of(S);

  ta la; tb lb;
  la.init(m0, g.m, g.lda, tid);
  lb.init(n0, g.n, g.ldb, tid);

  f16v acc[WMT][WNT];
#pragma unroll
  for (int i = 0; i < WMT; ++i)
#pragma unroll
    for (int j = 0; j < WNT; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int nk = (g.k + TK - 1) / TK;
#define STAGE_PTR(s) (S + (s) * STAGE)
#define STAGE_ADDR(s) (s_addr + (s) * STAGE * 2)
  // K steps 0 .. NST-1 are requested up front; steps past the end load nothing (all chunks absent)
#pragma unroll
  for (int s = 0; s < NST; ++s) {
#pragma unroll
    for (int i = 0; i < ta::NI; ++i) la.issue_one(i, ra, STAGE_ADDR(s), s, g.k, wave);
#pragma unroll
    for (int i = 0; i < tb::NI; ++i) lb.issue_one(i, rb, STAGE_ADDR(s) + TM * TK * 2, s, g.k, wave);
  }
  wait_and_barrier<(NST - 1) * LPT>();

  // Fragments are double-buffered in registers over the NSS = TK / 16 MFMA sub-steps of a K step:
  // while the MFMAs of sub-step ss run on fa/fb[ss & 1], the fragments of the next sub-step (of
  // the next stage after the last one) are read into the other set.
  constexpr int NSS = TK / 16, NM = WMT * WNT, NR = WMT + WNT;
  constexpr int IPA = (NR + NM - 1) / NM, IPB = (NR + LPT + NM - 1) / NM;
  bf16x8 fa[2][WMT], fb[2][WNT];
  auto read_frag = [&](bf16x8* a, bf16x8* b, const uint16_t* st, int ks, int idx) {
    // order: a[0], b[0..WNT-1], a[1..WMT-1] -- what the first MFMAs of the next sub-step need first
    if (idx == 0) a[0] = ta::fragment(st, wm, ks, lane);
    else if (idx <= WNT) b[idx - 1] = tb::fragment(st + TM * TK, wn + (idx - 1) * 32, ks, lane);
    else if (idx < NR) a[idx - WNT] = ta::fragment(st, wm + (idx - WNT) * 32, ks, lane);
  };
#pragma unroll
  for (int idx = 0; idx < NR; ++idx) read_frag(fa[0], fb[0], S, 0, idx);

  for (int kt0 = 0; kt0 < nk; kt0 += NST) {
#pragma unroll
    for (int s = 0; s < NST; ++s) {
      const int kt = kt0 + s;
      if (kt >= nk) break;
      const uint16_t* cur = STAGE_PTR(s);
      const uint16_t* nxt = STAGE_PTR((s + 1) % NST);
#pragma unroll
      for (int ss = 0; ss < NSS - 1; ++ss) {
#pragma unroll
        for (int q = 0; q < NM; ++q) {
          acc[q / WNT][q % WNT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ss & 1][q / WNT], fb[ss & 1][q % WNT],
                                                                          acc[q / WNT][q % WNT], 0, 0, 0);
#pragma unroll
          for (int u = 0; u < IPA; ++u) read_frag(fa[(ss + 1) & 1], fb[(ss + 1) & 1], cur, (ss + 1) * 16, q * IPA + u);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      // every wavefront has read all of stage `cur`; stage `nxt` (K step kt + 1) has landed
      wait_and_barrier<(NST - 2) * LPT>();
#pragma unroll
      for (int q = 0; q < NM; ++q) {
        acc[q / WNT][q % WNT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[(NSS - 1) & 1][q / WNT], fb[(NSS - 1) & 1][q % WNT],
                                                                        acc[q / WNT][q % WNT], 0, 0, 0);
#pragma unroll
        for (int u = 0; u < IPB; ++u) {
          const int it = q * IPB + u;
          if (it < ta::NI) la.issue_one(it, ra, STAGE_ADDR(s), kt + NST, g.k, wave);
          else if (it < LPT) lb.issue_one(it - ta::NI, rb, STAGE_ADDR(s) + TM * TK * 2, kt + NST, g.k, wave);
          else read_frag(fa[0], fb[0], nxt, 0, it - LPT);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
#undef STAGE_PTR
#undef STAGE_ADDR
  // every wavefront is done with the stage buffers (and the loads past the end have drained):
  // they become the staging area of the epilogue
  wait_and_barrier<0>();

  // Epilogue through LDS, one 32-row strip of at most 64 columns at a time: the accumulators
  // (lane = column, 4 consecutive rows per 4 elements) are written as fp32 [32][CW] with a pitch
  // that keeps the two half-wavefronts on disjoint banks, and read back with 4 consecutive
  // columns per lane, so that every global store instruction writes whole rows of the strip.
  // The strip is private to the wavefront and LDS serves one wavefront's accesses in order.
  constexpr int JG = WNT < 2 ? WNT : 2;       // 32-column blocks per strip
  constexpr int CW = JG * 32, EP = CW + 8, LPR = CW / 4, RPI = 64 / LPR;
  static_assert(WGM * WGN * 32 * EP * 4 <= NST * STAGE * 2, "staging area exceeds the stage buffers");
  float* stg = reinterpret_cast<float*>(S) + wave * (32 * EP);
  const int lr = lane / LPR, lc = (lane % LPR) * 4;
  constexpr bool kBias = EPI == HDET_EPI_BIAS_RELU_BF16 || EPI == HDET_EPI_BIAS_F32 || EPI == HDET_EPI_BIAS_BF16 ||
                         EPI == HDET_EPI_BIAS_GELU_BF16 || EPI == HDET_EPI_BIAS_RESID_BF16 || EPI == HDET_EPI_BIAS_DROP_RESID_BF16;
  // the second operand of the gating epilogues (the activations a ReLU or GELU gradient looks at) is
  // fetched one strip ahead, so that its latency hides behind the previous strip's pass through LDS
  constexpr bool kGate = EPI == HDET_EPI_MASK_BF16 || EPI == HDET_EPI_GELUGRAD_BF16 || EPI == HDET_EPI_BIAS_RESID_BF16 ||
                         EPI == HDET_EPI_BIAS_DROP_RESID_BF16;
  constexpr int NIT = 32 / RPI, NSTRIP = (WNT / JG) * WMT;
  us4 gate[2][NIT];
  auto fetch_gate = [&](int strip, us4 (&dst)[NIT]) {
    const int col = n0 + wn + (strip / WMT) * CW + lc;
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int row = m0 + wm + (strip % WMT) * 32 + it * RPI + lr;
      dst[it] = us4{0, 0, 0, 0};
      if (row < g.m && col < g.n)
        dst[it] = *reinterpret_cast<const us4*>(g.mask + (int64_t)z * g.mask_bs + (int64_t)row * g.mask_ld + col);
    }
  };
  uint32_t drop_thresh = 0u;
  float drop_scale = 1.f;
  if (EPI == HDET_EPI_BIAS_DROP_RESID_BF16) {
    const float p = (float)hdet_channel_value(g.drop_ctrl, g.drop_channel, z, 0.0);
    drop_thresh = (uint32_t)floor((double)p * 4294967296.0);
    drop_scale = 1.f / (1.f - p);
  }
  // HDET_EPI_ADAMW: the tile is the replica's gradient of a weight matrix and is applied at once (Eq. 2 with the
  // replica's rate); the matrix's parameters and moments of a strip are requested before the strip goes through LDS
  constexpr bool kUpd = EPI == HDET_EPI_ADAMW;
  hdet_um::rep_scalars us = {0.f, 0.f, 0.f, 0.f};
  if (kUpd) {
    us = hdet_um::replica_scalars(g.upd, z);
    if (bx == 0 && by == 0 && tid == 0 && g.upd.lr_channel == 0) g.upd.ctrl_out->lr_used[z] = us.lr;
  }
  f4 uth[kUpd ? NIT : 1], um[kUpd ? NIT : 1], uv[kUpd ? NIT : 1];
  // column sums of the stored result over the wavefront's rows, for the columns this lane stores (per strip column group)
  constexpr bool kColsum = EPI == HDET_EPI_GELUGRAD_BF16 || EPI == HDET_EPI_MASK_BF16;
  f4 csum[WNT / JG];
#pragma unroll
  for (int jg = 0; jg < WNT / JG; ++jg) csum[jg] = f4{0.f, 0.f, 0.f, 0.f};
  if (kGate) fetch_gate(0, gate[0]);
#pragma unroll
  for (int jg = 0; jg < WNT / JG; ++jg) {
    const int col = n0 + wn + jg * CW + lc;
    const bool col_ok = col < g.n;             // n is a multiple of 4: the 4 columns exist together
    f4 bias = {0.f, 0.f, 0.f, 0.f};
    if (kBias && col_ok) bias = *reinterpret_cast<const f4*>(g.bias + (int64_t)z * g.bias_bs + col);
#pragma unroll
    for (int i = 0; i < WMT; ++i) {
      const int strip = jg * WMT + i;
      if (kGate && strip + 1 < NSTRIP) fetch_gate(strip + 1, gate[(strip + 1) & 1]);
      if (kUpd) {
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
          const int row = m0 + wm + i * 32 + it * RPI + lr;
          if (row < g.m && col_ok) {
            const int64_t off = c_base + (int64_t)row * g.ldc + col;
            uth[it] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(g.upd.theta + off));
            um[it] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(g.upd.m + off));
            uv[it] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(g.upd.v + off));
          }
        }
      }
      // accumulator element e of lane l is C(row, col) with row = (e / 4) * 8 + (l / 32) * 4 + e % 4,
      // col = l % 32 inside its 32x32 block
#pragma unroll
      for (int j = 0; j < JG; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e)
          stg[((e >> 2) * 8 + (lane >> 5) * 4 + (e & 3)) * EP + j * 32 + (lane & 31)] = acc[i][jg * JG + j][e];
#pragma unroll
      for (int it = 0; it < 32 / RPI; ++it) {
        const int rl = it * RPI + lr;
        f4 v = *reinterpret_cast<const f4*>(stg + rl * EP + lc);
        const int row = m0 + wm + i * 32 + rl;
        if (row < g.m && col_ok) {
          const int64_t off = c_base + (int64_t)row * g.ldc + col;
          if (kBias) v += bias;
          if (EPI == HDET_EPI_BIAS_RELU_BF16) {
#pragma unroll
            for (int q = 0; q < 4; ++q) v[q] = v[q] > 0.f ? v[q] : 0.f;
          }
          if (EPI == HDET_EPI_MASK_BF16) {    // gradient through the ReLU of the layer below
            const us4 a = gate[strip & 1][it];
#pragma unroll
            for (int q = 0; q < 4; ++q) v[q] = bf2f(a[q]) > 0.f ? v[q] : 0.f;
          }
          if (EPI == HDET_EPI_BIAS_RESID_BF16) {  // the layer's output is rounded as the unfused path stores it, then added
            const us4 a = gate[strip & 1][it];
#pragma unroll
            for (int q = 0; q < 4; ++q) v[q] = bf2f(a[q]) + bf2f(f2bf(v[q]));
          }
          if (EPI == HDET_EPI_BIAS_DROP_RESID_BF16) {   // ... dropped out (one Philox block per 4 elements), then added
            const us4 a = gate[strip & 1][it];
            hdet_philox4 w = {{0xffffffffu, 0xffffffffu, 0xffffffffu, 0xffffffffu}};
            if (drop_thresh != 0u)
              w = hdet_philox4x32_10((uint32_t)(((int64_t)row * g.ldc + col) >> 2), g.drop_step, (uint32_t)z * 65536u + g.drop_site,
                                     g.drop_stream, g.drop_seed_lo, g.drop_seed_hi);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              float y = bf2f(f2bf(v[q]));
              if (drop_thresh != 0u) y = w.x[q] >= drop_thresh ? y * drop_scale : 0.f;
              v[q] = bf2f(a[q]) + y;
            }
          }
          if (EPI == HDET_EPI_GELUGRAD_BF16) {  // the incoming gradient is rounded as the unfused path stores it
            const us4 a = gate[strip & 1][it];
#pragma unroll
            for (int q = 0; q < 4; ++q) v[q] = bf2f(f2bf(v[q])) * hdet_gelu_tanh_grad_fast(bf2f(a[q]));
          }
          if (EPI == HDET_EPI_ADAMW) {
            f4 th = uth[it], mm = um[it], vv = uv[it];
            hdet_um::update_one<HDET_ADAMW, f4>(th, v, mm, vv, g.upd, us);
            __builtin_nontemporal_store(mm, reinterpret_cast<f4*>(g.upd.m + off));
            __builtin_nontemporal_store(vv, reinterpret_cast<f4*>(g.upd.v + off));
            __builtin_nontemporal_store(th, reinterpret_cast<f4*>(g.upd.theta + off));
            if (g.upd.shadow) {
              const us4 o = {hdet_um::to_bf16(th[0]), hdet_um::to_bf16(th[1]), hdet_um::to_bf16(th[2]), hdet_um::to_bf16(th[3])};
              __builtin_nontemporal_store(o, reinterpret_cast<us4*>(g.upd.shadow + off));
            }
          } else if (EPI == HDET_EPI_F32 || EPI == HDET_EPI_BIAS_F32) {
            *reinterpret_cast<f4*>(reinterpret_cast<float*>(g.c) + off) = v;
          } else if (EPI == HDET_EPI_BIAS_GELU_BF16) {
            const us4 pre = {f2bf(v[0]), f2bf(v[1]), f2bf(v[2]), f2bf(v[3])};
            *reinterpret_cast<us4*>(reinterpret_cast<uint16_t*>(g.c) + off) = pre;
            const us4 o = {f2bf(hdet_gelu_tanh_fast(bf2f(pre[0]))), f2bf(hdet_gelu_tanh_fast(bf2f(pre[1]))),
                           f2bf(hdet_gelu_tanh_fast(bf2f(pre[2]))), f2bf(hdet_gelu_tanh_fast(bf2f(pre[3])))};
            *reinterpret_cast<us4*>(reinterpret_cast<uint16_t*>(g.c2) + off) = o;
          } else {
            const us4 o = {f2bf(v[0]), f2bf(v[1]), f2bf(v[2]), f2bf(v[3])};
            *reinterpret_cast<us4*>(reinterpret_cast<uint16_t*>(g.c) + off) = o;
            if (kColsum) {
#pragma unroll
              for (int q = 0; q < 4; ++q) csum[jg][q] += bf2f(o[q]);
            }
          }
        }
      }
    }
  }
  // Stage 1 of the column sums: a lane has added its rows in ascending order; the RPI lanes that hold the same
  // columns are added by exchanges (a fixed tree), then the wavefronts that share a 128-row block in the order of
  // their rows.  Every (128-row block, column) of C is written by exactly one block of the grid.
  if (kColsum && g.colsum) {
    constexpr int RW = TM / WGM;                      // rows per wavefront
    static_assert(TM % 128 == 0 && RW <= 128 && 128 % RW == 0, "wavefronts must tile 128-row blocks");
    float* cbuf = reinterpret_cast<float*>(S);        // [WGM * WGN wavefronts][TN / WGN columns]
#pragma unroll
    for (int jg = 0; jg < WNT / JG; ++jg)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float x = csum[jg][q];
#pragma unroll
        for (int o = LPR; o < 64; o <<= 1) x += __shfl_xor(x, o);
        csum[jg][q] = x;
      }
    __syncthreads();                                   // the strips are no longer in use
    if (lane < LPR) {
#pragma unroll
      for (int jg = 0; jg < WNT / JG; ++jg)
#pragma unroll
        for (int q = 0; q < 4; ++q) cbuf[wave * (TN / WGN) + jg * CW + lc + q] = csum[jg][q];
    }
    __syncthreads();
    constexpr int WPC = RW >= 128 ? 1 : 128 / RW;      // wavefronts (along m) per 128-row block
    constexpr int CHUNKS = TM >= 128 ? TM / 128 : 1;
    const int nchunks = (g.m + 127) / 128;
    for (int t = tid; t < CHUNKS * TN; t += THREADS) {
      const int ch = t / TN, cn = t % TN;              // chunk of the tile, column of the tile
      const int wcol = cn / (TN / WGN), ccol = cn % (TN / WGN);
      float a = 0.f;
#pragma unroll
      for (int u = 0; u < WPC; ++u) a += cbuf[((ch * WPC + u) * WGN + wcol) * (TN / WGN) + ccol];
      const int chunk = m0 / 128 + ch, col = n0 + cn;
      if (chunk < nchunks && col < g.n) g.colsum[((int64_t)z * nchunks + chunk) * g.n + col] = a;
    }
  }
}

namespace {

bool chunk_regular(const void* base, int64_t ld, const int64_t* bs, int chunk_extent) {
  return (ld & 7) == 0 && ((bs[0] | bs[1] | bs[2]) & 7) == 0 && (chunk_extent & 7) == 0 &&
         (reinterpret_cast<uintptr_t>(base) & 15) == 0;
}

// compute units of the current device (queried once per device; 256 on MI355X)
int compute_units() { return hdet_compute_units(); }

}  // namespace

int hdet_compute_units() {
  static int cached[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  if (cached[dev] == 0) {
    int n = 0;
    cached[dev] = (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0) ? n : 256;
  }
  return cached[dev];
}

namespace {

template <bool AK, bool BK, int EPI>
hipError_t launch_shape(const hdet_bgemm_args& g, int batch, hipStream_t s) {
  auto blocks = [&](int tm, int tn) { return (int64_t)((g.m + tm - 1) / tm) * ((g.n + tn - 1) / tn) * batch; };
  const int kCus = compute_units();
  // a gating epilogue is long enough to want a second block on the CU up to K = 1024
  constexpr bool gating = EPI == HDET_EPI_MASK_BF16 || EPI == HDET_EPI_GELUGRAD_BF16;
  const bool long_k = g.k >= (gating ? 2048 : 1024);
  // Tile order inside a batch item: with many tile columns, the 32 blocks an XCD runs at a time would share one
  // operand tile of A and none of B; walking groups of 4 (2) tile rows column by column cuts the operand bytes its L2
  // has to fetch by up to two thirds (head product of the transformer, 125 tile columns: 9-11 % faster).
#define HDET_DMA_LAUNCH(TM, TN, WGM, WGN, NST, TK)                                                            \
  do {                                                                                                        \
    const dim3 grid((g.n + TN - 1) / TN, (g.m + TM - 1) / TM, batch);                                          \
    hdet_bgemm_args ga = g;                                                                                   \
    ga.tile_group = grid.x >= 64 ? 4 : grid.x >= 12 ? 2 : 1;                                                  \
    hipLaunchKernelGGL((hdet_bgemm_dma_kernel<AK, BK, EPI, TM, TN, WGM, WGN, NST, TK>), grid, dim3(64 * WGM * WGN), 0, s, ga); \
  } while (0)
  // short-K products with plenty of tiles also take the largest tile, unless the epilogue reads a second
  // operand: those do better with two blocks per CU, whose epilogues and main loops overlap
  // (a single round of the largest tile on nine tenths of the chip beats two rounds of the next one; but when the
  // largest tiles make between one and two rounds and leave the last one under 80 % full, the half-size tiles, which
  // the CUs take up two at a time and one by one, finish sooner: 3072 x 1024 x 8 replicas at K = 8192 by 5-12 %)
  const int64_t big = blocks(256, 256);
  const bool ragged_rounds = big > kCus && big < 2 * (int64_t)kCus && big * 10 < 2 * (int64_t)kCus * 8;
  if (((long_k && big * 10 >= (int64_t)kCus * 9) || (!gating && big >= 3 * kCus)) && !(long_k && ragged_rounds))
  {
    // weight gradients (both operands read with the transposing LDS loads) run 2-5 % faster on three stages of
    // K = 32 than on two of 64; the forward and input-gradient products 1-6 % slower
    if constexpr (!AK && !BK) HDET_DMA_LAUNCH(256, 256, 2, 4, 3, 32);                         // one block per CU, 96 KiB of stages
    else HDET_DMA_LAUNCH(256, 256, 2, 4, 2, 64);                                    // one block per CU, 128 KiB of stages
  } else if (long_k && ragged_rounds && EPI != HDET_EPI_ADAMW) {
    if constexpr (EPI != HDET_EPI_ADAMW) HDET_DMA_LAUNCH(256, 128, 4, 2, 3, 32);    // two blocks per CU, 72 KiB each
  } else if (blocks(256, 128) >= kCus) {
    // (the update epilogue holds a strip of theta, m and v in registers: too many for two blocks per CU)
    if (long_k || EPI == HDET_EPI_ADAMW) HDET_DMA_LAUNCH(256, 128, 4, 2, 3, 64);    // one block per CU, 144 KiB
    else if constexpr (EPI != HDET_EPI_ADAMW) HDET_DMA_LAUNCH(256, 128, 4, 2, 3, 32);   // two blocks per CU, 72 KiB each
  } else HDET_DMA_LAUNCH(128, 128, 2, 2, 2, 64);                                    // two blocks per CU, 64 KiB each
#undef HDET_DMA_LAUNCH
  return hipGetLastError();
}

}  // namespace

bool hdet_bgemm_dma_eligible(const hdet_bgemm_args& g, bool a_kmajor, bool b_kmajor, int epi) {
  const bool f32_out = epi == HDET_EPI_F32 || epi == HDET_EPI_BIAS_F32;
  const bool has_bias = epi == HDET_EPI_BIAS_F32 || epi == HDET_EPI_BIAS_BF16 || epi == HDET_EPI_BIAS_RELU_BF16 ||
                        epi == HDET_EPI_BIAS_GELU_BF16 || epi == HDET_EPI_BIAS_RESID_BF16 || epi == HDET_EPI_BIAS_DROP_RESID_BF16;
  if (g.m < 1 || g.n < 1 || g.k < 1) return false;
  // a chunk is 8 elements along the operand's contiguous axis: k if k-major, else the row axis
  if (!chunk_regular(g.a, g.lda, g.a_s, a_kmajor ? g.k : g.m)) return false;
  if (!chunk_regular(g.b, g.ldb, g.b_s, b_kmajor ? g.k : g.n)) return false;
  // operand extents of one batch item as 32-bit byte offsets below the "absent" mark
  const int64_t a_bytes = ((int64_t)((a_kmajor ? g.m : g.k) - 1) * g.lda + (a_kmajor ? g.k : g.m)) * 2;
  const int64_t b_bytes = ((int64_t)((b_kmajor ? g.n : g.k) - 1) * g.ldb + (b_kmajor ? g.k : g.n)) * 2;
  // the K loop may form offsets up to one stage row past the extent before they are replaced
  const int64_t slack = 64 * 2 * (a_kmajor ? 1 : g.lda) + 64 * 2 * (b_kmajor ? 1 : g.ldb);
  if (a_bytes + slack >= (int64_t)1 << 31 || b_bytes + slack >= (int64_t)1 << 31) return false;
  // C (and bias, mask) four columns at a time
  if ((g.ldc & 3) || ((g.c_s[0] | g.c_s[1] | g.c_s[2]) & 3) || (g.n & 3)) return false;
  if (reinterpret_cast<uintptr_t>(g.c) & (f32_out ? 15 : 7)) return false;
  if (has_bias && ((g.bias_bs & 3) || (reinterpret_cast<uintptr_t>(g.bias) & 15))) return false;
  if (epi == HDET_EPI_BIAS_DROP_RESID_BF16 && (!g.drop_ctrl || g.drop_channel < 0 || g.n1 * g.n2 != 1 || g.c_s[0] >= ((int64_t)1 << 34)))
    return false;        // the replica is the batch index; the element counter has 32 bits
  if ((epi == HDET_EPI_MASK_BF16 || epi == HDET_EPI_GELUGRAD_BF16 || epi == HDET_EPI_BIAS_RESID_BF16 || epi == HDET_EPI_BIAS_DROP_RESID_BF16) &&
      (!g.mask || (g.mask_ld & 3) || (g.mask_bs & 3) || (reinterpret_cast<uintptr_t>(g.mask) & 7)))
    return false;
  if (epi == HDET_EPI_BIAS_GELU_BF16 && (!g.c2 || (reinterpret_cast<uintptr_t>(g.c2) & 7))) return false;
  if (epi == HDET_EPI_ADAMW &&
      (g.n1 * g.n2 != 1 || !g.upd.theta || !g.upd.m || !g.upd.v || !g.upd.ctrl || !g.upd.ctrl_out ||
       ((reinterpret_cast<uintptr_t>(g.upd.theta) | reinterpret_cast<uintptr_t>(g.upd.m) | reinterpret_cast<uintptr_t>(g.upd.v)) & 15) ||
       (reinterpret_cast<uintptr_t>(g.upd.shadow) & 7)))
    return false;
  // instantiated combinations: what the MLP and the transformer use
  if (a_kmajor && b_kmajor)
    return epi == HDET_EPI_BIAS_RELU_BF16 || epi == HDET_EPI_BIAS_F32 || epi == HDET_EPI_BIAS_BF16 || epi == HDET_EPI_F32 ||
           epi == HDET_EPI_BIAS_GELU_BF16 || epi == HDET_EPI_BIAS_RESID_BF16 || epi == HDET_EPI_BIAS_DROP_RESID_BF16;
  if (a_kmajor && !b_kmajor) return epi == HDET_EPI_MASK_BF16 || epi == HDET_EPI_BF16 || epi == HDET_EPI_GELUGRAD_BF16;
  if (!a_kmajor && !b_kmajor) return epi == HDET_EPI_F32 || epi == HDET_EPI_BF16 || epi == HDET_EPI_ADAMW;
  return false;
}

hipError_t hdet_launch_bgemm_dma(const hdet_bgemm_args& g_in, bool a_kmajor, bool b_kmajor, int epi, int batch,
                                 hipStream_t s) {
  hdet_bgemm_args g = g_in;
  if (g.n1 < 1) g.n1 = 1;
  if (g.n2 < 1) g.n2 = 1;
  if (!hdet_bgemm_dma_eligible(g, a_kmajor, b_kmajor, epi)) return hipErrorInvalidValue;
  if (a_kmajor && b_kmajor) {            // forward
    switch (epi) {
      case HDET_EPI_BIAS_RELU_BF16: return launch_shape<true, true, HDET_EPI_BIAS_RELU_BF16>(g, batch, s);
      case HDET_EPI_BIAS_F32: return launch_shape<true, true, HDET_EPI_BIAS_F32>(g, batch, s);
      case HDET_EPI_BIAS_BF16: return launch_shape<true, true, HDET_EPI_BIAS_BF16>(g, batch, s);
      case HDET_EPI_BIAS_GELU_BF16: return launch_shape<true, true, HDET_EPI_BIAS_GELU_BF16>(g, batch, s);
      case HDET_EPI_BIAS_RESID_BF16: return launch_shape<true, true, HDET_EPI_BIAS_RESID_BF16>(g, batch, s);
      case HDET_EPI_BIAS_DROP_RESID_BF16: return launch_shape<true, true, HDET_EPI_BIAS_DROP_RESID_BF16>(g, batch, s);
      default: return launch_shape<true, true, HDET_EPI_F32>(g, batch, s);
    }
  }
  if (a_kmajor) {                        // dgrad
    if (epi == HDET_EPI_MASK_BF16) return launch_shape<true, false, HDET_EPI_MASK_BF16>(g, batch, s);
    if (epi == HDET_EPI_GELUGRAD_BF16) return launch_shape<true, false, HDET_EPI_GELUGRAD_BF16>(g, batch, s);
    return launch_shape<true, false, HDET_EPI_BF16>(g, batch, s);
  }
  if (epi == HDET_EPI_F32) return launch_shape<false, false, HDET_EPI_F32>(g, batch, s);   // wgrad
  if (epi == HDET_EPI_ADAMW) return launch_shape<false, false, HDET_EPI_ADAMW>(g, batch, s);
  return launch_shape<false, false, HDET_EPI_BF16>(g, batch, s);
}

// bf16 MFMA GEMM for gfx950:  D[i,j] = sum_k X[i,k] * Y[j,k]  (both operands K-contiguous), fp32
// accumulation with v_mfma_f32_32x32x16_bf16.
//
// Shape of the kernel (what measurements on MI355X pushed it to):
//   * one workgroup per CU: 256 x BN output tile (BN = 192 or 128), 4 wavefronts in a 2x2 grid, each
//     wavefront owns 128 x BN/2 (accumulators in AGPRs).  The L2 delivers about 32 B/clk to a CU, so
//     a tile needs >= 64..128 flop per loaded byte; 128x128 tiles are bound by that, 256x192 is not.
//     With few rows (one to eight states) the projections only stream weights: the same kernel with
//     128- or 64-row tiles does half or a quarter of the matrix work per tile and covers more CUs; the
//     narrow split-K projections of one or two states take 32-column tiles with one wavefront along a
//     32-wide side (64 x 32: two wavefronts, 32 x 32: one), so 256 workgroups stream instead of 128;
//     the gate/up projection of up to 128 rows takes 96-column tiles (256 workgroups instead of 192):
//     a 1 x 4 wavefront grid, three wavefronts own a 32-column block each, the fourth only loads.
//   * K advances in steps of 64 so every row segment is one full 128-byte line; operands go
//     global -> LDS directly (LDS-DMA loads, no register staging), rows XOR-swizzled so the
//     16-byte fragment reads are conflict-free.
//   * separate LDS rings for the two operands: the activation operand (mostly L2 hits) gets 2 stages,
//     the weight operand (streamed from HBM) SD = 3-4 stages, 128-144 KB in all.
//   * one barrier per K-tile; the loads of later tiles and the LDS fragment reads of the next
//     16-wide K step are threaded between the MFMAs of the current step, fragments double-buffered
//     in registers, partial s_waitcnt vmcnt so younger loads stay in flight across the barrier.
//   * workgroup ids are remapped so that the workgroups sharing a weight tile sit on one XCD.
//
// Epilogues:
//   EPI_STORE    C = X W^T (+bias), W given as up to three row segments (q | k | v)
//   EPI_RESID    C = R + X W^T
//   EPI_SWIGLU   C = silu(X Wg^T) * (X Wu^T); gate and up rows are interleaved 16/16 inside every
//                32-column MFMA tile, partner values meet through one lane shuffle
//   EPI_PARTIAL  fp32 partial sums of one K slice (split-K for narrow N; reduced by a second kernel
//                in a fixed order, the slice count depends on (N, K) only)
//   EPI_LMHEAD   rows i = vocabulary entries, columns j = tokens: each lane owns token columns and
//                reduces its logits to (top, lowest index, runner-up, sum exp) in registers; logits
//                are never stored (Alg. 1 steps 1-2 fused into the GEMM)
//
// The accumulation order along K of every output element is fixed by (N, K) alone, so a row's result
// does not depend on how many other states are verified with it.
#include <type_traits>

#include "kernels.h"

namespace spiffy {

namespace {

constexpr int BM = 256, BKK = 64;

typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* glb_ptr_t;

template <int N>
__device__ __forceinline__ void wait_vmcnt() {   // vmcnt <= N; lgkmcnt / expcnt untouched
  __builtin_amdgcn_s_waitcnt((N & 0xF) | (7 << 4) | (0xF << 8) | ((N >> 4) << 14));
}
__device__ __forceinline__ void wait_lgkm0() { __builtin_amdgcn_s_waitcnt(0xC07F); }

// 64-row tiles, and 128-row tiles up to 128 columns wide, are weight-streaming shapes: both operand rings SD deep
constexpr bool uniform_rings(int epi, int bn, int bmt) { return epi != EPI_LMHEAD && (bmt <= 64 || (bmt == 128 && bn <= 128)); }
// stages of the shallow operand's ring = how many K-tiles ahead it is loaded; SA = 0 picks the default of the shape
constexpr int shallow_stages(int epi, int bn, int bmt, int sd, int sa) { return sa ? sa : (uniform_rings(epi, bn, bmt) ? sd : 2); }
// wavefronts of a workgroup: a 2 x 2 grid over the tile; a 32-row or 32-column tile has one wavefront along that side.
// A 96-column tile (three 32-column blocks: what gives 256 workgroups when 128 columns give 192) has a 1 x 4 grid whose
// first three wavefronts own one block each; the fourth only takes its share of the loads.
constexpr int waves_m(int bmt, int bn) { return bn == 96 ? 1 : (bmt >= 64 ? 2 : 1); }
constexpr int waves_n(int bn) { return bn == 96 ? 4 : (bn >= 64 ? 2 : 1); }
constexpr int wave_cols(int bn) { return bn == 96 ? 32 : bn / waves_n(bn); }

template <int EPI, int BN, int SD, int BMT = 256, int SA = 0>
__global__ __launch_bounds__(256) void gemm_bf16_mfma_kernel(GemmArgs a, int tiles_i, int tiles_j) {
  constexpr int BM = BMT;                         // rows of the output tile: 256, or 128 / 64 / 32 when there are few rows
  constexpr int WM = waves_m(BMT, BN), WN = waves_n(BN), NW = WM * WN;
  constexpr int RW = BM / WM, CW = wave_cols(BN);  // rows and columns of the tile that one wavefront owns
  constexpr int NW_MATH = WM * (BN / CW);          // wavefronts that own a part of the tile (all but one of a 96-column tile's)
  static_assert(EPI != EPI_LMHEAD || NW == 4, "the LM-head epilogue assumes the 2 x 2 wavefront grid");
  // which operand is the weight matrix (deep ring): Y for the projections, X for the LM head
  constexpr bool XDEEP = (EPI == EPI_LMHEAD);
  // The deep operand (weights) rides a ring of SD stages and is loaded SD tiles ahead; the shallow one (activations)
  // a ring of SH stages, SH tiles ahead.  The load counter retires in order, so waiting for the shallow operand of
  // the next tile also waits for every older load: across a barrier stay in flight the deep loads issued with that
  // shallow tile and the SH-2 whole groups after it (SH = 2: only the newest weight tile, whatever SD; SH = SD, the
  // weight-streaming shapes with few rows: SD-2 whole tiles).
  constexpr int SH = shallow_stages(EPI, BN, BMT, SD, SA);
  static_assert(SH >= 2 && SH <= SD, "the shallow ring is at most as deep as the deep one");
  constexpr int SX = XDEEP ? SD : SH, SY = XDEEP ? SH : SD;
  constexpr int TM = RW / 32, TN = CW / 32;
  constexpr int LX = BM / (8 * NW), LY = BN / (8 * NW);   // 1-KB wave-loads (8 rows x 128 B) per wavefront per K-tile
  constexpr int NL = LX + LY;
  constexpr int XSTAGE = BM * BKK, YSTAGE = BN * BKK;
  constexpr int NMF = TM * TN, NF = TM + TN;
  constexpr int NSLOT = 4 * NMF;                  // MFMAs between two barriers
  extern __shared__ __align__(1024) unsigned char smem_raw[];
  bf16_t* Xs = reinterpret_cast<bf16_t*>(smem_raw);
  bf16_t* Ys = Xs + SX * XSTAGE;

  // the wavefront id is uniform: keep it (and all LDS destination arithmetic) in scalar registers
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int wm = wave / WN, wn = wave % WN;
  const int l32 = lane & 31, hh = lane >> 5;
  const bool math = NW_MATH == NW || wave < NW_MATH;    // wavefront-uniform

  int i_max, j_max, kz, ti, tj;
  if (EPI == EPI_LMHEAD) {
    // The grid covers the row capacity; the number of rows in use is only known on the device.  The first
    // (vocabulary tiles x token tiles in use) workgroup ids take the real tiles, token tiles running fastest
    // so that the workgroups sharing a vocabulary tile sit next to each other on one XCD; the rest leave.
    i_max = a.N;
    j_max = a.M_dev ? min(*a.M_dev, a.M) : a.M;
    const int used_j = (j_max + BN - 1) / BN;
    const int used = tiles_i * used_j;
    if ((int)blockIdx.x >= used) return;
    const int L = xcd_contiguous(blockIdx.x, used);
    kz = 0;
    ti = L / used_j;
    tj = L % used_j;
  } else {
    // XCD-aware order: workgroup ids go round-robin over the 8 XCDs; give each XCD a contiguous range
    // of logical tiles, running fastest over the activation tiles, so the workgroups that stream the
    // same weight tile share one L2 and run at the same time.
    const int per_z = tiles_i * tiles_j;
    kz = blockIdx.x / per_z;
    const int L = xcd_contiguous(blockIdx.x % per_z, per_z);
    ti = L % tiles_i;
    tj = L / tiles_i;
    i_max = a.M_dev ? min(*a.M_dev, a.M) : a.M;
    j_max = a.N;
    if (ti * BM >= i_max) return;
  }
  const int i0 = ti * BM, j0 = tj * BN;

  const int ldw = a.ldw ? a.ldw : a.K;
  // K range of this slice
  const int KT_all = a.K / BKK;
  const int kt0 = (int)(((long long)KT_all * kz) / a.ksplit);
  const int KT = (int)(((long long)KT_all * (kz + 1)) / a.ksplit) - kt0;

  // ---- global sources.  A wave-load covers 8 rows; lane -> (row, swizzled 16-byte chunk).  Addresses are a
  // wavefront-uniform base (scalar registers) plus a 32-bit per-lane byte offset that never changes: the
  // loads take the scalar-base form and the K loop needs no vector arithmetic for them.
  const char* xbase;
  const char* ybase[LY];
  unsigned xoff[LX], yoff[LY];
  {
    const bf16_t* X = (EPI == EPI_LMHEAD) ? (const bf16_t*)a.W[0] : (const bf16_t*)a.A;
    const int ldx = (EPI == EPI_LMHEAD) ? ldw : a.lda;
    xbase = reinterpret_cast<const char*>(X + (size_t)kt0 * BKK);
#pragma unroll
    for (int q = 0; q < LX; ++q) {
      const int row = 8 * (wave * LX + q) + (lane >> 3);
      const int chunk = (lane & 7) ^ ((row >> 1) & 7);
      const int gi = min(i0 + row, i_max - 1);
      xoff[q] = (unsigned)gi * (unsigned)(ldx * 2) + chunk * 16;
    }
#pragma unroll
    for (int q = 0; q < LY; ++q) {
      const int row0 = 8 * (wave * LY + q);            // first row of the wave-load: uniform
      const int row = row0 + (lane >> 3);
      const int chunk = (lane & 7) ^ ((row >> 1) & 7);
      const bf16_t* base;
      int r;                                            // row inside the matrix `base` points to
      if (EPI == EPI_LMHEAD) {
        base = (const bf16_t*)a.A;
        r = min(j0 + row, j_max - 1);
        yoff[q] = (unsigned)r * (unsigned)(a.lda * 2) + chunk * 16;
      } else {
        if (EPI == EPI_SWIGLU) {
          // rows of every 32-row MFMA tile: 16 gate rows then the 16 up rows of the same features
          base = (row0 & 16) ? (const bf16_t*)a.W[1] : (const bf16_t*)a.W[0];
          r = tj * (BN / 2) + (row >> 5) * 16 + (row & 15);
        } else {
          const int n0 = j0 + row0;   // column of the fused [seg0 | seg1 | seg2] output; 8-row groups never straddle
          int seg0;
          if (n0 < a.Nseg[0]) { base = (const bf16_t*)a.W[0]; seg0 = 0; }
          else if (n0 < a.Nseg[0] + a.Nseg[1]) { base = (const bf16_t*)a.W[1]; seg0 = a.Nseg[0]; }
          else { base = (const bf16_t*)a.W[2]; seg0 = a.Nseg[0] + a.Nseg[1]; }
          r = j0 + row - seg0;
        }
        yoff[q] = (unsigned)r * (unsigned)(ldw * 2) + chunk * 16;
      }
      ybase[q] = reinterpret_cast<const char*>(base + (size_t)kt0 * BKK);
    }
  }
  // 16 bytes per lane, global (scalar base + 32-bit lane offset) -> LDS (M0 = destination of lane 0).  Written
  // out because the compiler only emits the 64-bit-lane-address form, which costs a 64-bit vector add per load.
  auto dma16 = [](const char* ubase, unsigned lane_off, const bf16_t* lds_dst) {
    const unsigned m0v = (unsigned)(size_t)(lds_ptr_t)lds_dst;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(m0v), "v"(lane_off), "s"(ubase) : "memory");
  };
  auto load_x = [&](int q, int t) {
    dma16(xbase + (size_t)t * (BKK * 2), xoff[q], Xs + (t % SX) * XSTAGE + (wave * LX + q) * 512);
  };
  auto load_y = [&](int q, int t) {
    dma16(ybase[q] + (size_t)t * (BKK * 2), yoff[q], Ys + (t % SY) * YSTAGE + (wave * LY + q) * 512);
  };
  constexpr int LS = XDEEP ? LY : LX, LD = XDEEP ? LX : LY;   // wave-loads of the shallow / deep operand
  auto load_sh = [&](int q, int t) { if (XDEEP) load_y(q, t); else load_x(q, t); };
  auto load_dp = [&](int q, int t) { if (XDEEP) load_x(q, t); else load_y(q, t); };
  // load `idx` of group g (the loads issued after barrier g): shallow operand of tile g+SH first, then
  // the deep operand of tile g+SD
  constexpr int SH_AHEAD = SH;
  auto group_load = [&](int idx, int g, bool checked = true) {
    if (idx < LS) { if (!checked || g + SH_AHEAD < KT) load_sh(idx, g + SH_AHEAD); }
    else { if (!checked || g + SD < KT) load_dp(idx - LS, g + SD); }
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // short K: not enough tiles for the steady-state wait counts, wait for everything each time
  const bool short_k = KT <= SD;
  // prologue, in the order the partial waits rely on: D0 S0 | D1 [S1] .. D(SD-2) [S(SD-2)] (shallow tiles up to SH-2)
  // | first quarter of group -1 (what a "K step 3 of tile -1" would have issued); the loop issues the rest
  static_assert(SD >= 3, "the steady-state wait keeps one deep-operand tile in flight across the barrier");
#pragma unroll
  for (int q = 0; q < LD; ++q) load_dp(q, 0);
#pragma unroll
  for (int q = 0; q < LS; ++q) load_sh(q, 0);
#pragma unroll
  for (int t = 1; t < SD - 1; ++t)
    if (t < KT) {
#pragma unroll
      for (int q = 0; q < LD; ++q) load_dp(q, t);
      if (t < SH - 1) {
#pragma unroll
        for (int q = 0; q < LS; ++q) load_sh(q, t);
      }
    }
#pragma unroll
  for (int idx = 0; idx < NL / 4; ++idx) group_load(idx, -1);

  const int sw_r = (l32 >> 1) & 7;
  const int xrow = (wm * RW + l32) * BKK;
  const int yrow = (wn * CW + l32) * BKK;
  bf16x8 fx[2][TM], fy[2][TN];
  auto ldfrag = [&](int buf, const bf16_t* xs, const bf16_t* ys, int kk, int r) {
    if (!math) return;
    const int slot = ((kk * 2 + hh) ^ sw_r) * 8;
    if (r < TM) fx[buf][r] = *reinterpret_cast<const bf16x8*>(xs + xrow + r * 32 * BKK + slot);
    else fy[buf][r - TM] = *reinterpret_cast<const bf16x8*>(ys + yrow + (r - TM) * 32 * BKK + slot);
  };
  // loads younger than tile 0's: the deep halves of tiles 1 .. SD-2, the shallow halves of tiles 1 .. SH-2, and the
  // start of group -1.  Steady state: younger than the shallow operand of the next tile are the deep loads of its
  // own group and the SH-2 groups after it (every group when both rings have the same depth).
  constexpr int W_FIRST = (SD - 2) * LD + (SH - 2) * LS + NL / 4;
  constexpr int W_STEADY = SH == SD ? (SD - 2) * NL : LD + (SH - 2) * NL;
  static_assert(W_FIRST <= 63 && W_STEADY <= 63, "vmcnt is a 6-bit counter");
  if (short_k) wait_vmcnt<0>(); else wait_vmcnt<W_FIRST>();   // tile 0 is in LDS
  __builtin_amdgcn_s_barrier();
#pragma unroll
  for (int r = 0; r < NF; ++r) ldfrag(0, Xs, Ys, 0, r);

  // fragment reads of the next K step issued after MFMA m of the current one: [frag_lo(m), frag_lo(m+1)).
  // One per MFMA from the second on when there are enough MFMAs, else spread over all but the last.
  auto frag_lo = [](int m) {
    if (NMF == 1) return m < 1 ? 0 : NF;
    if (NF <= NMF - 1) return m < 1 ? 0 : (m - 1 < NF ? m - 1 : NF);
    return m < NMF - 1 ? (m * NF) / (NMF - 1) : NF;
  };
  // one K-tile; STEADY = every tile this iteration prefetches exists (no bounds checks, no branches)
  auto k_tile = [&](int kt, auto steady_tag) {
    constexpr bool STEADY = decltype(steady_tag)::value;
    const bf16_t* xs = Xs + (kt % SX) * XSTAGE;
    const bf16_t* ys = Ys + (kt % SY) * YSTAGE;
    // K steps 0..2 of the tile: MFMAs on fragment buffer kk&1, fragments of step kk+1 into the other
    // buffer, remaining loads of group kt-1
#pragma unroll
    for (int kk = 0; kk < 3; ++kk) {
#pragma unroll
      for (int m = 0; m < NMF; ++m) {
        const int i = m / TN, j = m % TN;
        if (math) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fx[kk & 1][i], fy[kk & 1][j], acc[i][j], 0, 0, 0);
#pragma unroll
        for (int r = frag_lo(m); r < frag_lo(m + 1); ++r) ldfrag((kk + 1) & 1, xs, ys, kk + 1, r);
        const int slot = NMF + kk * NMF + m;      // position among the NSLOT MFMAs that follow barrier kt-1
#pragma unroll
        for (int idx = (slot * NL) / NSLOT; idx < ((slot + 1) * NL) / NSLOT; ++idx) group_load(idx, kt - 1, !STEADY);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    // barrier kt: tile kt+1 is in LDS for every wavefront (only the deep-operand loads of group kt-1
    // may still fly), and no wavefront reads the stages of tile kt after this point
    if (STEADY || (!short_k && kt + SD - 1 < KT)) wait_vmcnt<W_STEADY>(); else wait_vmcnt<0>();
    wait_lgkm0();
    __builtin_amdgcn_s_barrier();
    const bf16_t* xs1 = Xs + ((kt + 1) % SX) * XSTAGE;
    const bf16_t* ys1 = Ys + ((kt + 1) % SY) * YSTAGE;
    // K step 3: MFMAs on buffer 1, fragments (kt+1, step 0) into buffer 0, first loads of group kt
#pragma unroll
    for (int m = 0; m < NMF; ++m) {
      const int i = m / TN, j = m % TN;
      if (math) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fx[1][i], fy[1][j], acc[i][j], 0, 0, 0);
#pragma unroll
      for (int r = frag_lo(m); r < frag_lo(m + 1); ++r) ldfrag(0, xs1, ys1, 0, r);
#pragma unroll
      for (int idx = (m * NL) / NSLOT; idx < ((m + 1) * NL) / NSLOT; ++idx) group_load(idx, kt, !STEADY);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // steady state: kt >= 1 (group kt-1 exists as a whole) and kt + SD < KT (everything prefetched exists)
  int kt = 0;
  if (!short_k) {
    k_tile(0, std::false_type{});
    for (kt = 1; kt + SD < KT; ++kt) k_tile(kt, std::true_type{});
  }
  for (; kt < KT; ++kt) k_tile(kt, std::false_type{});
  if (!math) return;      // (no barrier follows the K loop)

  // accumulator element (i,j,v) of this lane: row  = i0 + wm*RW + i*32 + 8*(v/4) + 4*hh + v%4
  //                                           col  = wn*CW + j*32 + l32   (within the tile)
  if (EPI == EPI_LMHEAD) {
    // Per token column: top value, its lowest vocabulary index, runner-up and sum of exponentials over the
    // lane's 64 vocabulary rows, on the unscaled accumulators (the scale is positive, so the order is the
    // same); the lane's rows are visited in increasing vocabulary index, so "strictly greater" keeps the
    // lowest index among equals.  One median-of-three per value maintains the runner-up.
    TopPartial* part = reinterpret_cast<TopPartial*>(a.C);
    const float c = a.scale * 1.4426950408889634f;
    auto reduce_columns = [&](auto checked_tag) {
      constexpr bool CHECKED = decltype(checked_tag)::value;   // the last vocabulary tile: rows beyond V count as -inf
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        float m = -INFINITY, m2 = -INFINITY;
        int code = 0;      // 16 * i + v of the top value
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            float l = acc[i][j][v];
            if (CHECKED) {
              const int idx = i0 + wm * RW + i * 32 + 8 * (v >> 2) + 4 * hh + (v & 3);
              if (idx >= i_max) l = -INFINITY;
              acc[i][j][v] = l;
            }
            m2 = __builtin_amdgcn_fmed3f(m, m2, l);
            code = l > m ? 16 * i + v : code;
            m = __builtin_amdgcn_fmed3f(m, l, INFINITY);   // max(m, l) as one instruction
          }
        // in the last tile a lane may have no row below V: it keeps m = -inf and contributes nothing
        const float mc = (m == -INFINITY) ? 0.f : m * c;
        float sum = 0.f;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int v = 0; v < 16; ++v) sum += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[i][j][v], c, -mc));
        Top t;
        t.m = m * a.scale;
        t.m2 = m2 * a.scale;
        t.s = sum;
        t.idx = (m == -INFINITY) ? 0x7fffffff
                                 : i0 + wm * RW + (code >> 4) * 32 + 8 * ((code & 15) >> 2) + 4 * hh + (code & 3);
        t = top_merge(t, top_shfl_xor(t, 32));
        const int tokr = j0 + wn * CW + j * 32 + l32;
        if (hh == 0 && tokr < j_max) part[(size_t)(ti * 2 + wm) * a.ldc + tokr] = TopPartial{t.m, t.m2, t.s, t.idx};
      }
    };
    if (i0 + BM <= i_max) reduce_columns(std::false_type{}); else reduce_columns(std::true_type{});
    return;
  }

  if (EPI == EPI_PARTIAL) {
    float* P = reinterpret_cast<float*>(a.C) + (size_t)kz * (a.Mz ? a.Mz : a.M) * a.ldc;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int r = i0 + wm * RW + i * 32 + 8 * (v >> 2) + 4 * hh + (v & 3);
        if (r >= i_max) continue;
#pragma unroll
        for (int j = 0; j < TN; ++j) P[(size_t)r * a.ldc + j0 + wn * CW + j * 32 + l32] = acc[i][j][v];
      }
    return;
  }

  bf16_t* C = reinterpret_cast<bf16_t*>(a.C);
  if (EPI == EPI_SWIGLU) {
    // lanes 0-15 of a half hold gate values, lanes 16-31 the up values of the same features.  For every
    // pair of rows (v, v+1) the two lanes swap one value (v_permlane16_swap): the gate lane keeps row v and
    // receives up(v), the up lane keeps row v+1 and receives gate(v+1); each then finishes one row.  Two such
    // row pairs (v, v+1), (v+2, v+3) are stored together: neighbouring lanes (features f, f+1) trade one result,
    // the even lane stores both features of the first pair's row, the odd lane those of the second pair's row.
    typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
    const int up = (l32 & 16) ? 1 : 0, odd = l32 & 1;
    // per-lane part of the address once; the row part below is the same for every lane of the half
    bf16_t* Cl = C + (size_t)(up + 2 * odd) * a.ldc + tj * (BN / 2) + wn * TN * 16 + (l32 & 15) - odd;
    auto silu_mul = [](float g, float u) { return g * __builtin_amdgcn_rcpf(1.f + __expf(-g)) * u; };
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int v = 0; v < 16; v += 4) {
        const int r = i0 + wm * RW + i * 32 + 8 * (v >> 2) + 4 * hh;   // row of accumulator element v in the gate lanes
        const bool ok = r + up + 2 * odd < i_max;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const u32x2 s0 = __builtin_amdgcn_permlane16_swap(__float_as_uint(acc[i][j][v]), __float_as_uint(acc[i][j][v + 1]),
                                                            false, false);
          const u32x2 s1 = __builtin_amdgcn_permlane16_swap(__float_as_uint(acc[i][j][v + 2]), __float_as_uint(acc[i][j][v + 3]),
                                                            false, false);
          const float h0 = silu_mul(__uint_as_float(s0[0]), __uint_as_float(s0[1]));   // row r + up
          const float h1 = silu_mul(__uint_as_float(s1[0]), __uint_as_float(s1[1]));   // row r + 2 + up
          const float keep = odd ? h1 : h0;
          const float got = __shfl_xor(odd ? h0 : h1, 1, 64);
          bf16x2 out2;
          out2[0] = static_cast<bf16_t>(odd ? got : keep);
          out2[1] = static_cast<bf16_t>(odd ? keep : got);
          if (ok) *reinterpret_cast<bf16x2*>(Cl + (size_t)r * a.ldc + j * 16) = out2;
        }
      }
    return;
  }

  const bf16_t* R = reinterpret_cast<const bf16_t*>(a.R);
  const bool has_bias = EPI == EPI_STORE && (a.bias[0] || a.bias[1] || a.bias[2]);
  // rows (v, v+1) of two neighbouring columns are regrouped so that every lane stores one 4-byte pair: the
  // even lane takes row v (its own column and the next one), the odd lane row v+1
  const int odd = l32 & 1;
  float bv[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int n = j0 + wn * CW + j * 32 + l32;
    bv[j] = 0.f;
    if (has_bias) {
      const bf16_t* bp = nullptr;
      if (n < a.Nseg[0]) { if (a.bias[0]) bp = (const bf16_t*)a.bias[0] + n; }
      else if (n < a.Nseg[0] + a.Nseg[1]) { if (a.bias[1]) bp = (const bf16_t*)a.bias[1] + (n - a.Nseg[0]); }
      else { if (a.bias[2]) bp = (const bf16_t*)a.bias[2] + (n - a.Nseg[0] - a.Nseg[1]); }
      if (bp) bv[j] = static_cast<float>(*bp);
    }
  }
  // per-lane part of the address once; the row part below is the same for every lane of the half
  const size_t lane_off = (size_t)odd * a.ldc + (j0 + wn * CW + l32 - odd);
  bf16_t* Cl = C + lane_off;
  const bf16_t* Rl = R + lane_off;
  auto store_all = [&](auto checked_tag) {
    constexpr bool CHECKED = decltype(checked_tag)::value;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int v = 0; v < 16; v += 2) {
        const int r = i0 + wm * RW + i * 32 + 8 * (v >> 2) + 4 * hh + (v & 3);   // the even lane's row
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          float a0 = acc[i][j][v] + bv[j], a1 = acc[i][j][v + 1] + bv[j];
          asm volatile("" : "+v"(a0), "+v"(a1));   // two plain selects below, not a lane-indexed element extract
          const float keep = odd ? a1 : a0;
          const float give = odd ? a0 : a1;
          const float got = __shfl_xor(give, 1, 64);
          float lo = odd ? got : keep, hi = odd ? keep : got;   // columns n-odd, n-odd+1 of row r+odd
          if (CHECKED && r + odd >= i_max) continue;
          const size_t o = (size_t)r * a.ldc + j * 32;
          if (EPI == EPI_RESID) {
            const bf16x2 rr = *reinterpret_cast<const bf16x2*>(Rl + o);
            lo += static_cast<float>(rr[0]);
            hi += static_cast<float>(rr[1]);
          }
          bf16x2 out2;
          out2[0] = static_cast<bf16_t>(lo);
          out2[1] = static_cast<bf16_t>(hi);
          *reinterpret_cast<bf16x2*>(Cl + o) = out2;
        }
      }
  };
  if (i0 + BM <= i_max) store_all(std::false_type{}); else store_all(std::true_type{});
}

template <int EPI, int BN, int SD, int BMT, int SA>
constexpr size_t smem_bytes() {
  constexpr int SH = shallow_stages(EPI, BN, BMT, SD, SA);
  return sizeof(bf16_t) * (size_t)(EPI == EPI_LMHEAD ? SD * BMT + SH * BN : SH * BMT + SD * BN) * BKK;
}

template <int EPI, int BN, int SD, int BMT = 256, int SA = 0>
hipError_t launch_t(const GemmArgs& a, int tiles_i, int tiles_j, hipStream_t st) {
  static_assert(smem_bytes<EPI, BN, SD, BMT, SA>() <= 160 * 1024, "a workgroup has 160 KB of LDS");
  static std::atomic<unsigned long long> lds_ok{0};
  const hipError_t e = allow_dynamic_lds((const void*)gemm_bf16_mfma_kernel<EPI, BN, SD, BMT, SA>,
                                         (int)smem_bytes<EPI, BN, SD, BMT, SA>(), lds_ok);
  if (e != hipSuccess) return e;
  gemm_bf16_mfma_kernel<EPI, BN, SD, BMT, SA><<<tiles_i * tiles_j * a.ksplit, 64 * waves_m(BMT, BN) * waves_n(BN), smem_bytes<EPI, BN, SD, BMT, SA>(), st>>>(a, tiles_i, tiles_j);
  return hipGetLastError();
}

// out[m,:] = R[m,:] + sum_z P[z][m,:]  (fixed order), optionally followed by RMSNorm of that row.
// One workgroup per row, of 256 or 1024 threads: with few rows the launch is latency-bound and 1024 threads have every
// load of a row in flight at once.  The thread count is scheduling only.  The row's sum of squares is defined by the
// 256-thread order: a lane adds the sums of its four elements over the 256-element chunks w, w+4, w+8, .. (w = its
// wavefront), the 64 lanes of a wavefront are summed, then the four wavefront sums.  With 1024 threads every
// (chunk, lane) sum goes through LDS and the first four wavefronts add them in that same order.
template <bool NORM>
__global__ __launch_bounds__(1024) void splitk_reduce_kernel(const float* __restrict__ P, int ksplit,
                                                            const bf16_t* __restrict__ R, bf16_t* __restrict__ out,
                                                            const bf16_t* __restrict__ gain, float eps,
                                                            bf16_t* __restrict__ normed, int M, int N,
                                                            const int32_t* __restrict__ n_rows_dev,
                                                            const int32_t* __restrict__ out_rows) {
  __shared__ float red[4];
  extern __shared__ float rowbuf[];               // NORM: the row in fp32; 1024 threads: then one sum per (chunk, lane)
  const int m = blockIdx.x;
  if (n_rows_dev && m >= *n_rows_dev) return;
  const size_t mo = out_rows ? (size_t)out_rows[m] : (size_t)m;     // where the row goes (compacted rows scatter back)
  const int stride = 4 * (int)blockDim.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const bool wide = blockDim.x > 256;
  float* lane_ss = rowbuf + N;
  float ss = 0.f;
  for (int base = wave * 256; base < N; base += stride) {     // wavefront-uniform: one chunk per trip
    const int n = base + lane * 4;
    float c = 0.f;
    if (n < N) {
      f32x4 s = *reinterpret_cast<const f32x4*>(P + (size_t)m * N + n);
      for (int z = 1; z < ksplit; ++z) {
        const f32x4 p = *reinterpret_cast<const f32x4*>(P + ((size_t)z * M + m) * N + n);
        s[0] += p[0]; s[1] += p[1]; s[2] += p[2]; s[3] += p[3];
      }
      const bf16x4 r = *reinterpret_cast<const bf16x4*>(R + (size_t)m * N + n);
      bf16x4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        s[e] += static_cast<float>(r[e]);
        o[e] = static_cast<bf16_t>(s[e]);
        if (NORM) { rowbuf[n + e] = s[e]; c += s[e] * s[e]; }
      }
      *reinterpret_cast<bf16x4*>(out + mo * N + n) = o;
    }
    if (NORM) {
      if (wide) lane_ss[(base >> 8) * 64 + lane] = c; else ss += c;
    }
  }
  if (!NORM) return;
  if (wide) {
    __syncthreads();
    if (wave < 4)
      for (int k = wave; k < (N + 255) / 256; k += 4) ss += lane_ss[k * 64 + lane];
  }
  if (wave < 4) {
    ss = wave_sum(ss);
    if (lane == 0) red[wave] = ss;
  }
  __syncthreads();
  const float inv = 1.0f / sqrtf((red[0] + red[1] + red[2] + red[3]) / (float)N + eps);
  for (int n = threadIdx.x * 4; n < N; n += stride) {
    const bf16x4 g = *reinterpret_cast<const bf16x4*>(gain + n);
    bf16x4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = static_cast<bf16_t>(rowbuf[n + e] * inv * static_cast<float>(g[e]));
    *reinterpret_cast<bf16x4*>(normed + (size_t)m * N + n) = o;
  }
}

}  // namespace

// number of K slices for the narrow-N projections: a function of (N, K) only
int mfma_ksplit(int N, int K) {
  const int n_tiles = cdiv(N, 128), kt = K / BKK;
  int ks = 1;
  while (ks < 4 && 4 * n_tiles * ks < 224 && kt / (ks + 1) >= 8) ++ks;
  // and no slice longer than 128 K-tiles (8192 elements): a split-K launch is one round of workgroups whose time is the
  // slice length.  K = 18944 over 768 rows and 3584 columns: 118.5 us with two slices (168 workgroups), 97.2 us with
  // three (252), 129.7 us with four (two rounds); 1024 rows of that shape pay for it (336 workgroups with three).
  const int by_length = cdiv(kt, 128);
  if (by_length > ks) ks = by_length < 4 ? by_length : 4;
  return ks;
}

bool mfma_gemm_supported(int epi, const GemmArgs& a) {
  if (a.K % BKK != 0 || a.K < BKK || a.M < 1) return false;
  // per-lane byte offsets inside an operand are 32-bit
  const size_t lim = (size_t)1 << 32;
  const size_t ldw = a.ldw ? a.ldw : a.K;
  if ((size_t)a.M * a.lda * 2 >= lim || (size_t)a.N * ldw * 2 >= lim) return false;
  if (epi == EPI_SWIGLU) return a.N % 32 == 0;
  if (epi == EPI_LMHEAD) return a.N >= 1;
  if (a.N % 64 != 0) return false;
  int n = 0;
  for (int s = 0; s < 3; ++s) {
    if (a.Nseg[s] < 0 || a.Nseg[s] % 8 != 0) return false;
    n += a.Nseg[s];
  }
  return n == a.N && a.Nseg[0] > 0;
}

int mfma_lmhead_partials_per_row(int V) { return cdiv(V, BM) * 2; }

// Tile shape: a pure scheduling choice (it never changes the K order of any output element, so a row's result
// is bit-identical whatever shape runs it).  Estimated cost = rounds over the 256 CUs x time of one K-tile of
// one workgroup, the larger of its matrix-pipe time (32 cycles per 32x32x16 MFMA, 4 K steps, a penalty for
// narrow tiles) and the time to bring its operands in (about 40 bytes per clock per CU).  With few rows
// (one or a few states) the projections are weight-streaming problems: 64- and 128-row tiles spend a quarter
// or half of the matrix work of a 256-row tile on them and cover more CUs.
struct TileShape { int bm, bn; };
static const int kTileWidths[5] = {192, 128, 96, 64, 32};
// estimated time of one K-tile of one workgroup of shape bm x kTileWidths[wi]
static float tile_cost(int bm, int wi) {
  const float eff[5] = {1.0f, 0.85f, 0.6f, 0.55f, 0.4f};
  const int bn = kTileWidths[wi];
  const float mfma = (float)(bm / 64) * ((float)bn / 64.0f) * 128.0f / eff[wi];
  const float load = (float)(bm + bn) * 3.2f;
  return mfma > load ? mfma : load;
}
static TileShape choose_tile(int M, int n_cols, int unit, int ksplit, bool allow192, bool allow32 = false, bool allow96 = false,
                             bool allow96_two_rows = false, float* cost_out = nullptr) {
  const int heights[4] = {256, 128, 64, 32};
  const int* widths = kTileWidths;
  TileShape best = {256, 0};
  float best_cost = 1e30f;
  for (int h = 0; h < 4; ++h)
    for (int i = 0; i < 5; ++i) {
      const int bm = heights[h], bn = widths[i];
      const int cols = bn / unit;                 // output columns (or SwiGLU features) per tile
      if ((bn == 192 && (!allow192 || bm <= 64)) || (bn == 64 && bm == 128) || n_cols % cols != 0) continue;
      // 96-wide tiles: one row of tiles over few rows (weight streaming), where they turn 192 workgroups into 256
      // (the QKV projection also takes them over two rows of 128- or 64-row tiles: 256 workgroups where 128 columns
      // give 192; 41.4 against 43.3 us at 256 rows, 31.9 against 35.2 us at 128 rows in interleaved runs)
      if (bn == 96 && !((allow96 && (bm == 64 || bm == 128) && M <= bm) ||
                        (allow96_two_rows && (bm == 64 || bm == 128) && M <= 2 * bm))) continue;
      // 32-wide tiles (one or two wavefronts per workgroup) exist for the split-K projections of one or two states
      if ((bn == 32 || bm == 32) && !(allow32 && bn == 32 && bm <= 64)) continue;
      const int tiles = cdiv(M, bm) * (n_cols / cols) * ksplit;
      const float cost = (float)cdiv(tiles, 256) * tile_cost(bm, i);
      if (cost < best_cost) { best_cost = cost; best = {bm, bn}; }
    }
  if (cost_out) *cost_out = best_cost;
  return best;
}

template <int EPI>
static hipError_t launch_shape(const GemmArgs& a, TileShape t, int unit, hipStream_t st) {
  const int mt = cdiv(a.M, t.bm), nt = a.N / (t.bn / unit);
  constexpr bool W192 = EPI != EPI_PARTIAL;       // the split-K projections never take the 192-wide tile
  if (t.bm == 256) {
    if constexpr (W192) if (t.bn == 192) return launch_t<EPI, 192, 3>(a, mt, nt, st);
    // 256 x 128: room for a third activation stage beside four weight stages (160 KB); in interleaved A/B runs 2-5%
    // faster than two stages on every projection that takes this tile (down projection 95.9 -> 91.4 us at 1024 rows)
    if (t.bn == 128) return launch_t<EPI, 128, 4, 256, 3>(a, mt, nt, st);
    return launch_t<EPI, 64, 4>(a, mt, nt, st);
  }
  // few rows: the weight ring is as deep as the LDS allows (bytes in flight are what sets the streaming rate)
  if constexpr (EPI == EPI_SWIGLU) {
    if (t.bn == 96) return t.bm == 128 ? launch_t<EPI, 96, 5, 128>(a, mt, nt, st) : launch_t<EPI, 96, 7, 64>(a, mt, nt, st);
  }
  if constexpr (EPI == EPI_STORE) {
    if (t.bn == 96) return t.bm == 128 ? launch_t<EPI, 96, 4, 128>(a, mt, nt, st) : launch_t<EPI, 96, 6, 64>(a, mt, nt, st);
  }
  if (t.bm == 128) {
    if constexpr (W192) if (t.bn == 192) return launch_t<EPI, 192, 4, 128>(a, mt, nt, st);
    return launch_t<EPI, 128, 4, 128>(a, mt, nt, st);
  }
  if constexpr (EPI == EPI_PARTIAL) {
    if (t.bm == 32) return launch_t<EPI, 32, 9, 32>(a, mt, nt, st);
    if (t.bn == 32) return launch_t<EPI, 32, 10, 64>(a, mt, nt, st);
  }
  if (t.bn == 64) return launch_t<EPI, 64, 8, 64>(a, mt, nt, st);
  return launch_t<EPI, 128, 6, 64>(a, mt, nt, st);
}

// The launches of one projection: one, or two column ranges (the two-part schedule of the gate/up projection).
// Host arithmetic only; launch_gemm_mfma executes exactly this plan.
GemmPlan plan_gemm_mfma(int epi, int M, int N, int ksplit) {
  GemmPlan p = {};
  if (ksplit < 1) ksplit = 1;
  auto one = [&](TileShape t, int unit) {
    p.n_parts = 1;
    p.part[0] = {t.bm, t.bn, 0, N, cdiv(M, t.bm) * (N / (t.bn / unit)) * ksplit};
  };
  switch (epi) {
    case EPI_STORE:
      one(choose_tile(M, N, 1, 1, true, false, false, true), 1);
      break;
    case EPI_RESID: {
      // 256-row tiles only; 128 columns wide unless N is an odd multiple of 64 or the narrower tile fills the chip better
      const TileShape t = choose_tile(M, N, 1, 1, false);
      one(TileShape{256, (N % 128 != 0 || (t.bm == 256 && t.bn == 64)) ? 64 : 128}, 1);
      break;
    }
    case EPI_PARTIAL:
      one(choose_tile(M, N, 1, ksplit, false, true), 1);
      break;
    case EPI_SWIGLU: {
      float whole = 0.f;
      const TileShape t = choose_tile(M, N, 2, 1, true, false, true, false, &whole);   // a tile of width w holds w/2 features
      one(t, 2);
      // Two-part column schedule, for widths whose best single shape leaves the last round of workgroups mostly empty
      // (18944 features over 768 rows: 888 tiles of 256 x 128 = 3.47 rounds, and 96 does not divide the width; over 128
      // rows: 296 tiles of 128 x 128, 1.16 rounds): one shape over as many leading features as fill whole rounds of the
      // 256 CUs - 256 x 192 tiles, or the best single shape - then the best shape for the rest, as a second launch on
      // the same stream.  Same K order in every shape, so the output bits are those of the single launch; measured
      // 207.8 -> 190.5 us at 768 rows (170 column tiles of 256 x 192, then 246 tiles of 128 x 128) and 83.9 -> 69.7 us
      // at 128 rows (256 tiles of 128 x 128, then 160 of 64 x 64).
      float best = 0.9f * whole;          // a second launch has to promise at least a tenth
      auto try_main = [&](TileShape tm) {
        int wi = 0;
        while (wi < 5 && kTileWidths[wi] != tm.bn) ++wi;
        if (wi == 5) return;
        const int per = tm.bn / 2, mt = cdiv(M, tm.bm);               // features per tile, row tiles
        const int rounds = (int)(((long long)mt * (N / per)) / 256);
        if (rounds < 1) return;
        const int main_tiles = (256 * rounds) / mt;                    // column tiles of the first part
        const int rest = N - per * main_tiles;                         // features left; a multiple of 32 as N is
        if (rest <= 0) return;
        float rest_cost = 0.f;
        const TileShape tr = choose_tile(M, rest, 2, 1, true, false, true, false, &rest_cost);
        const float cost = (float)rounds * tile_cost(tm.bm, wi) + rest_cost;
        if (tr.bn == 0 || cost > best) return;
        best = cost;
        p.n_parts = 2;
        p.part[0] = {tm.bm, tm.bn, 0, per * main_tiles, mt * main_tiles};
        p.part[1] = {tr.bm, tr.bn, per * main_tiles, rest, cdiv(M, tr.bm) * (rest / (tr.bn / 2))};
      };
      try_main(TileShape{256, 192});
      if (t.bn != 0 && !(t.bm == 256 && t.bn == 192)) try_main(t);
      break;
    }
    case EPI_LMHEAD:      // vocabulary rows x token columns; the token tiles in use are only known on the device
      p.n_parts = 1;
      p.part[0] = {256, 192, 0, N, cdiv(N, BM) * cdiv(M, 192)};
      break;
    default:
      break;
  }
  return p;
}

hipError_t launch_gemm_mfma(int epi, const GemmArgs& a0, hipStream_t st) {
  GemmArgs a = a0;
  if (a.ksplit < 1) a.ksplit = 1;
  const GemmPlan p = plan_gemm_mfma(epi, a.M, a.N, a.ksplit);
  if (p.n_parts < 1) return hipErrorInvalidValue;
  switch (epi) {
    case EPI_STORE:
      return launch_shape<EPI_STORE>(a, TileShape{p.part[0].bm, p.part[0].bn}, 1, st);
    case EPI_RESID:
      if (p.part[0].bn == 64) return launch_t<EPI_RESID, 64, 4>(a, cdiv(a.M, BM), a.N / 64, st);
      return launch_t<EPI_RESID, 128, 4>(a, cdiv(a.M, BM), a.N / 128, st);
    case EPI_PARTIAL:
      return launch_shape<EPI_PARTIAL>(a, TileShape{p.part[0].bm, p.part[0].bn}, 1, st);
    case EPI_SWIGLU: {
      const size_t ldw = a.ldw ? a.ldw : a.K;
      for (int i = 0; i < p.n_parts; ++i) {
        GemmArgs g = a;
        g.N = p.part[i].ncols;
        g.W[0] = (const bf16_t*)a.W[0] + (size_t)p.part[i].col0 * ldw;
        g.W[1] = (const bf16_t*)a.W[1] + (size_t)p.part[i].col0 * ldw;
        g.C = (bf16_t*)a.C + p.part[i].col0;
        const hipError_t e = launch_shape<EPI_SWIGLU>(g, TileShape{p.part[i].bm, p.part[i].bn}, 2, st);
        if (e != hipSuccess) return e;
      }
      return hipSuccess;
    }
    case EPI_LMHEAD:
      return launch_t<EPI_LMHEAD, 192, 3>(a, cdiv(a.N, BM), cdiv(a.M, 192), st);
    default:
      return hipErrorInvalidValue;
  }
}

hipError_t launch_splitk_reduce(const float* P, int ksplit, const void* R, void* out, const void* gain, float eps,
                                void* normed, int M, int N, hipStream_t st, const int32_t* n_rows_dev,
                                const int32_t* out_rows) {
  // 1024 threads per row with few rows, while the row and its (chunk, lane) sums fit the 64 KB a launch gets by default
  const bool wide_fits = sizeof(float) * ((size_t)N + 64 * ((N + 255) / 256)) <= 64 * 1024;
  const int threads = (N >= 4096 && M <= 512 && (!normed || wide_fits)) ? 1024 : 256;
  if (normed)
    splitk_reduce_kernel<true><<<M, threads, sizeof(float) * ((size_t)N + (threads > 256 ? 64 * ((N + 255) / 256) : 0)), st>>>(P, ksplit, (const bf16_t*)R, (bf16_t*)out,
                                                                       (const bf16_t*)gain, eps, (bf16_t*)normed, M, N,
                                                                       n_rows_dev, out_rows);
  else
    splitk_reduce_kernel<false><<<M, threads, 0, st>>>(P, ksplit, (const bf16_t*)R, (bf16_t*)out, nullptr, 0.f, nullptr, M, N,
                                                   n_rows_dev, out_rows);
  return hipGetLastError();
}

}  // namespace spiffy

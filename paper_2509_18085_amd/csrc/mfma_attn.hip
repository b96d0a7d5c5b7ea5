// Shared-prefix block attention for gfx950 (bf16 MFMA, head_dim 128).
//
// Every one of the G states attends to the same P cached keys and to its own B keys only
// (Fig. 4: a draft block sees the true context and itself; Sec. 3.1 prefix caching).  The mask is
// never built: the prefix part is dense and shared, the own-block part is the block diagonal of
// the (G*B) x (G*B) score matrix.
//
// Work split: one workgroup = (query head, 128 consecutive query rows, one split of the prefix).
// A prefix K/V tile of 64 keys is staged in LDS once and used by all 128 query rows (4 states of
// 32 tokens, or 32 states of 4); workgroups of the same head run next to each other on one XCD
// so the tile comes from HBM once and from L2 afterwards.  The number of prefix splits depends on
// P only, so a row's arithmetic does not depend on G.  With few states (fewer such workgroups than CUs) a
// workgroup owns 96, 64 or 32 of the 128 rows instead and the other wavefront pairs only move data: more CUs
// stream, nothing else changes.  A step that carries a second group of rows (the recomputed suffix of a
// full-sequence model, or the block being committed) runs both attention problems in one launch.
//
// Everything the workgroup reads travels global -> LDS directly as whole 256-byte rows (LDS-DMA loads, no
// registers): the 128 Q rows and the own-block K/V rows once at the start, the prefix tiles into a ring of
// NSTAGE stages, up to NSTAGE-1 tiles ahead of the MFMAs, one barrier per tile.  Rows keep their [row][hd]
// layout in LDS, 16-byte chunks permuted per row so that fragment reads are conflict-free:
//   Q / K row r: chunk c sits at position c ^ (r & 15)      (16-byte reads of one chunk per lane)
//   V row r: 64-byte unit u sits at position u ^ (r & 3)    (transposing 8-byte reads, below)
// The loop over full prefix tiles is software-pipelined: the score MFMAs of tile t+1 are issued between
// the exponentials of tile t.  The O rescale is skipped when no lane's running maximum moved (multiplying
// by exactly 1 changes nothing).
//
// Eight wavefronts per workgroup: wavefront pair p owns query rows 32p..32p+31, and the two wavefronts
// of a pair split every 64-key tile between them (32 keys each), each keeping its own running
// (max, sum, O); the pair is merged through LDS at the end.  Two wavefronts per SIMD let the softmax
// arithmetic of one overlap the MFMAs of the other.
//
// Per wavefront (32 query rows x 32 keys of a tile) everything is kept "query per lane":
//   S^T = K Q^T    A operand = K rows from LDS, B operand = rotated, pre-scaled Q in registers
//                  -> lane (q, half) holds 16 of the 32 keys of a sub-tile for its query q
//   online softmax max / sum are reductions over the lane's own registers plus one half swap
//   O^T = V^T P^T  A operand = V^T, read from the row-major V tile with the transposing LDS read
//                  (ds_read_b64_tr_b16: in every group of 16 lanes, lane 4q+c receives element c of the
//                  8-byte pieces addressed by lanes q, q+4, q+8, q+12), B operand = P^T straight from
//                  the S^T accumulators (no trip through LDS); the rescale factor is per lane.
// Own-block keys (the block diagonal) come first, handled by the last prefix split: they always go to the
// wavefront of a pair that takes the first key half, 32 keys at a time in row order, so a state's arithmetic does not depend on
// where its rows sit in the tile; the mask is applied per element (any B works).
// Rotary embedding (positions pos0..pos0+B-1 for every state, Sec. 4.3) is applied to the Q and own-block K
// fragments in registers, on their way from LDS to the matrix pipe; the cached prefix K arrives rotated.
#include <type_traits>

#include "kernels.h"

namespace spiffy {

namespace {

constexpr int HD = 128;
constexpr int KTILE = 64;
constexpr int QTILE = 128;
constexpr int NSTAGE = 4;
constexpr int TILE_ELEMS = KTILE * HD;          // one K or V tile: 16 KB
constexpr int STAGE_ELEMS = 2 * TILE_ELEMS;     // K tile then V tile
constexpr int SPLIT_KEYS = 2048;
constexpr size_t kAttnSmem = sizeof(bf16_t) * NSTAGE * STAGE_ELEMS;  // 131,072 B

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* glb_ptr_t;
typedef __attribute__((address_space(3))) bf16x4* lds_bf16x4_ptr_t;

constexpr int NT = 512;   // threads per workgroup
constexpr int DMA_PER_TILE = 4;   // LDS-DMA loads per thread per prefix tile (2 for K, 2 for V)

template <int N>
__device__ __forceinline__ void wait_vmcnt() {   // vmcnt <= N; lgkmcnt / expcnt untouched
  __builtin_amdgcn_s_waitcnt((N & 0xF) | (7 << 4) | (0xF << 8) | ((N >> 4) << 14));
}

// position (in 16-byte chunks) of chunk c of row r inside the LDS tiles
__device__ __forceinline__ int k_pos(int r, int c) { return c ^ (r & 15); }
__device__ __forceinline__ int v_pos(int r, int c) { return c ^ ((r & 3) << 2); }

struct WaveState {
  bf16x8 qf[8];     // rotated, scaled Q^T fragments: hd = 16*kk + 8*half + e
  f32x16 o[4];      // O^T accumulators: hd = 32*n + 8*(v/4) + 4*half + v%4, query = lane%32
  float m_run, l_run;
};

// O *= alpha, in place (the multiplies are opaque to the compiler so that the rarely taken branch around
// them does not cost a copy of the 64 accumulator registers on every tile)
__device__ __forceinline__ void rescale_in_place(WaveState& w, float alpha) {
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      float x = w.o[n][v];
      asm volatile("v_mul_f32 %0, %1, %0" : "+v"(x) : "v"(alpha));
      w.o[n][v] = x;
    }
}

// max of a value and its partner 32 lanes away, without a trip through LDS: after the swap one result
// holds the low half's values in both halves, the other the high half's
__device__ __forceinline__ float max_with_other_half(float x) {
  typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
  const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// Reference value m of the online softmax (probabilities are exp2(s - m), log2 domain).  It only follows the running
// maximum when that has moved by more than 8: until then exp2(s - m) stays below 2^8, which bf16 and the fp32 sums
// hold as well as values below 1, and a reference that stays put needs no rescale of O and l (the factor is exactly
// 1 and the 64 multiplies are skipped).  The choice is made per query, so a row's arithmetic does not depend on the
// rows that share its wavefront; (m, l, O) stay consistent and every later merge weighs partials by exp2(m - max m).
__device__ __forceinline__ float next_reference(float m_run, float tile_max) {
  const float m_cand = fmaxf(m_run, tile_max);
  return (m_cand - m_run > 8.0f) ? m_cand : m_run;     // first tile: m_run = -inf, the difference is +inf
}

// S^T of the wavefront's 32-key half of a tile in LDS: 8 MFMAs
__device__ __forceinline__ void scores(const WaveState& w, f32x16& s, const bf16_t* __restrict__ ks, int st, int lane) {
  const int row = st * 32 + (lane & 31), hh = lane >> 5;
  const bf16_t* kp = ks + row * HD;
#pragma unroll
  for (int v = 0; v < 16; ++v) s[v] = 0.f;
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) {
    const bf16x8 kf = *reinterpret_cast<const bf16x8*>(kp + k_pos(row, 2 * kk + hh) * 8);
    s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, w.qf[kk], s, 0, 0, 0);
  }
}

// Online-softmax update and O += P V for the 32 keys of half `st` of a tile whose scores `s` are in registers
// (log2 domain: Q carries log2(e)/sqrt(hd)).  `valid(key_in_tile)` masks keys (only called when MASKED).
template <bool MASKED, typename ValidFn>
__device__ __forceinline__ void finish_tile(WaveState& w, f32x16& s, const bf16_t* __restrict__ vs, int st, int lane, ValidFn valid) {
  const int hh = lane >> 5;
  float tmax = -INFINITY;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    if (MASKED) {
      const int key = st * 32 + 8 * (v >> 2) + 4 * hh + (v & 3);
      if (!valid(key)) s[v] = -INFINITY;
    }
    tmax = fmaxf(tmax, s[v]);
  }
  tmax = max_with_other_half(tmax);
  const float m_new = next_reference(w.m_run, tmax);
  const float alpha = (w.m_run == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(w.m_run - m_new);
  const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
  bf16x8 pf[2];
  float psum = 0.f;
  const bf16x2 ones = {static_cast<bf16_t>(1.0f), static_cast<bf16_t>(1.0f)};
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    f32x2 e;
    e[0] = __builtin_amdgcn_exp2f(s[2 * i] - m_safe);
    e[1] = __builtin_amdgcn_exp2f(s[2 * i + 1] - m_safe);
    const bf16x2 pb = __builtin_convertvector(e, bf16x2);
    psum = __builtin_amdgcn_fdot2_f32_bf16(pb, ones, psum, false);
    pf[i >> 2][(2 * i) & 7] = pb[0];
    pf[i >> 2][(2 * i + 1) & 7] = pb[1];
  }
  w.l_run = w.l_run * alpha + psum;
  w.m_run = m_new;
  // multiplying by exactly 1 changes nothing: skip the rescale when no lane's maximum moved
  if (__builtin_amdgcn_ballot_w64(alpha != 1.f) != 0) rescale_in_place(w, alpha);
  // V^T fragments: lane j of a 16-lane group addresses key (j / 4) of its 4-key run, hd block 4 * (j % 4)
  // of the group's 16 rows; the transposing read hands lane 4q+c the 4 keys of hd row 4q+c
  const int g = lane >> 4, j = lane & 15;
  const int vkey = st * 32 + 4 * (g >> 1) + (j >> 2);     // + 16*k2 + 8*eh, which keep (key & 3)
  const bf16_t* vp = vs + vkey * HD + 16 * (g & 1) + 4 * (j & 3);
#pragma unroll
  for (int n = 0; n < 4; ++n) {
    const int unit = (n ^ (vkey & 3)) * 32;
#pragma unroll
    for (int k2 = 0; k2 < 2; ++k2) {
      const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr_t)(vp + (16 * k2) * HD + unit));
      const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr_t)(vp + (16 * k2 + 8) * HD + unit));
      bf16x8 vf;
      vf[0] = lo[0]; vf[1] = lo[1]; vf[2] = lo[2]; vf[3] = lo[3];
      vf[4] = hi[0]; vf[5] = hi[1]; vf[6] = hi[2]; vf[7] = hi[3];
      w.o[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[k2], w.o[n], 0, 0, 0);
    }
  }
}

// The wavefront's 32-key half (`st`) of a 64-key tile in LDS against its 32 queries
template <bool MASKED, typename ValidFn>
__device__ __forceinline__ void process_tile(WaveState& w, const bf16_t* __restrict__ ks, const bf16_t* __restrict__ vs,
                                             int st, int lane, ValidFn valid) {
  f32x16 s;
  scores(w, s, ks, st, lane);
  finish_tile<MASKED>(w, s, vs, st, lane, valid);
}

// One step of the software pipeline over full prefix tiles: the online-softmax arithmetic on the scores
// `s` of tile t runs between the score MFMAs of tile t+1 (K from `k_next`, result in `sn`, when NEXT),
// then O += P V for tile t (V from `v_cur`).  Same arithmetic, in the same order, as process_tile<false>.
template <bool NEXT>
__device__ __forceinline__ void pipe_step(WaveState& w, const f32x16& s, f32x16& sn, const bf16_t* __restrict__ k_next,
                                          const bf16_t* __restrict__ v_cur, int st, int lane) {
  const int l32 = lane & 31, hh = lane >> 5;
  bf16x8 kf[8];
  if (NEXT) {
    const int row = st * 32 + l32;
    const bf16_t* kp = k_next + row * HD;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) kf[kk] = *reinterpret_cast<const bf16x8*>(kp + k_pos(row, 2 * kk + hh) * 8);
  }
  float tmax = s[0];
#pragma unroll
  for (int v = 1; v < 16; ++v) tmax = fmaxf(tmax, s[v]);
  tmax = max_with_other_half(tmax);
  const float m_new = next_reference(w.m_run, tmax);     // finite: a full tile has no masked score
  const float alpha = (w.m_run == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(w.m_run - m_new);
  const int g = lane >> 4, j = lane & 15;
  const int vkey = st * 32 + 4 * (g >> 1) + (j >> 2);
  const bf16_t* vp = v_cur + vkey * HD + 16 * (g & 1) + 4 * (j & 3);
  if (NEXT) {
#pragma unroll
    for (int v = 0; v < 16; ++v) sn[v] = 0.f;
  }
  bf16x8 pf[2];
  bf16x4 vlo[8], vhi[8];
  float psum = 0.f;
  const bf16x2 ones = {static_cast<bf16_t>(1.0f), static_cast<bf16_t>(1.0f)};
  __builtin_amdgcn_sched_barrier(0);   // K fragment reads and the running-max chain stay above this line
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    if (NEXT) sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i], w.qf[i], sn, 0, 0, 0);
    f32x2 e;
    e[0] = __builtin_amdgcn_exp2f(s[2 * i] - m_new);
    e[1] = __builtin_amdgcn_exp2f(s[2 * i + 1] - m_new);
    const bf16x2 pb = __builtin_convertvector(e, bf16x2);
    psum = __builtin_amdgcn_fdot2_f32_bf16(pb, ones, psum, false);
    pf[i >> 2][(2 * i) & 7] = pb[0];
    pf[i >> 2][(2 * i + 1) & 7] = pb[1];
    {   // V^T fragment i: key step k2 = i / 4, hd block n = i % 4
      const int k2 = i >> 2, n = i & 3;
      const int unit = (n ^ (vkey & 3)) * 32;
      vlo[i] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr_t)(vp + (16 * k2) * HD + unit));
      vhi[i] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr_t)(vp + (16 * k2 + 8) * HD + unit));
    }
  }
  // issue order for the loop above: per score MFMA two exponentials with their subtract / convert / sum
  // and two V fragment reads
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    if (NEXT) __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);
    __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
    __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);
  }
  w.l_run = w.l_run * alpha + psum;
  w.m_run = m_new;
  // the branch below must not move above the block it follows: make its condition depend on the block's results
  float alpha_c = alpha;
  if (NEXT) asm volatile("" : "+v"(alpha_c) : "v"(psum), "v"(sn[15]));
  else asm volatile("" : "+v"(alpha_c) : "v"(psum));
  if (__builtin_amdgcn_ballot_w64(alpha_c != 1.f) != 0) rescale_in_place(w, alpha_c);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const bf16x8 vf = __builtin_shufflevector(vlo[i], vhi[i], 0, 1, 2, 3, 4, 5, 6, 7);
    w.o[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[i >> 2], w.o[i & 3], 0, 0, 0);
  }
}

struct AttnKArgs {
  const bf16_t* qkv;
  const bf16_t* pk;
  const bf16_t* pv;
  const float2* rope;   // [64][B] (cos, sin) of angle (pos0+b) * base^(-2f/128): lanes that differ in b read neighbours
  bf16_t* out;
  float* opart;         // [nS][M][Hq][128]
  float* mlpart;        // [nS][M][Hq][2]
  int M, B, Hq, Hkv, P, S, ldp, ld, nQ, nS;   // ldp = rows allocated per KV head of the cache; S = suffix rows
  int own;                                     // 0: no own-block keys (queries that only read the cache)
  int split;                                   // cached rows per split: the P + S rows shared out evenly, whole tiles
  int qrows;                                   // query rows a workgroup owns: 128, or 96 / 64 / 32 when there are few workgroups (scheduling only)
};

// the lane's 8 MFMA operand fragments of LDS tile row `row` (K layout): hd = 16*kk + 8*hh + e
__device__ __forceinline__ void load_frags(bf16x8 (&f)[8], const bf16_t* __restrict__ tile, int row, int hh) {
  const bf16_t* p = tile + row * HD;
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) f[kk] = *reinterpret_cast<const bf16x8*>(p + k_pos(row, 2 * kk + hh) * 8);
}
// rotary embedding of the fragments of global row `row` (position row % B) and scaling; fragment kk pairs with
// kk + 4 (hd and hd + 64).  `rope` is [64][B] (cos, sin).
__device__ __forceinline__ void rotate_frags(bf16x8 (&f)[8], const float2* __restrict__ rope, int B, int row, int hh, float scale) {
  const float2* rp = rope + (size_t)(hh * 8) * B + (row % B);
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    const bf16x8 x1 = f[kk], x2 = f[kk + 4];
    bf16x8 y1, y2;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float2 cs = rp[(size_t)(kk * 16 + e) * B];
      const float a1 = static_cast<float>(x1[e]), a2 = static_cast<float>(x2[e]);
      y1[e] = static_cast<bf16_t>((a1 * cs.x - a2 * cs.y) * scale);
      y2[e] = static_cast<bf16_t>((a2 * cs.x + a1 * cs.y) * scale);
    }
    f[kk] = y1;
    f[kk + 4] = y2;
  }
}

// DUAL: the cache also holds rows of the tokens after the block (a.S > 0)
template <bool DUAL>
__device__ __forceinline__ void attn_prefix_body(const AttnKArgs& a, int bid) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16_t* smem = reinterpret_cast<bf16_t*>(smem_raw);

  const int total = a.nQ * a.nS * a.Hq;
  const int L = xcd_contiguous(bid, total);
  const int qt = L % a.nQ;
  const int sp = (L / a.nQ) % a.nS;
  const int h = L / (a.nQ * a.nS);
  const int kvh = h / (a.Hq / a.Hkv);

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int l32 = lane & 31, hh = lane >> 5;
  // query group of the wavefront pair, and this wavefront's role in it: the key half it takes (role 0 also takes the
  // own-block keys and finishes the pair's rows).  Role 0 sits on wavefronts 0, 2, 5, 7, one per SIMD when wavefronts go
  // round the four SIMDs in order: the four pairs' own-block phases and final merges then do not share SIMDs two by two.
  const int qw = wave >> 1, st = (wave ^ (wave >> 2)) & 1;
  const int m0 = qt * a.qrows;
  const int m_end = min(a.M, m0 + a.qrows);     // the workgroup's query rows are m0 .. m_end-1
  const int m0w = m0 + qw * 32;
  const int qrow = min(m0w + l32, a.M - 1);
  // A wavefront pair whose 32 query rows all lie beyond M (one or two states in a 128-row tile) takes part in the
  // transfers and barriers only: the pairs that do have rows then keep their SIMDs to themselves.
  const bool active = __builtin_amdgcn_readfirstlane(m0w) < m_end;

  WaveState w;
  w.m_run = -INFINITY;
  w.l_run = 0.f;
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int v = 0; v < 16; ++v) w.o[n][v] = 0.f;

  // The cached keys form one axis of P + S rows: the prefix (cache rows 0 .. P-1), then the tokens after the
  // block (dual cache: cache rows P+B .. P+B+S-1).  Split `sp` owns a.split consecutive rows of that axis
  // and streams its prefix part, then its suffix part; [kbeg, kend) are cache rows of the part in progress.
  const int v0 = sp * a.split, v1 = min(a.P + a.S, v0 + a.split);
  int kbeg = min(v0, a.P);
  int kend = min(v1, a.P);
  int n_tiles = kend > kbeg ? (kend - kbeg + KTILE - 1) / KTILE : 0;
  const bf16_t* pk = a.pk + (size_t)kvh * a.ldp * HD;
  const bf16_t* pv = a.pv + (size_t)kvh * a.ldp * HD;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  // LDS-DMA of N_ROWS rows of 256 bytes (rows row0 .. clamped to row_max of a matrix with row stride `ld`
  // elements, starting at `src`) into an LDS tile; wavefront `wave` brings N_ROWS/8 consecutive rows:
  // lane -> (row, LDS position) -> source chunk
  auto issue_rows = [&](auto n_rows_tag, auto vswz_tag, bf16_t* dst, const bf16_t* src, int row0, int row_max, size_t ld) {
    constexpr int N_ROWS = decltype(n_rows_tag)::value;
    constexpr bool VSWZ = decltype(vswz_tag)::value;
    constexpr int PER_WAVE = N_ROWS / 8;
#pragma unroll
    for (int q = 0; q < PER_WAVE / 4; ++q) {
      const int row = PER_WAVE * wave_u + 4 * q + (lane >> 4), pos = lane & 15;
      const int chunk = VSWZ ? v_pos(row, pos) : k_pos(row, pos);
      __builtin_amdgcn_global_load_lds((glb_ptr_t)(src + (size_t)min(row0 + row, row_max) * ld + chunk * 8),
                                       (lds_ptr_t)(dst + (PER_WAVE * wave_u + 4 * q) * HD), 16, 0, 0);
    }
  };
  using R64 = std::integral_constant<int, 64>;
  using R128 = std::integral_constant<int, 128>;
  auto issue_tile = [&](int t) {     // prefix tile t of this split into its ring stage
    bf16_t* stage = smem + (t % NSTAGE) * STAGE_ELEMS;
    issue_rows(R64{}, std::false_type{}, stage, pk, kbeg + t * KTILE, kend - 1, HD);
    issue_rows(R64{}, std::true_type{}, stage + TILE_ELEMS, pv, kbeg + t * KTILE, kend - 1, HD);
  };
  // own-block rows c0 .. c0+127 (K and V columns of the fused activations) into stages 1 and 2
  const bool has_own = a.own && sp == a.nS - 1;
  const int own_lo = (m0 / a.B) * a.B;
  const int own_hi = min(a.M, ((m_end - 1) / a.B + 1) * a.B);
  auto issue_own = [&](int c0) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      bf16_t* stage = smem + (1 + i) * STAGE_ELEMS;
      issue_rows(R64{}, std::false_type{}, stage, a.qkv + (a.Hq + kvh) * HD, c0 + 64 * i, a.M - 1, a.ld);
      issue_rows(R64{}, std::true_type{}, stage + TILE_ELEMS, a.qkv + (a.Hq + a.Hkv + kvh) * HD, c0 + 64 * i, a.M - 1, a.ld);
    }
  };

  // ---- start every transfer known up front: the 128 Q rows (stage 3), the first own-block rows (stages 1, 2)
  // and prefix tile 0 (stage 0); all of them arrive as whole 256-byte rows
  issue_rows(R128{}, std::false_type{}, smem + 3 * STAGE_ELEMS, a.qkv + h * HD, m0, a.M - 1, a.ld);
  if (has_own) issue_own(own_lo);
  if (n_tiles > 0) issue_tile(0);
  wait_vmcnt<0>();
  __builtin_amdgcn_s_barrier();

  // ---- Q: fragments of the wavefront pair's rows, rotated at position pos0 + (row % B), scaled by
  // log2(e)/sqrt(128), rounded to bf16
  load_frags(w.qf, smem + 3 * STAGE_ELEMS, qw * 32 + l32, hh);
  rotate_frags(w.qf, a.rope, a.B, qrow, hh, 1.4426950408889634f * 0.08838834764831845f);

  // ---- own-block keys: the block diagonal, handled by the last split.  They always go to the role-0 wavefront
  // of the pair, 32 keys at a time in row order, so a state's arithmetic does not depend on where its rows sit
  // in the 128-row tile.  K fragments are rotated in registers on their way from LDS to the matrix pipe.
  if (has_own) {
    // rows of the states this wave's queries belong to
    const int w_lo = (min(m0w, a.M - 1) / a.B) * a.B;
    const int w_hi = (min(m0w + 31, a.M - 1) / a.B + 1) * a.B;
    const int q_lo = (qrow / a.B) * a.B;    // this lane's state: rows [q_lo, q_lo + B)
    const int q_hi = q_lo + a.B;
    for (int c0 = own_lo; c0 < own_hi; c0 += 128) {
      if (c0 != own_lo) {      // more than 128 own rows (B does not divide the tile): next chunk
        __syncthreads();
        issue_own(c0);
        wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
      }
      if (st == 0 && active) {
#pragma unroll
        for (int sub = 0; sub < 4; ++sub) {
          const int k_lo = c0 + sub * 32;
          if (k_lo < w_hi && k_lo + 32 > w_lo && k_lo < own_hi) {   // wave-uniform: this sub-tile holds keys of my states
            const bf16_t* stage = smem + (1 + (sub >> 1)) * STAGE_ELEMS;
            bf16x8 kf[8];
            load_frags(kf, stage, (sub & 1) * 32 + l32, hh);
            rotate_frags(kf, a.rope, a.B, min(k_lo + l32, a.M - 1), hh, 1.0f);
            f32x16 sc;
#pragma unroll
            for (int v = 0; v < 16; ++v) sc[v] = 0.f;
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], w.qf[kk], sc, 0, 0, 0);
            const int t0 = c0 + (sub >> 1) * 64;     // first row of the 64-row tile
            finish_tile<true>(w, sc, stage + TILE_ELEMS, sub & 1, lane, [t0, q_lo, q_hi, own_hi](int key) {
              const int row = t0 + key;
              return row >= q_lo && row < q_hi && row < own_hi;
            });
          }
        }
      }
    }
  }
  __syncthreads();   // Q and own-block stages are free again

  // ---- cached keys of this split: LDS-DMA ring, up to NSTAGE-1 tiles ahead --------------------------
#pragma nounroll
  for (int part = 0; part < (DUAL ? 2 : 1); ++part) {
  if (part == 1) {
    kbeg = max(v0, a.P) + a.B;
    kend = max(v1, a.P) + a.B;
    n_tiles = kend > kbeg ? (kend - kbeg + KTILE - 1) / KTILE : 0;
    if (n_tiles > 0) issue_tile(0);      // the ring is drained: every stage is free
  }
  if (n_tiles == 0) continue;
  if (1 < n_tiles) issue_tile(1);
  if (2 < n_tiles) issue_tile(2);
  // full tiles run through the software pipeline (scores of tile t+1 under the softmax of tile t); a ragged
  // last tile takes the masked path afterwards
  const bool ragged = n_tiles > 0 && ((kend - kbeg) % KTILE) != 0;
  const int n_pipe = ragged ? n_tiles - 1 : n_tiles;
  if (n_pipe > 0) {
    // tile 0 has landed; tiles 1 .. min(2, n_tiles-1) may still be in flight
    if (n_tiles >= 3) wait_vmcnt<2 * DMA_PER_TILE>(); else if (n_tiles == 2) wait_vmcnt<DMA_PER_TILE>(); else wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    f32x16 sa, sb;
    if (active) scores(w, sa, smem, st, lane);
    // step t: tile t+1 has landed (tile t+2 may be in flight) and every wavefront is done with step t-1,
    // i.e. with K of tile t and V of tile t-1, whose stage the next prefetch overwrites
    auto sync_and_prefetch = [&](int t) {
      if (t + 2 < n_tiles) wait_vmcnt<DMA_PER_TILE>(); else wait_vmcnt<0>();
      __builtin_amdgcn_s_barrier();
      if (t + NSTAGE - 1 < n_tiles) issue_tile(t + NSTAGE - 1);
    };
    auto k_of = [&](int t) { return smem + (t % NSTAGE) * STAGE_ELEMS; };
    auto v_of = [&](int t) { return smem + (t % NSTAGE) * STAGE_ELEMS + TILE_ELEMS; };
    int t = 0;
    for (; t + 2 < n_pipe; t += 2) {     // two steps per trip: the score registers swap roles
      sync_and_prefetch(t);
      if (active) pipe_step<true>(w, sa, sb, k_of(t + 1), v_of(t), st, lane);
      sync_and_prefetch(t + 1);
      if (active) pipe_step<true>(w, sb, sa, k_of(t + 2), v_of(t + 1), st, lane);
    }
    if (t + 1 < n_pipe) {
      sync_and_prefetch(t);
      if (active) pipe_step<true>(w, sa, sb, k_of(t + 1), v_of(t), st, lane);
      sync_and_prefetch(t + 1);
      if (active) pipe_step<false>(w, sb, sa, nullptr, v_of(t + 1), st, lane);
    } else {
      sync_and_prefetch(t);
      if (active) pipe_step<false>(w, sa, sb, nullptr, v_of(t), st, lane);
    }
  }
  if (ragged) {
    wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    const bf16_t* ks = smem + ((n_tiles - 1) % NSTAGE) * STAGE_ELEMS;
    const int nvalid = kend - (kbeg + (n_tiles - 1) * KTILE);
    if (active) process_tile<true>(w, ks, ks + TILE_ELEMS, st, lane, [nvalid](int key) { return key < nvalid; });
  }
  __syncthreads();   // all tiles consumed, no DMA in flight: the ring can be reused
  }

  // ---- merge the two key halves of each wavefront pair through LDS ------------------------------
  {
    float* xb = reinterpret_cast<float*>(smem_raw) + (size_t)qw * 66 * 64;   // [66][64 lanes] per pair
    if (st == 1) {
#pragma unroll
      for (int n = 0; n < 4; ++n)
#pragma unroll
        for (int v = 0; v < 16; ++v) xb[(n * 16 + v) * 64 + lane] = w.o[n][v];
      xb[64 * 64 + lane] = w.m_run;
      xb[65 * 64 + lane] = w.l_run;
    }
    __syncthreads();
    if (st == 1) return;
    const float m1 = xb[64 * 64 + lane], l1 = xb[65 * 64 + lane];
    const float mm = fmaxf(w.m_run, m1);
    const float a0 = (w.m_run == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(w.m_run - mm);
    const float a1 = (m1 == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m1 - mm);
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
      for (int v = 0; v < 16; ++v) w.o[n][v] = w.o[n][v] * a0 + xb[(n * 16 + v) * 64 + lane] * a1;
    w.l_run = w.l_run * a0 + l1 * a1;
    w.m_run = mm;
  }

  // ---- write ----------------------------------------------------------------------------------
  const float l_tot = w.l_run + __shfl_xor(w.l_run, 32, 64);
  if (m0w + l32 >= m_end) return;
  if (a.nS == 1) {
    const float inv = 1.0f / l_tot;
    bf16_t* op = a.out + (size_t)qrow * (a.Hq * HD) + h * HD + 4 * hh;
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        bf16x4 t;
#pragma unroll
        for (int e = 0; e < 4; ++e) t[e] = static_cast<bf16_t>(w.o[n][g4 * 4 + e] * inv);
        *reinterpret_cast<bf16x4*>(op + n * 32 + g4 * 8) = t;
      }
  } else {
    const size_t rowh = ((size_t)sp * a.M + qrow) * a.Hq + h;
    float* op = a.opart + rowh * HD + 4 * hh;
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        f32x4 t;
#pragma unroll
        for (int e = 0; e < 4; ++e) t[e] = w.o[n][g4 * 4 + e];
        *reinterpret_cast<f32x4*>(op + n * 32 + g4 * 8) = t;
      }
    if (hh == 0) {
      a.mlpart[rowh * 2] = w.m_run;
      a.mlpart[rowh * 2 + 1] = l_tot;
    }
  }
}

template <bool DUAL>
__global__ __launch_bounds__(NT) void attn_prefix_mfma_kernel(AttnKArgs a) {
  attn_prefix_body<DUAL>(a, (int)blockIdx.x);
}

// Two independent attention problems in one launch (the G states and, beside them, the rows that ride along with a
// step: the recomputed suffix, or the block being committed): the first n_a workgroups take `a`, the rest `b`.
// Each part alone would leave most CUs idle when there are few states.
__global__ __launch_bounds__(NT) void attn_prefix_mfma_pair_kernel(AttnKArgs a, AttnKArgs b, int n_a) {
  if ((int)blockIdx.x < n_a) attn_prefix_body<true>(a, (int)blockIdx.x);
  else attn_prefix_body<true>(b, (int)blockIdx.x - n_a);
}

// merge the prefix splits of each (row, head): weights 2^(m_s - max m).  32 lanes per (row, head), four head
// dimensions per lane, eight (row, head) pairs per workgroup.
__global__ __launch_bounds__(256) void attn_combine_kernel(const float* __restrict__ opart,
                                                           const float* __restrict__ mlpart, bf16_t* __restrict__ out,
                                                           int M, int Hq, int nS) {
  const size_t n_rowh = (size_t)M * Hq;
  const size_t rowh = (size_t)blockIdx.x * 8 + (threadIdx.x >> 5);   // row * Hq + head
  if (rowh >= n_rowh) return;
  const int t = (threadIdx.x & 31) * 4;
  float mx = -INFINITY;
  for (int s = 0; s < nS; ++s) mx = fmaxf(mx, mlpart[((size_t)s * n_rowh + rowh) * 2]);
  f32x4 num = {0.f, 0.f, 0.f, 0.f};
  float den = 0.f;
  for (int s = 0; s < nS; ++s) {
    const size_t i = (size_t)s * n_rowh + rowh;
    const float ms = mlpart[i * 2];
    const float wgt = (ms == -INFINITY) ? 0.f : exp2f(ms - mx);
    den += wgt * mlpart[i * 2 + 1];
    const f32x4 o = *reinterpret_cast<const f32x4*>(opart + i * HD + t);
#pragma unroll
    for (int e = 0; e < 4; ++e) num[e] += wgt * o[e];
  }
  bf16x4 r;
#pragma unroll
  for (int e = 0; e < 4; ++e) r[e] = static_cast<bf16_t>(num[e] / den);
  *reinterpret_cast<bf16x4*>(out + rowh * HD + t) = r;
}

__global__ void rope_table_kernel(float2* __restrict__ tab, int B, int half, int hd, int pos0, float base) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= B * half) return;
  const int f = i / B, b = i % B;      // tab[f][b]
  const double inv_freq = pow((double)base, -2.0 * (double)f / (double)hd);
  const double ang = (double)(pos0 + b) * inv_freq;
  tab[i] = make_float2((float)cos(ang), (float)sin(ang));
}

inline int n_splits(int P) { return P > 0 ? cdiv(P, SPLIT_KEYS) : 1; }

}  // namespace

bool mfma_attn_supported(const AttnArgs& a) {
  return a.hd == HD && a.Hq % a.Hkv == 0 && a.B >= 1 && a.G >= 1;
}

// rope table + split partials; P = cached keys, prefix and suffix together
size_t mfma_attn_partial_bytes(int G, int B, int Hq, int hd, int P) {
  const size_t M = (size_t)G * B;
  size_t bytes = align_up(sizeof(float2) * (size_t)B * (hd / 2), 256);
  const int nS = n_splits(P);
  if (nS > 1) {
    bytes += align_up(sizeof(float) * nS * M * Hq * hd, 256);
    bytes += align_up(sizeof(float) * nS * M * Hq * 2, 256);
  }
  return bytes;
}

// The rotary table of an attention problem with B rows per state at positions pos0 ..: [hd/2][B] (cos, sin), at the start
// of that problem's scratch.  Callers that need it before the attention launch (the cache append) build it here and
// pass rope_ready = 1 to the attention launch.
const void* launch_rope_table(void* partial, int B, int pos0, float rope_base, hipStream_t st) {
  const int nrope = B * (HD / 2);
  rope_table_kernel<<<cdiv(nrope, 256), 256, 0, st>>>(reinterpret_cast<float2*>(partial), B, HD / 2, HD, pos0, rope_base);
  return partial;
}

namespace {

// kernel arguments of one attention problem; launches the rotary table kernel when the table is not in place yet
AttnKArgs prepare_attn(const AttnArgs& a, hipStream_t st) {
  const int M = a.G * a.B;
  const int nS = n_splits(a.P + a.S);
  unsigned char* ws = reinterpret_cast<unsigned char*>(a.partial);
  float2* rope = reinterpret_cast<float2*>(ws);
  ws += align_up(sizeof(float2) * (size_t)a.B * (HD / 2), 256);
  float* opart = reinterpret_cast<float*>(ws);
  ws += align_up(sizeof(float) * (size_t)nS * M * a.Hq * HD, 256);
  float* mlpart = reinterpret_cast<float*>(ws);

  const int nrope = a.B * (HD / 2);
  if (!a.rope_ready) rope_table_kernel<<<cdiv(nrope, 256), 256, 0, st>>>(rope, a.B, HD / 2, HD, a.pos0, a.rope_base);

  AttnKArgs k;
  k.qkv = (const bf16_t*)a.qkv;
  k.pk = (const bf16_t*)a.prefix_k;
  k.pv = (const bf16_t*)a.prefix_v;
  k.rope = rope;
  k.out = (bf16_t*)a.out;
  k.opart = opart;
  k.mlpart = mlpart;
  k.M = M; k.B = a.B; k.Hq = a.Hq; k.Hkv = a.Hkv; k.P = a.P; k.S = a.S; k.ldp = a.ldp ? a.ldp : a.P;
  k.own = a.own;
  k.ld = (a.Hq + 2 * a.Hkv) * HD;
  // With few workgroups (one to eight states) a workgroup takes 64 or 32 query rows instead of 128, so that more CUs
  // stream the keys; the wavefront pairs without rows only move data.  A row's arithmetic is the same (own-block keys
  // are visited in 32-row groups counted from a multiple of 32 either way) as long as B divides 32 or 32 divides B,
  // and always when there are no own-block keys.
  k.qrows = QTILE;
  if (!a.own || 32 % a.B == 0 || a.B % 32 == 0) {
    const int wgs = cdiv(M, QTILE) * nS * a.Hq;
    if (wgs <= 64) k.qrows = 32;
    else if (wgs <= 128) k.qrows = 64;
    // between half and the whole chip (28 heads x 6 tiles of 128 rows = 168 workgroups): 96 rows, three of the four
    // wavefront pairs at work, if that brings more workgroups and still one round of them (28 x 8 = 224)
    else if (wgs < 256 && cdiv(M, 96) > cdiv(M, QTILE) && cdiv(M, 96) * nS * a.Hq <= 256) k.qrows = 96;
  }
  k.nQ = cdiv(M, k.qrows);
  k.nS = nS;
  k.split = (int)align_up(cdiv(a.P + a.S, nS), KTILE);      // at most SPLIT_KEYS; a function of P + S only
  return k;
}

hipError_t attn_lds_limits() {
  static std::atomic<unsigned long long> lds_ok[3];
  hipError_t e = allow_dynamic_lds((const void*)attn_prefix_mfma_kernel<false>, (int)kAttnSmem, lds_ok[0]);
  if (e != hipSuccess) return e;
  e = allow_dynamic_lds((const void*)attn_prefix_mfma_kernel<true>, (int)kAttnSmem, lds_ok[1]);
  if (e != hipSuccess) return e;
  return allow_dynamic_lds((const void*)attn_prefix_mfma_pair_kernel, (int)kAttnSmem, lds_ok[2]);
}

}  // namespace

hipError_t launch_attn_mfma(const AttnArgs& a, hipStream_t st) {
  const hipError_t e = attn_lds_limits();
  if (e != hipSuccess) return e;
  const AttnKArgs k = prepare_attn(a, st);
  const int grid = k.nQ * k.nS * a.Hq;
  if (a.S > 0) attn_prefix_mfma_kernel<true><<<grid, NT, kAttnSmem, st>>>(k);
  else attn_prefix_mfma_kernel<false><<<grid, NT, kAttnSmem, st>>>(k);
  if (k.nS > 1) attn_combine_kernel<<<cdiv(k.M * a.Hq, 8), 256, 0, st>>>(k.opart, k.mlpart, k.out, k.M, a.Hq, k.nS);
  return hipGetLastError();
}

// two independent problems (different query rows, outputs and scratch; they may read the same cache) in one launch
hipError_t launch_attn_mfma_pair(const AttnArgs& a, const AttnArgs& b, hipStream_t st) {
  const hipError_t e = attn_lds_limits();
  if (e != hipSuccess) return e;
  const AttnKArgs ka = prepare_attn(a, st), kb = prepare_attn(b, st);
  const int n_a = ka.nQ * ka.nS * a.Hq, n_b = kb.nQ * kb.nS * b.Hq;
  attn_prefix_mfma_pair_kernel<<<n_a + n_b, NT, kAttnSmem, st>>>(ka, kb, n_a);
  if (ka.nS > 1) attn_combine_kernel<<<cdiv(ka.M * a.Hq, 8), 256, 0, st>>>(ka.opart, ka.mlpart, ka.out, ka.M, a.Hq, ka.nS);
  if (kb.nS > 1) attn_combine_kernel<<<cdiv(kb.M * b.Hq, 8), 256, 0, st>>>(kb.opart, kb.mlpart, kb.out, kb.M, b.Hq, kb.nS);
  return hipGetLastError();
}

}  // namespace spiffy

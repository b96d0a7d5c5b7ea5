// bf16 MFMA GEMM for gfx950:  D[i,j] = sum_k X[i,k] * Y[j,k]  (both operands K-contiguous),
// fp32 accumulation with v_mfma_f32_32x32x16_bf16, 128x128x64 workgroup tile, 4 wavefronts of
// 64x64, double-buffered LDS fed through registers, XCD-aware tile order.
//
// One kernel template, four epilogues:
//   EPI_STORE   C = X W^T (+bias)         W given as up to three [N_i,K] segments (q | k | v)
//   EPI_RESID   C = R + X W^T             (output projection, FFN down projection)
//   EPI_SWIGLU  C = silu(X Wg^T) * (X Wu^T)   the tile's 128 "columns" are 64 gate + 64 up rows
//   EPI_LMHEAD  rows i = vocabulary entries, columns j = tokens: each lane owns a token column
//               and reduces its logits to (top, lowest index, runner-up, sum exp) in registers;
//               logits are never stored (Alg. 1 steps 1-2 fused into the GEMM).
//
// Accumulation order along K is the same for every output element whatever M, N or the tile
// position, so a row's result does not depend on how many other states are verified with it.
#include "kernels.h"

namespace spiffy {

namespace {

constexpr int BM = 128, BN = 128, BK = 64;
constexpr int LDS_STRIDE = BK + 8;  // bf16 elements per LDS row: 144 B keeps 16-byte fragment reads conflict-free
constexpr int TILE_ELEMS = 128 * LDS_STRIDE;

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
struct Frag4 {
  u32x4 v[4];
};

// 128 rows x 64 k of a K-contiguous matrix -> registers (4 x 16 B per thread)
__device__ __forceinline__ void load_tile(Frag4& f, const bf16_t* __restrict__ base, int ld, int row0, int row_max,
                                          int k0) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = threadIdx.x + 256 * i;
    int row = row0 + (c >> 3);
    row = row < row_max ? row : row_max - 1;
    f.v[i] = *reinterpret_cast<const u32x4*>(base + (size_t)row * ld + k0 + (c & 7) * 8);
  }
}
// SwiGLU operand tile: rows 0..63 from the gate matrix, rows 64..127 from the up matrix
__device__ __forceinline__ void load_tile_pair(Frag4& f, const bf16_t* __restrict__ g, const bf16_t* __restrict__ u,
                                               int ld, int row0, int k0) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = threadIdx.x + 256 * i;
    const int r = c >> 3;
    const bf16_t* base = r < 64 ? g : u;
    f.v[i] = *reinterpret_cast<const u32x4*>(base + (size_t)(row0 + (r & 63)) * ld + k0 + (c & 7) * 8);
  }
}
__device__ __forceinline__ void store_tile(const Frag4& f, bf16_t* lds) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = threadIdx.x + 256 * i;
    *reinterpret_cast<u32x4*>(lds + (c >> 3) * LDS_STRIDE + (c & 7) * 8) = f.v[i];
  }
}

template <int EPI>
__global__ __launch_bounds__(256) void gemm_bf16_mfma_kernel(GemmArgs a, int tiles_i, int tiles_j) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16_t* Xs = reinterpret_cast<bf16_t*>(smem_raw);  // [2][128][LDS_STRIDE]
  bf16_t* Ys = Xs + 2 * TILE_ELEMS;                  // [2][128][LDS_STRIDE]

  // XCD-aware order: workgroup ids go round-robin over the 8 XCDs, so give each XCD a contiguous
  // range of logical tiles; the logical order runs fastest over the activation tiles, which keeps
  // all workgroups that stream the same weight tile on one XCD (one L2) and close in time.
  const int total = tiles_i * tiles_j;
  int L = blockIdx.x;
  if ((total & 7) == 0) L = (blockIdx.x >> 3) + (blockIdx.x & 7) * (total >> 3);
  const int ti = (EPI == EPI_LMHEAD) ? L / tiles_j : L % tiles_i;
  const int tj = (EPI == EPI_LMHEAD) ? L % tiles_j : L / tiles_i;
  const int i0 = ti * BM, j0 = tj * BN;

  // operand roles
  const bf16_t* X;      // rows i
  int ldx, i_max;
  const bf16_t* Y = nullptr;  // rows j
  const bf16_t* Y2 = nullptr;
  int ldy, j_max, jrow0;
  const bf16_t* bias = nullptr;
  if (EPI == EPI_LMHEAD) {
    X = (const bf16_t*)a.W[0]; ldx = a.K; i_max = a.N;          // vocabulary rows
    Y = (const bf16_t*)a.A; ldy = a.lda; jrow0 = j0;            // token rows
    j_max = a.M_dev ? min(*a.M_dev, a.M) : a.M;
    if (j0 >= j_max) return;
  } else {
    X = (const bf16_t*)a.A; ldx = a.lda;
    i_max = a.M_dev ? min(*a.M_dev, a.M) : a.M;
    if (i0 >= i_max) return;
    ldy = a.K;
    if (EPI == EPI_SWIGLU) {
      Y = (const bf16_t*)a.W[0]; Y2 = (const bf16_t*)a.W[1]; jrow0 = tj * 64; j_max = a.N;
    } else {
      // segment of this column tile (no runtime indexing of the argument block: that would spill it)
      if (j0 < a.Nseg[0]) {
        Y = (const bf16_t*)a.W[0]; jrow0 = j0; j_max = a.Nseg[0]; bias = (const bf16_t*)a.bias[0];
      } else if (j0 < a.Nseg[0] + a.Nseg[1]) {
        Y = (const bf16_t*)a.W[1]; jrow0 = j0 - a.Nseg[0]; j_max = a.Nseg[1]; bias = (const bf16_t*)a.bias[1];
      } else {
        Y = (const bf16_t*)a.W[2]; jrow0 = j0 - a.Nseg[0] - a.Nseg[1]; j_max = a.Nseg[2];
        bias = (const bf16_t*)a.bias[2];
      }
      if (bias) bias += jrow0;
    }
  }

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wi = wave >> 1, wj = wave & 1;
  const int l32 = lane & 31, hh = lane >> 5;

  f32x16 acc[2][2];
#pragma unroll
  for (int p = 0; p < 2; ++p)
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[p][q][v] = 0.f;

  const int KT = a.K / BK;
  Frag4 fx, fy;
  load_tile(fx, X, ldx, i0, i_max, 0);
  if (EPI == EPI_SWIGLU) load_tile_pair(fy, Y, Y2, ldy, jrow0, 0); else load_tile(fy, Y, ldy, jrow0, j_max, 0);
  store_tile(fx, Xs);
  store_tile(fy, Ys);
  __syncthreads();

  for (int kt = 0; kt < KT; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < KT) {
      load_tile(fx, X, ldx, i0, i_max, (kt + 1) * BK);
      if (EPI == EPI_SWIGLU) load_tile_pair(fy, Y, Y2, ldy, jrow0, (kt + 1) * BK);
      else load_tile(fy, Y, ldy, jrow0, j_max, (kt + 1) * BK);
    }
    const bf16_t* xs = Xs + cur * TILE_ELEMS + (wi * 64 + l32) * LDS_STRIDE + hh * 8;
    // wave wj owns j-columns {wj*32 + 0..31} and {64 + wj*32 + 0..31}: column c and c+64 of the tile
    // sit in the same lane (gate/up pairing for SwiGLU)
    const bf16_t* ys = Ys + cur * TILE_ELEMS + (wj * 32 + l32) * LDS_STRIDE + hh * 8;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 xa[2], yb[2];
#pragma unroll
      for (int p = 0; p < 2; ++p) xa[p] = *reinterpret_cast<const bf16x8*>(xs + p * 32 * LDS_STRIDE + kk * 16);
#pragma unroll
      for (int q = 0; q < 2; ++q) yb[q] = *reinterpret_cast<const bf16x8*>(ys + q * 64 * LDS_STRIDE + kk * 16);
#pragma unroll
      for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int q = 0; q < 2; ++q)
          acc[p][q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa[p], yb[q], acc[p][q], 0, 0, 0);
    }
    if (kt + 1 < KT) {
      store_tile(fx, Xs + (cur ^ 1) * TILE_ELEMS);
      store_tile(fy, Ys + (cur ^ 1) * TILE_ELEMS);
    }
    __syncthreads();
  }

  // accumulator element (p,q,v) of this lane: i = i0 + wi*64 + p*32 + 8*(v/4) + 4*hh + v%4,
  //                                           j-column (within the 128 of the tile) = q*64 + wj*32 + l32
  if (EPI == EPI_LMHEAD) {
    // lane owns token columns j(q); reduce over its 32 vocabulary rows per column
    TopPartial* part = reinterpret_cast<TopPartial*>(a.C);
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const int tokr = j0 + q * 64 + wj * 32 + l32;
      Top t = top_empty();
      float mx = -INFINITY;
#pragma unroll
      for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          acc[p][q][v] *= a.scale;
          mx = fmaxf(mx, acc[p][q][v]);
        }
      // (top, lowest index, runner-up) in one ordered pass, sum of exp against the lane's own top
      float s = 0.f;
#pragma unroll
      for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float l = acc[p][q][v];
          const int idx = i0 + wi * 64 + p * 32 + 8 * (v >> 2) + 4 * hh + (v & 3);
          if (l > t.m || (l == t.m && idx < t.idx)) { t.m2 = t.m; t.m = l; t.idx = idx; }
          else t.m2 = fmaxf(t.m2, l);
          s += __expf(l - mx);
        }
      t.s = s;
      t = top_merge(t, top_shfl_xor(t, 32));
      if (hh == 0 && tokr < j_max) part[(size_t)(ti * 2 + wi) * a.ldc + tokr] = TopPartial{t.m, t.m2, t.s, t.idx};
    }
    return;
  }

  bf16_t* C = reinterpret_cast<bf16_t*>(a.C);
  const bf16_t* R = reinterpret_cast<const bf16_t*>(a.R);
#pragma unroll
  for (int p = 0; p < 2; ++p)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int i = i0 + wi * 64 + p * 32 + 8 * (v >> 2) + 4 * hh + (v & 3);
      if (i >= i_max) continue;
      if (EPI == EPI_SWIGLU) {
        const float g = acc[p][0][v], u = acc[p][1][v];
        const int f = tj * 64 + wj * 32 + l32;
        C[(size_t)i * a.ldc + f] = static_cast<bf16_t>(g / (1.f + __expf(-g)) * u);
      } else {
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          const int jc = q * 64 + wj * 32 + l32;
          float val = acc[p][q][v];
          if (EPI == EPI_STORE && bias) val += static_cast<float>(bias[jc]);
          const size_t o = (size_t)i * a.ldc + j0 + jc;
          if (EPI == EPI_RESID) val += static_cast<float>(R[o]);
          C[o] = static_cast<bf16_t>(val);
        }
      }
    }
}

constexpr size_t kSmemBytes = sizeof(bf16_t) * 4 * TILE_ELEMS;  // 73,728 B

template <int EPI>
hipError_t launch_t(const GemmArgs& a, int tiles_i, int tiles_j, hipStream_t st) {
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)gemm_bf16_mfma_kernel<EPI>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)kSmemBytes);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  gemm_bf16_mfma_kernel<EPI><<<tiles_i * tiles_j, 256, kSmemBytes, st>>>(a, tiles_i, tiles_j);
  return hipGetLastError();
}

}  // namespace

bool mfma_gemm_supported(int epi, const GemmArgs& a) {
  if (a.K % BK != 0 || a.K < BK || a.M < 1) return false;
  if (epi == EPI_SWIGLU) return a.N % 64 == 0;
  if (epi == EPI_LMHEAD) return a.N % BM == 0;
  int n = 0;
  for (int s = 0; s < 3; ++s) {
    if (a.Nseg[s] < 0 || a.Nseg[s] % BN != 0) return false;
    n += a.Nseg[s];
  }
  return n == a.N && a.Nseg[0] > 0;
}

int mfma_lmhead_partials_per_row(int V) { return V / BM * 2; }

hipError_t launch_gemm_mfma(int epi, const GemmArgs& a, hipStream_t st) {
  switch (epi) {
    case EPI_STORE: return launch_t<EPI_STORE>(a, cdiv(a.M, BM), a.N / BN, st);
    case EPI_RESID: return launch_t<EPI_RESID>(a, cdiv(a.M, BM), a.N / BN, st);
    case EPI_SWIGLU: return launch_t<EPI_SWIGLU>(a, cdiv(a.M, BM), a.N / 64, st);
    case EPI_LMHEAD: return launch_t<EPI_LMHEAD>(a, a.N / BM, cdiv(a.M, BN), st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace spiffy

// Shared device/host helpers for the gfx950 kernels (no entry points here).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "../../include/spiffy.h"

namespace spiffy {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kWave = 64;

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return static_cast<float>(x); }
template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float x) { return static_cast<bf16_t>(x); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// Running summary of a set of logits: top value, its lowest index, runner-up value and
// sum of exp(l - top).  Merging two summaries is exact for (top, index) and stable for the sum.
struct Top {
  float m;   // top logit (-inf when empty)
  float m2;  // second logit (-inf when fewer than two)
  float s;   // sum exp(l - m)
  int idx;   // lowest index attaining m
};
__device__ __forceinline__ Top top_empty() { return Top{-INFINITY, -INFINITY, 0.f, 0x7fffffff}; }
__device__ __forceinline__ Top top_merge(const Top& a, const Top& b) {
  Top r;
  if (a.m > b.m || (a.m == b.m && a.idx <= b.idx)) {
    r.m = a.m; r.idx = a.idx; r.m2 = fmaxf(a.m2, b.m);
  } else {
    r.m = b.m; r.idx = b.idx; r.m2 = fmaxf(b.m2, a.m);
  }
  float sa = (a.m == -INFINITY) ? 0.f : a.s * __expf(a.m - r.m);
  float sb = (b.m == -INFINITY) ? 0.f : b.s * __expf(b.m - r.m);
  r.s = sa + sb;
  return r;
}
__device__ __forceinline__ Top top_push(const Top& a, float l, int idx) {
  Top b{l, -INFINITY, 1.f, idx};
  return top_merge(a, b);
}
__device__ __forceinline__ Top top_shfl_xor(const Top& a, int o) {
  Top b;
  b.m = __shfl_xor(a.m, o, 64);
  b.m2 = __shfl_xor(a.m2, o, 64);
  b.s = __shfl_xor(a.s, o, 64);
  b.idx = __shfl_xor(a.idx, o, 64);
  return b;
}

// Per-row partial written by the LM-head kernels and merged by the combine kernel.
struct alignas(16) TopPartial {
  float m, m2, s;
  int idx;
};

// ---------------------------------------------------------------------------------------------
// launch parameter blocks (plain structs passed by value)
// ---------------------------------------------------------------------------------------------

// C[M,N] = A[M,K] * W^T where W is given as up to three row-major [N_i,K] segments laid side by
// side along N (q | k | v), or as a (gate, up) pair for the SwiGLU epilogue.
enum GemmEpi { EPI_STORE = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_LMHEAD = 3, EPI_PARTIAL = 4 };

struct GemmArgs {
  const void* A;        // [M,K]
  const void* W[3];     // segments, each [Nseg[i],K]; SWIGLU: W[0]=gate, W[1]=up, each [N,K]
  const void* bias[3];  // optional per-segment bias (fp32 math), NULL = none
  int Nseg[3];
  void* C;              // [M,N] (STORE/RESID/SWIGLU); LMHEAD: TopPartial [M, n_tiles_total]
  const void* R;        // residual [M,N] for EPI_RESID
  const int* M_dev;     // optional device row count (rows >= *M_dev are skipped), NULL = use M
  int M, N, K;
  int lda, ldc;
  int ldw;              // row stride of the weight segments in elements (0 = K, i.e. dense rows)
  float scale;          // LMHEAD: logit scale
  int ksplit;           // PARTIAL: number of K slices (C = fp32 [ksplit][Mz][N]); otherwise 1
  int Mz;               // PARTIAL: rows per K slice of C when only some of them are computed by this launch (0 = M)
};

// Workgroup ids are handed to the 8 XCDs round-robin (id % 8).  Map id -> logical index so that every
// XCD owns one contiguous range of logical indices (XCD x owns ids x, x+8, ...), for any total.
__device__ __forceinline__ int xcd_contiguous(int id, int total) {
  const int x = id & 7, j = id >> 3;
  const int q = total >> 3, r = total & 7;
  return x * q + (x < r ? x : r) + j;
}

inline int cdiv(int a, int b) { return (a + b - 1) / b; }

// Raise a kernel's dynamic LDS limit once per device: `done` holds one bit per device id.  Safe from several host
// threads (setting the attribute twice is harmless).
inline hipError_t allow_dynamic_lds(const void* kernel, int bytes, std::atomic<unsigned long long>& done) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const unsigned long long bit = 1ull << (dev & 63);
  if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
  return e;
}
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

}  // namespace spiffy

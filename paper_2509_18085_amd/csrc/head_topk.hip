// Drafting source (Sec. 4.4.2): the K most likely tokens of the accepted node's distribution at every
// masked position of its block, with their probabilities (vocabulary ranks j = 1..K).
//
// The LM head pass of the step has already reduced every masked row to (top logit, its token, sum of
// exponentials) and, on the MFMA path, left one such summary per 128-token chunk of the vocabulary.  The K
// best tokens of a row lie in the K chunks with the largest chunk maxima (a token outside them is beaten by
// the K maxima; equal logits go to the lower token id and chunks are contiguous id ranges), so only those
// K x 128 logits are recomputed - 1/250 of a second pass over the vocabulary matrix at V = 126k:
//   topk_refine_kernel   workgroup (position b, k): picks the k-th best chunk of the row, recomputes its 128
//                        logits (one wavefront per vocabulary row), keeps the chunk's K best
//   topk_full_kernel     path without chunk summaries (fp32 / shapes the MFMA head does not take): one
//                        workgroup per position scans the whole vocabulary
//   topk_merge_kernel    one wavefront per position: K best of the K x K candidates, probabilities from the
//                        row's (top logit, sum of exponentials); the row's argmax stays first with exactly the
//                        confidence the head reported
#include "kernels.h"

namespace spiffy {

namespace {

constexpr int KMAX = SPIFFY_MAX_TOPK;

// compacted row of flattened position f, or -1 (row_idx is ascending)
__device__ __forceinline__ int find_row(const int32_t* __restrict__ row_idx, int n, int f) {
  int lo = 0, hi = n;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (row_idx[mid] < f) lo = mid + 1; else hi = mid;
  }
  return (lo < n && row_idx[lo] == f) ? lo : -1;
}

// (value, index) ordering of the drafting source: larger value first, equal values to the lower index
__device__ __forceinline__ bool better(float v, int i, float v2, int i2) { return v > v2 || (v == v2 && i < i2); }

// best (value, index) over the wavefront
__device__ __forceinline__ void wave_best(float& v, int& i) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float v2 = __shfl_xor(v, o, 64);
    const int i2 = __shfl_xor(i, o, 64);
    if (better(v2, i2, v, i)) { v = v2; i = i2; }
  }
}

template <typename T>
__device__ __forceinline__ float dot_row(const T* __restrict__ x, const T* __restrict__ w, int d, int lane);
template <>
__device__ __forceinline__ float dot_row<bf16_t>(const bf16_t* __restrict__ x, const bf16_t* __restrict__ w, int d, int lane) {
  float acc = 0.f;
  for (int e = lane * 8; e < d; e += 512) {        // d % 8 == 0 on this path
    const bf16x8 a = *reinterpret_cast<const bf16x8*>(x + e);
    const bf16x8 b = *reinterpret_cast<const bf16x8*>(w + e);
#pragma unroll
    for (int t = 0; t < 8; ++t) acc = fmaf(static_cast<float>(a[t]), static_cast<float>(b[t]), acc);
  }
  return wave_sum(acc);
}
template <>
__device__ __forceinline__ float dot_row<float>(const float* __restrict__ x, const float* __restrict__ w, int d, int lane) {
  float acc = 0.f;
  for (int e = lane; e < d; e += 64) acc = fmaf(x[e], w[e], acc);
  return wave_sum(acc);
}

// dot products of x with four consecutive rows of w (row stride d): the same per-lane order and wavefront sum as dot_row
template <typename T>
__device__ __forceinline__ void dot_rows4(const T* __restrict__ x, const T* __restrict__ w, int d, int lane, float (&out)[4]);
template <>
__device__ __forceinline__ void dot_rows4<bf16_t>(const bf16_t* __restrict__ x, const bf16_t* __restrict__ w, int d, int lane,
                                                  float (&out)[4]) {
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int e = lane * 8; e < d; e += 512) {
    const bf16x8 a = *reinterpret_cast<const bf16x8*>(x + e);
    bf16x8 b[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) b[u] = *reinterpret_cast<const bf16x8*>(w + (size_t)u * d + e);
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int t = 0; t < 8; ++t) acc[u] = fmaf(static_cast<float>(a[t]), static_cast<float>(b[u][t]), acc[u]);
  }
#pragma unroll
  for (int u = 0; u < 4; ++u) out[u] = wave_sum(acc[u]);
}
template <>
__device__ __forceinline__ void dot_rows4<float>(const float* __restrict__ x, const float* __restrict__ w, int d, int lane,
                                                 float (&out)[4]) {
#pragma unroll
  for (int u = 0; u < 4; ++u) out[u] = dot_row<float>(x, w + (size_t)u * d, d, lane);
}

template <typename T>
__global__ __launch_bounds__(256) void topk_refine_kernel(HeadTopkArgs a) {
  __shared__ float s_val[4];
  __shared__ int s_idx[4];
  __shared__ float s_logit[128];
  __shared__ int s_chunk;
  const int b = blockIdx.x, k = blockIdx.y;
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int node = a.result ? a.result->node : a.node;
  float* cv = a.cand_val + ((size_t)b * KMAX + k) * KMAX;
  int32_t* ci = a.cand_idx + ((size_t)b * KMAX + k) * KMAX;
  const int r = (node >= 0 && node < a.G) ? find_row(a.row_idx, min(*a.count, a.G * a.B), node * a.B + b) : -1;
  if (r < 0) {
    if (tid < a.K) { cv[tid] = -INFINITY; ci[tid] = -1; }
    return;
  }
  // ---- the k-th best chunk of the row: k+1 rounds of a workgroup-wide best, each excluding the winners so far
  float mine[8];
  const int per = (a.n_part + 255) / 256;          // <= 8 (n_part <= 2048)
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    const int p = tid + 256 * q;
    mine[q] = (q < per && p < a.n_part) ? a.part[(size_t)p * a.m_cap + r].m : -INFINITY;
  }
  int chunk = -1;
  for (int round = 0; round <= k; ++round) {
    float v = -INFINITY;
    int i = 0x7fffffff;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int p = tid + 256 * q;
      if (better(mine[q], p, v, i)) { v = mine[q]; i = p; }
    }
    wave_best(v, i);
    if (lane == 0) { s_val[w] = v; s_idx[w] = i; }
    __syncthreads();
    if (tid == 0) {
      float bv = s_val[0];
      int bi = s_idx[0];
      for (int x = 1; x < 4; ++x)
        if (better(s_val[x], s_idx[x], bv, bi)) { bv = s_val[x]; bi = s_idx[x]; }
      s_chunk = (bv == -INFINITY) ? -1 : bi;
    }
    __syncthreads();
    chunk = s_chunk;
    if (chunk < 0) break;
#pragma unroll
    for (int q = 0; q < 8; ++q)
      if (tid + 256 * q == chunk) mine[q] = -INFINITY;
    __syncthreads();
  }
  if (chunk < 0) {                                  // fewer than k+1 chunks hold anything
    if (tid < a.K) { cv[tid] = -INFINITY; ci[tid] = -1; }
    return;
  }
  // ---- its 128 logits: wavefront w takes vocabulary rows v0 + 32w .. v0 + 32w + 31
  const int v0 = chunk * 128;
  const T* x = reinterpret_cast<const T*>(a.nf) + (size_t)r * a.d;
  // four vocabulary rows at a time, so that their loads are in flight together (every row keeps its own accumulation
  // order: the logits are those of one row after the other)
  for (int i = 0; i < 32; i += 4) {
    float l[4];
    if (v0 + w * 32 + i + 3 < a.V) {
      dot_rows4<T>(x, reinterpret_cast<const T*>(a.w_vocab) + (size_t)(v0 + w * 32 + i) * a.d, a.d, lane, l);
#pragma unroll
      for (int u = 0; u < 4; ++u) l[u] *= a.scale;
    } else {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int v = v0 + w * 32 + i + u;
        l[u] = -INFINITY;
        if (v < a.V) l[u] = dot_row<T>(x, reinterpret_cast<const T*>(a.w_vocab) + (size_t)v * a.d, a.d, lane) * a.scale;
      }
    }
    if (lane == 0) {
#pragma unroll
      for (int u = 0; u < 4; ++u) s_logit[w * 32 + i + u] = l[u];
    }
  }
  __syncthreads();
  // ---- the chunk's K best
  if (w == 0) {
    float c0 = s_logit[lane], c1 = s_logit[lane + 64];
    for (int j = 0; j < a.K; ++j) {
      float v = c0;
      int i = v0 + lane;
      if (better(c1, v0 + lane + 64, v, i)) { v = c1; i = v0 + lane + 64; }
      wave_best(v, i);
      if (lane == 0) { cv[j] = v; ci[j] = (v == -INFINITY) ? -1 : i; }
      if (i == v0 + lane) c0 = -INFINITY;
      if (i == v0 + lane + 64) c1 = -INFINITY;
    }
  }
}

// one workgroup per position, whole vocabulary; candidates go to slot k = 0
template <typename T>
__global__ __launch_bounds__(256) void topk_full_kernel(HeadTopkArgs a) {
  __shared__ float s_v[4][KMAX];
  __shared__ int s_i[4][KMAX];
  const int b = blockIdx.x;
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int node = a.result ? a.result->node : a.node;
  float* cv = a.cand_val + (size_t)b * KMAX * KMAX;
  int32_t* ci = a.cand_idx + (size_t)b * KMAX * KMAX;
  for (int e = tid; e < KMAX * KMAX; e += 256) { cv[e] = -INFINITY; ci[e] = -1; }
  const int r = (node >= 0 && node < a.G) ? find_row(a.row_idx, min(*a.count, a.G * a.B), node * a.B + b) : -1;
  if (r < 0) return;
  const T* x = reinterpret_cast<const T*>(a.nf) + (size_t)r * a.d;
  float tv[KMAX];
  int ti[KMAX];
#pragma unroll
  for (int j = 0; j < KMAX; ++j) { tv[j] = -INFINITY; ti[j] = 0x7fffffff; }
  for (int v = w; v < a.V; v += 4) {                // increasing token id per wavefront
    float l = dot_row<T>(x, reinterpret_cast<const T*>(a.w_vocab) + (size_t)v * a.d, a.d, lane) * a.scale;
    int li = v;
#pragma unroll
    for (int j = 0; j < KMAX; ++j) {               // sorted insertion: swap down while the newcomer is better
      if (better(l, li, tv[j], ti[j])) {
        const float fv = tv[j]; const int fi = ti[j];
        tv[j] = l; ti[j] = li;
        l = fv; li = fi;
      }
    }
  }
  if (lane == 0) {
#pragma unroll
    for (int j = 0; j < KMAX; ++j) { s_v[w][j] = tv[j]; s_i[w][j] = ti[j]; }
  }
  __syncthreads();
  if (tid == 0) {
    int pos[4] = {0, 0, 0, 0};
    for (int j = 0; j < a.K; ++j) {                 // merge of four sorted lists
      int bw = -1;
      for (int x2 = 0; x2 < 4; ++x2) {
        if (pos[x2] >= KMAX) continue;
        if (bw < 0 || better(s_v[x2][pos[x2]], s_i[x2][pos[x2]], s_v[bw][pos[bw]], s_i[bw][pos[bw]])) bw = x2;
      }
      const float v = s_v[bw][pos[bw]];
      cv[j] = v;
      ci[j] = (v == -INFINITY) ? -1 : s_i[bw][pos[bw]];
      ++pos[bw];
    }
  }
}

__global__ __launch_bounds__(64) void topk_merge_kernel(HeadTopkArgs a) {
  const int b = blockIdx.x, lane = threadIdx.x;
  const int node = a.result ? a.result->node : a.node;
  int32_t* ot = a.out_tokens + (size_t)b * a.K;
  float* op = a.out_probs + (size_t)b * a.K;
  const bool node_ok = node >= 0 && node < a.G;
  const int f = node_ok ? node * a.B + b : 0;
  const int r = node_ok ? find_row(a.row_idx, min(*a.count, a.G * a.B), f) : -1;
  if (r < 0) {                                      // not masked: nothing to draft here
    if (lane < a.K) { ot[lane] = node_ok ? a.tokens[f] : -1; op[lane] = 0.f; }
    return;
  }
  const TopPartial top = a.row_top[r];
  // Column 0 is the head's own argmax with the confidence it reported, whatever the recomputed candidates say
  // (their logits are summed in another order, so on a near-tie the head's token could otherwise drop out of its
  // chunk's K best, or come second).  The other K-1 places go to the best candidates other than that token; a
  // candidate whose recomputed logit exceeds the head's top logit is held at it, so probabilities never increase
  // along a row.
  if (lane == 0) { ot[0] = top.idx; op[0] = 1.0f / top.s; }
  // lane = k * K + j of the candidate table
  float v = -INFINITY;
  int i = -1;
  if (lane < a.K * a.K) {
    const int k = lane / a.K, j = lane % a.K;
    v = a.cand_val[((size_t)b * KMAX + k) * KMAX + j];
    i = a.cand_idx[((size_t)b * KMAX + k) * KMAX + j];
  }
  if (i < 0 || i == top.idx) { v = -INFINITY; i = -1; }
  float key = v;
  const float val = fminf(v, top.m);
  for (int j = 1; j < a.K; ++j) {
    float bk = key;
    int bi = (i < 0) ? 0x7fffffff : i;
    wave_best(bk, bi);
    const bool won = (i >= 0) && i == bi && key == bk && bk != -INFINITY;
    const unsigned long long wm = __ballot(won);
    float pv = 0.f;
    int pt = -1;
    if (wm) {
      const int src = __ffsll((long long)wm) - 1;
      const float lv = __shfl(val, src, 64);
      pt = bi;
      pv = __expf(lv - top.m) / top.s;
    }
    if (lane == 0) { ot[j] = pt; op[j] = pv; }
    if (won) key = -INFINITY;
  }
}

}  // namespace

hipError_t launch_head_topk(const HeadTopkArgs& a, hipStream_t st) {
  if (a.K < 1 || a.K > KMAX || a.B < 1) return hipErrorInvalidValue;
  if (a.n_part > 0) {
    if (a.n_part > 2048 || a.dtype != SPIFFY_BF16 || a.d % 8 != 0) return hipErrorInvalidValue;
    topk_refine_kernel<bf16_t><<<dim3(a.B, a.K), 256, 0, st>>>(a);
  } else if (a.dtype == SPIFFY_F32) {
    topk_full_kernel<float><<<a.B, 256, 0, st>>>(a);
  } else {
    if (a.d % 8 != 0) return hipErrorInvalidValue;
    topk_full_kernel<bf16_t><<<a.B, 256, 0, st>>>(a);
  }
  topk_merge_kernel<<<a.B, 64, 0, st>>>(a);
  return hipGetLastError();
}

}  // namespace spiffy

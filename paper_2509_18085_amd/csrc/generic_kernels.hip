// Shape-agnostic kernels (fp32 math, float or bf16 storage).  They carry the fp32 configuration
// and any bf16 shape the MFMA kernels do not cover, and the small integer / reduction steps of
// every configuration: embedding gather, RMSNorm, masked-row compaction, the LM-head combine and
// decision step (Alg. 1 steps 1-4), and the rotary table.
#include "kernels.h"

namespace spiffy {

// ---------------------------------------------------------------------------------------------
// embedding gather: out[m,:] = w[tok[m],:]
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void embed_kernel(const T* __restrict__ w, const int32_t* __restrict__ tok,
                                                    int d, int V, T* __restrict__ out) {
  const int m = blockIdx.x;
  int t = tok[m];
  t = t < 0 ? 0 : (t >= V ? V - 1 : t);
  const uint4* src = reinterpret_cast<const uint4*>(w + (size_t)t * d);
  uint4* dst = reinterpret_cast<uint4*>(out + (size_t)m * d);
  const int n16 = d * (int)sizeof(T) / 16;
  for (int i = threadIdx.x; i < n16; i += blockDim.x) dst[i] = src[i];
}

hipError_t launch_embed(int dtype, const void* w, const int32_t* tok, int M, int d, int V, void* out,
                        hipStream_t st) {
  if (dtype == SPIFFY_F32)
    embed_kernel<float><<<M, 256, 0, st>>>((const float*)w, tok, d, V, (float*)out);
  else
    embed_kernel<bf16_t><<<M, 256, 0, st>>>((const bf16_t*)w, tok, d, V, (bf16_t*)out);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// row gather of two matrices with one row list: a_out[r,:] = a[row_idx[r],:], b_out[r,:] = b[row_idx[r],:]
// for r < *count (the masked rows of the last layer: attention output and residual stream)
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void gather_rows2_kernel(const uint4* __restrict__ a, int a16, const uint4* __restrict__ b,
                                                           int b16, const int32_t* __restrict__ row_idx,
                                                           const int32_t* __restrict__ count, uint4* __restrict__ a_out,
                                                           uint4* __restrict__ b_out) {
  const int r = blockIdx.x;
  if (r >= *count) return;
  const size_t src = (size_t)row_idx[r];
  for (int i = threadIdx.x; i < a16; i += 256) a_out[(size_t)r * a16 + i] = a[src * a16 + i];
  for (int i = threadIdx.x; i < b16; i += 256) b_out[(size_t)r * b16 + i] = b[src * b16 + i];
}

// out[row_idx[r],:] = in[r,:] for r < *count
__global__ __launch_bounds__(256) void scatter_rows_kernel(const uint4* __restrict__ in, int n16, const int32_t* __restrict__ row_idx,
                                                           const int32_t* __restrict__ count, uint4* __restrict__ out) {
  const int r = blockIdx.x;
  if (r >= *count) return;
  const size_t dst = (size_t)row_idx[r];
  for (int i = threadIdx.x; i < n16; i += 256) out[dst * n16 + i] = in[(size_t)r * n16 + i];
}

hipError_t launch_scatter_rows(const void* in, size_t row_bytes, const int32_t* row_idx, const int32_t* count, int M,
                               void* out, hipStream_t st) {
  scatter_rows_kernel<<<M, 256, 0, st>>>((const uint4*)in, (int)(row_bytes / 16), row_idx, count, (uint4*)out);
  return hipGetLastError();
}

hipError_t launch_gather_rows2(const void* a, size_t a_row_bytes, const void* b, size_t b_row_bytes,
                               const int32_t* row_idx, const int32_t* count, int M, void* a_out, void* b_out,
                               hipStream_t st) {
  gather_rows2_kernel<<<M, 256, 0, st>>>((const uint4*)a, (int)(a_row_bytes / 16), (const uint4*)b, (int)(b_row_bytes / 16),
                                         row_idx, count, (uint4*)a_out, (uint4*)b_out);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// RMSNorm with optional row gather
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float block_sum_256(float v, float* red) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}
__device__ __forceinline__ float block_max_256(float v, float* red) {
  v = wave_max(v);
  const int w = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

// 16 bytes per thread per step; d * sizeof(T) is a multiple of 16 (checked by the host)
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const T* __restrict__ x, const T* __restrict__ gain, float eps,
                                                      int M, int d, const int32_t* __restrict__ row_idx,
                                                      const int32_t* __restrict__ n_rows_dev, T* __restrict__ out) {
  constexpr int VEC = 16 / sizeof(T);
  typedef T vec_t __attribute__((ext_vector_type(VEC)));
  __shared__ float red[4];
  const int r = blockIdx.x;
  const int n_rows = n_rows_dev ? *n_rows_dev : M;
  if (r >= n_rows) return;
  const int src = row_idx ? row_idx[r] : r;
  const vec_t* xr = reinterpret_cast<const vec_t*>(x + (size_t)src * d);
  const vec_t* gr = reinterpret_cast<const vec_t*>(gain);
  vec_t* o = reinterpret_cast<vec_t*>(out + (size_t)r * d);
  const int nv = d / VEC;
  float ss = 0.f;
  for (int i = threadIdx.x; i < nv; i += 256) {
    const vec_t v = xr[i];
#pragma unroll
    for (int e = 0; e < VEC; ++e) { const float f = to_f32(v[e]); ss += f * f; }
  }
  ss = block_sum_256(ss, red);
  const float inv = 1.0f / sqrtf(ss / (float)d + eps);
  for (int i = threadIdx.x; i < nv; i += 256) {
    const vec_t v = xr[i], g = gr[i];
    vec_t w;
#pragma unroll
    for (int e = 0; e < VEC; ++e) w[e] = from_f32<T>(to_f32(v[e]) * inv * to_f32(g[e]));
    o[i] = w;
  }
}

hipError_t launch_rmsnorm(int dtype, const void* x, const void* gain, float eps, int M, int d,
                          const int32_t* row_idx, const int32_t* n_rows_dev, void* out, hipStream_t st) {
  if (dtype == SPIFFY_F32)
    rmsnorm_kernel<float><<<M, 256, 0, st>>>((const float*)x, (const float*)gain, eps, M, d, row_idx, n_rows_dev,
                                             (float*)out);
  else
    rmsnorm_kernel<bf16_t><<<M, 256, 0, st>>>((const bf16_t*)x, (const bf16_t*)gain, eps, M, d, row_idx,
                                              n_rows_dev, (bf16_t*)out);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// generic GEMM  C[m, c0+n] = epi( sum_k A[m,k] W[n,k] ), 64x64 tile, 4x4 per thread
// ---------------------------------------------------------------------------------------------
template <typename T, int EPI>
__global__ __launch_bounds__(256) void gemm_generic_kernel(const T* __restrict__ A, int lda, const T* __restrict__ W,
                                                           const T* __restrict__ W2, const T* __restrict__ bias,
                                                           T* __restrict__ C, int ldc, int c0,
                                                           const T* __restrict__ R, int M, int N, int K,
                                                           const int* __restrict__ M_dev) {
  constexpr int BM = 64, BN = 64, BK = 16;
  __shared__ float As[BK][BM + 4];
  __shared__ float Ws[BK][BN + 4];
  __shared__ float Us[EPI == EPI_SWIGLU ? BK : 1][BN + 4];
  const int Mrows = M_dev ? min(*M_dev, M) : M;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  if (m0 >= Mrows) return;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int lr = threadIdx.x >> 2, lk = (threadIdx.x & 3) * 4;
  float acc[4][4] = {}, acc2[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += BK) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int k = k0 + lk + j;
      const int am = m0 + lr, wn = n0 + lr;
      As[lk + j][lr] = (am < Mrows && k < K) ? to_f32(A[(size_t)am * lda + k]) : 0.f;
      Ws[lk + j][lr] = (wn < N && k < K) ? to_f32(W[(size_t)wn * K + k]) : 0.f;
      if (EPI == EPI_SWIGLU) Us[lk + j][lr] = (wn < N && k < K) ? to_f32(W2[(size_t)wn * K + k]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < BK; ++k) {
      float a[4], b[4], u[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Ws[k][tx * 4 + j];
      if (EPI == EPI_SWIGLU) {
#pragma unroll
        for (int j = 0; j < 4; ++j) u[j] = Us[k][tx * 4 + j];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
          if (EPI == EPI_SWIGLU) acc2[i][j] = fmaf(a[i], u[j], acc2[i][j]);
        }
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= Mrows) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= N) continue;
      float v = acc[i][j];
      if (EPI == EPI_STORE && bias) v += to_f32(bias[n]);
      if (EPI == EPI_RESID) v += to_f32(R[(size_t)m * ldc + c0 + n]);
      if (EPI == EPI_SWIGLU) v = v / (1.f + __expf(-v)) * acc2[i][j];
      C[(size_t)m * ldc + c0 + n] = from_f32<T>(v);
    }
  }
}

template <typename T>
static hipError_t gemm_generic_t(int epi, const GemmArgs& a, hipStream_t st) {
  const dim3 blk(256);
  if (epi == EPI_SWIGLU) {
    dim3 grid(cdiv(a.N, 64), cdiv(a.M, 64));
    gemm_generic_kernel<T, EPI_SWIGLU><<<grid, blk, 0, st>>>((const T*)a.A, a.lda, (const T*)a.W[0], (const T*)a.W[1],
                                                             nullptr, (T*)a.C, a.ldc, 0, nullptr, a.M, a.N, a.K,
                                                             a.M_dev);
    return hipGetLastError();
  }
  int c0 = 0;
  for (int s = 0; s < 3; ++s) {
    if (a.Nseg[s] <= 0 || !a.W[s]) continue;
    dim3 grid(cdiv(a.Nseg[s], 64), cdiv(a.M, 64));
    if (epi == EPI_RESID)
      gemm_generic_kernel<T, EPI_RESID><<<grid, blk, 0, st>>>((const T*)a.A, a.lda, (const T*)a.W[s], nullptr, nullptr,
                                                              (T*)a.C, a.ldc, c0, (const T*)a.R, a.M, a.Nseg[s], a.K,
                                                              a.M_dev);
    else
      gemm_generic_kernel<T, EPI_STORE><<<grid, blk, 0, st>>>((const T*)a.A, a.lda, (const T*)a.W[s], nullptr,
                                                              (const T*)a.bias[s], (T*)a.C, a.ldc, c0, nullptr, a.M,
                                                              a.Nseg[s], a.K, a.M_dev);
    c0 += a.Nseg[s];
  }
  return hipGetLastError();
}

hipError_t launch_gemm_generic(int dtype, int epi, const GemmArgs& a, hipStream_t st) {
  return dtype == SPIFFY_F32 ? gemm_generic_t<float>(epi, a, st) : gemm_generic_t<bf16_t>(epi, a, st);
}

// ---------------------------------------------------------------------------------------------
// generic attention: one workgroup per (state g, position b, query head h)
// keys = [P cached keys ; the B keys of state g ; S cached keys of the tokens after the block (dual cache)],
// bidirectional inside the block (Fig. 4); cache row j holds sequence position j, so rows P .. P+B-1 of the
// cache (the slot of the block itself) are never read
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void attn_generic_kernel(const T* __restrict__ qkv, const T* __restrict__ pk,
                                                           const T* __restrict__ pv, T* __restrict__ out, int G,
                                                           int B, int Hq, int Hkv, int hd, int P, int S, int ldp,
                                                           int pos0, float rope_base, int own) {
  extern __shared__ float smem[];
  __shared__ float red[4];
  const int half = hd >> 1;
  float* qs = smem;              // [hd] rotated query
  float* cs = qs + hd;           // [B][half] cos
  float* sn = cs + B * half;     // [B][half] sin
  float* sc = sn + B * half;     // [P+B+S] scores
  float* acc = sc + (P + B + S); // [nchunk][hd]
  const int h = blockIdx.x % Hq;
  const int m = blockIdx.x / Hq;       // flattened (g,b)
  const int g = m / B, b = m % B;
  const int kvh = h / (Hq / Hkv);
  const int ld = (Hq + 2 * Hkv) * hd;
  // own == 0 (queries that are not a block of their own: the true suffix): cache rows 0 .. P-1 only
  const int T_all = own ? P + B + S : P;
  for (int i = threadIdx.x; i < B * half; i += 256) {
    const int bb = i / half, f = i % half;
    const double inv_freq = pow((double)rope_base, -2.0 * (double)f / (double)hd);
    const double ang = (double)(pos0 + bb) * inv_freq;
    cs[i] = (float)cos(ang);
    sn[i] = (float)sin(ang);
  }
  __syncthreads();
  const T* qrow = qkv + (size_t)m * ld + h * hd;
  for (int f = threadIdx.x; f < half; f += 256) {
    const float x1 = to_f32(qrow[f]), x2 = to_f32(qrow[f + half]);
    const float c = cs[b * half + f], s = sn[b * half + f];
    qs[f] = x1 * c - x2 * s;
    qs[f + half] = x2 * c + x1 * s;
  }
  __syncthreads();
  const float scale = 1.0f / sqrtf((float)hd);
  float mx = -INFINITY;
  for (int j = threadIdx.x; j < T_all; j += 256) {
    float dot = 0.f;
    if (j < P || j >= P + B) {
      const T* kr = pk + ((size_t)kvh * ldp + j) * hd;
      for (int i = 0; i < hd; ++i) dot = fmaf(qs[i], to_f32(kr[i]), dot);
    } else {
      const int bb = j - P;
      const T* kr = qkv + (size_t)(g * B + bb) * ld + (Hq + kvh) * hd;
      for (int f = 0; f < half; ++f) {
        const float x1 = to_f32(kr[f]), x2 = to_f32(kr[f + half]);
        const float c = cs[bb * half + f], s = sn[bb * half + f];
        dot = fmaf(qs[f], x1 * c - x2 * s, dot);
        dot = fmaf(qs[f + half], x2 * c + x1 * s, dot);
      }
    }
    dot *= scale;
    sc[j] = dot;
    mx = fmaxf(mx, dot);
  }
  mx = block_max_256(mx, red);
  float sum = 0.f;
  for (int j = threadIdx.x; j < T_all; j += 256) {
    const float e = __expf(sc[j] - mx);
    sc[j] = e;
    sum += e;
  }
  sum = block_sum_256(sum, red);   // also orders the sc[] writes before the reads below
  const int nchunk = max(1, 256 / hd);
  const int c = threadIdx.x / hd, t = threadIdx.x % hd;
  if (c < nchunk) {
    const int per = (T_all + nchunk - 1) / nchunk;
    const int j0 = c * per, j1 = min(T_all, j0 + per);
    float o = 0.f;
    for (int j = j0; j < j1; ++j) {
      const float v = (j < P || j >= P + B) ? to_f32(pv[((size_t)kvh * ldp + j) * hd + t])
                              : to_f32(qkv[(size_t)(g * B + (j - P)) * ld + (Hq + Hkv + kvh) * hd + t]);
      o = fmaf(sc[j], v, o);
    }
    acc[c * hd + t] = o;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < hd; i += 256) {
    float o = 0.f;
    for (int cc = 0; cc < nchunk; ++cc) o += acc[cc * hd + i];
    out[(size_t)m * (Hq * hd) + h * hd + i] = from_f32<T>(o / sum);
  }
}

size_t attn_generic_smem(int B, int hd, int P) {   // P = cached keys, prefix and suffix together
  const int nchunk = 256 / hd > 0 ? 256 / hd : 1;
  return sizeof(float) * ((size_t)hd + (size_t)B * hd + (size_t)(P + B) + (size_t)nchunk * hd);
}

hipError_t launch_attn_generic(int dtype, const AttnArgs& a, hipStream_t st) {
  const size_t smem = attn_generic_smem(a.B, a.hd, a.P + a.S);
  const int grid = a.G * a.B * a.Hq;
  if (dtype == SPIFFY_F32) {
    hipError_t e = hipFuncSetAttribute((const void*)attn_generic_kernel<float>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attn_generic_kernel<float><<<grid, 256, smem, st>>>((const float*)a.qkv, (const float*)a.prefix_k,
                                                        (const float*)a.prefix_v, (float*)a.out, a.G, a.B, a.Hq,
                                                        a.Hkv, a.hd, a.P, a.S, a.ldp ? a.ldp : a.P, a.pos0, a.rope_base, a.own);
  } else {
    hipError_t e = hipFuncSetAttribute((const void*)attn_generic_kernel<bf16_t>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attn_generic_kernel<bf16_t><<<grid, 256, smem, st>>>((const bf16_t*)a.qkv, (const bf16_t*)a.prefix_k,
                                                         (const bf16_t*)a.prefix_v, (bf16_t*)a.out, a.G, a.B, a.Hq,
                                                         a.Hkv, a.hd, a.P, a.S, a.ldp ? a.ldp : a.P, a.pos0, a.rope_base, a.own);
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// masked-row compaction: row_idx[0..count) ascending, plus count (single workgroup)
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void compact_rows_kernel(const int32_t* __restrict__ tok,
                                                           const uint8_t* __restrict__ mask, int mask_id, int M,
                                                           int32_t* __restrict__ row_idx, int32_t* __restrict__ count) {
  __shared__ int cnt[256];
  const int per = (M + 255) / 256;
  const int i0 = threadIdx.x * per, i1 = min(M, i0 + per);
  int c = 0;
  for (int i = i0; i < i1; ++i) c += mask ? (mask[i] != 0) : (tok[i] == mask_id);
  cnt[threadIdx.x] = c;
  __syncthreads();
  // exclusive scan by a simple doubling pass
  for (int o = 1; o < 256; o <<= 1) {
    const int v = (threadIdx.x >= o) ? cnt[threadIdx.x - o] : 0;
    __syncthreads();
    cnt[threadIdx.x] += v;
    __syncthreads();
  }
  int pos = cnt[threadIdx.x] - c;
  for (int i = i0; i < i1; ++i) {
    const bool mk = mask ? (mask[i] != 0) : (tok[i] == mask_id);
    if (mk) row_idx[pos++] = i;
  }
  if (threadIdx.x == 255) *count = cnt[255];
}

hipError_t launch_compact_rows(const int32_t* tok, const uint8_t* mask, int mask_id, int M, int32_t* row_idx,
                               int32_t* count, hipStream_t st) {
  compact_rows_kernel<<<1, 256, 0, st>>>(tok, mask, mask_id, M, row_idx, count);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// prefix-cache extension: one thread per (token b, kv head, frequency f)
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void kv_append_kernel(const T* __restrict__ qkv, int Hq, int Hkv, int hd, int B,
                                                        int pos0, float base, T* __restrict__ ck, T* __restrict__ cv,
                                                        int P, int ldp, int B0, int skip,
                                                        const float2* __restrict__ tab_a,
                                                        const float2* __restrict__ tab_b) {
  const int half = hd / 2;
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= B * Hkv * half) return;
  const int f = i % half, kvh = (i / half) % Hkv, b = i / (half * Hkv);
  const int ld = (Hq + 2 * Hkv) * hd;
  const int src = b < B0 ? b : b + skip;      // the rows may come in two runs: B0 rows, `skip` rows that are not appended, the rest
  const T* kr = qkv + (size_t)src * ld + (Hq + kvh) * hd;
  const T* vr = qkv + (size_t)src * ld + (Hq + Hkv + kvh) * hd;
  // same table values as the attention kernels use: angle in double, cos / sin rounded to float
  float c, s;
  if (tab_a) {      // the table the attention kernels rotate with: [f][row]
    const float2 cs = b < B0 ? tab_a[(size_t)f * B0 + b] : tab_b[(size_t)f * (B - B0) + (b - B0)];
    c = cs.x;
    s = cs.y;
  } else {
    const double inv_freq = pow((double)base, -2.0 * (double)f / (double)hd);
    const double ang = (double)(pos0 + b) * inv_freq;
    c = (float)cos(ang);
    s = (float)sin(ang);
  }
  const float x1 = to_f32(kr[f]), x2 = to_f32(kr[f + half]);
  T* kd = ck + ((size_t)kvh * ldp + P + b) * hd;
  T* vd = cv + ((size_t)kvh * ldp + P + b) * hd;
  kd[f] = from_f32<T>(x1 * c - x2 * s);
  kd[f + half] = from_f32<T>(x2 * c + x1 * s);
  vd[f] = vr[f];
  vd[f + half] = vr[f + half];
}

hipError_t launch_kv_append(int dtype, const void* qkv, int Hq, int Hkv, int hd, int B, int pos0, float rope_base,
                            void* cache_k, void* cache_v, int P, int ldp, hipStream_t st, int B0, int skip,
                            const void* tab_a, const void* tab_b) {
  if (B0 <= 0) { B0 = B; skip = 0; }
  if (!tab_a || (B0 < B && !tab_b)) tab_a = tab_b = nullptr;
  const int n = B * Hkv * (hd / 2);
  if (dtype == SPIFFY_F32)
    kv_append_kernel<float><<<cdiv(n, 256), 256, 0, st>>>((const float*)qkv, Hq, Hkv, hd, B, pos0, rope_base,
                                                          (float*)cache_k, (float*)cache_v, P, ldp, B0, skip,
                                                          (const float2*)tab_a, (const float2*)tab_b);
  else
    kv_append_kernel<bf16_t><<<cdiv(n, 256), 256, 0, st>>>((const bf16_t*)qkv, Hq, Hkv, hd, B, pos0, rope_base,
                                                           (bf16_t*)cache_k, (bf16_t*)cache_v, P, ldp, B0, skip,
                                                           (const float2*)tab_a, (const float2*)tab_b);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// generic LM head: one workgroup per compacted row, logits live only in registers
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void lmhead_generic_kernel(const T* __restrict__ n, const T* __restrict__ wv, int d,
                                                             int V, float scale, const int32_t* __restrict__ count,
                                                             TopPartial* __restrict__ row_top) {
  extern __shared__ float smem[];
  __shared__ TopPartial wtop[4];
  const int r = blockIdx.x;
  if (r >= *count) return;
  float* ns = smem;
  for (int i = threadIdx.x; i < d; i += 256) ns[i] = to_f32(n[(size_t)r * d + i]);
  __syncthreads();
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  Top top = top_empty();
  for (int v = w; v < V; v += 4) {
    const T* wr = wv + (size_t)v * d;
    float dot = 0.f;
    for (int i = lane; i < d; i += 64) dot = fmaf(ns[i], to_f32(wr[i]), dot);
    dot = wave_sum(dot) * scale;
    top = top_push(top, dot, v);
  }
  if (lane == 0) wtop[w] = TopPartial{top.m, top.m2, top.s, top.idx};
  __syncthreads();
  if (threadIdx.x == 0) {
    Top t = top_empty();
    for (int i = 0; i < 4; ++i) t = top_merge(t, Top{wtop[i].m, wtop[i].m2, wtop[i].s, wtop[i].idx});
    row_top[r] = TopPartial{t.m, t.m2, t.s, t.idx};
  }
}

hipError_t launch_lmhead_generic(int dtype, const void* n, const void* w_vocab, int d, int V, float scale,
                                 const int32_t* count, int M, TopPartial* row_top, hipStream_t st) {
  const size_t smem = sizeof(float) * (size_t)d;
  if (dtype == SPIFFY_F32)
    lmhead_generic_kernel<float><<<M, 256, smem, st>>>((const float*)n, (const float*)w_vocab, d, V, scale, count,
                                                       row_top);
  else
    lmhead_generic_kernel<bf16_t><<<M, 256, smem, st>>>((const bf16_t*)n, (const bf16_t*)w_vocab, d, V, scale,
                                                        count, row_top);
  return hipGetLastError();
}

// merge the per-tile partial summaries part[n_part][m_cap] of each row; lanes run along rows so
// the reads are coalesced, four wavefronts split the partials of the same 64 rows.  blockIdx.y
// selects a slice of the partials (two-level merge when there are many): out is [gridDim.y][m_cap].
__global__ __launch_bounds__(256) void lmhead_combine_kernel(const TopPartial* __restrict__ part, int n_part,
                                                             int m_cap, const int32_t* __restrict__ count,
                                                             TopPartial* __restrict__ out) {
  __shared__ TopPartial sh[4][64];
  const int n = *count;
  const int r0 = blockIdx.x * 64;
  if (r0 >= n) return;
  const int per = (n_part + gridDim.y - 1) / gridDim.y;
  const int p0 = blockIdx.y * per, p1 = min(n_part, p0 + per);
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r = r0 + lane;
  Top t = top_empty();
  if (r < n) {
    for (int i = p0 + w; i < p1; i += 4) {
      const TopPartial p = part[(size_t)i * m_cap + r];
      t = top_merge(t, Top{p.m, p.m2, p.s, p.idx});
    }
  }
  sh[w][lane] = TopPartial{t.m, t.m2, t.s, t.idx};
  __syncthreads();
  if (w == 0 && r < n) {
    Top a = top_empty();
    for (int i = 0; i < 4; ++i) a = top_merge(a, Top{sh[i][lane].m, sh[i][lane].m2, sh[i][lane].s, sh[i][lane].idx});
    out[(size_t)blockIdx.y * m_cap + r] = TopPartial{a.m, a.m2, a.s, a.idx};
  }
}

hipError_t launch_lmhead_combine(const TopPartial* part, int n_part, int m_cap, const int32_t* count, int M,
                                 TopPartial* tmp, TopPartial* row_top, hipStream_t st) {
  const int slices = kLmheadCombineSlices;
  if (n_part > 2 * slices && tmp) {
    lmhead_combine_kernel<<<dim3(cdiv(M, 64), slices), 256, 0, st>>>(part, n_part, m_cap, count, tmp);
    lmhead_combine_kernel<<<dim3(cdiv(M, 64), 1), 256, 0, st>>>(tmp, slices, m_cap, count, row_top);
  } else {
    lmhead_combine_kernel<<<dim3(cdiv(M, 64), 1), 256, 0, st>>>(part, n_part, m_cap, count, row_top);
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// decisions per state (Alg. 1 steps 2-4 + threshold rule): one wavefront per state g
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void head_finalize_kernel(const TopPartial* __restrict__ row_top,
                                                           const int32_t* __restrict__ row_idx,
                                                           const int32_t* __restrict__ count,
                                                           const int32_t* __restrict__ tok,
                                                           const uint8_t* __restrict__ mask, int mask_id, int B,
                                                           float threshold, int force_one,
                                                           int32_t* __restrict__ argmax, float* __restrict__ conf,
                                                           uint8_t* __restrict__ unmask, float* __restrict__ margin,
                                                           int32_t* __restrict__ target) {
  const int g = blockIdx.x;
  const int lane = threadIdx.x;
  const int n = *count;
  // first compacted row belonging to state g: lower bound of g*B in the ascending row list
  int lo = 0, hi = n;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (row_idx[mid] < g * B) lo = mid + 1; else hi = mid;
  }
  float best_c = -1.f;     // highest confidence among this lane's masked positions
  int best_b = 0x7fffffff, best_am = 0;
  bool any_pass = false;
  int base = lo;
  for (int b0 = 0; b0 < B; b0 += 64) {
    const int b = b0 + lane;
    const bool in = b < B;
    const int m = g * B + (in ? b : 0);
    const int t = in ? tok[m] : 0;
    const bool mk = in && (mask ? (mask[m] != 0) : (t == mask_id));
    const unsigned long long bal = __ballot(mk);
    const int r = base + __popcll(bal & ((1ull << lane) - 1ull));
    base += __popcll(bal);
    if (in) {
      int am = t;
      float cf = 0.f, mg = INFINITY;
      uint8_t um = 0;
      if (mk) {
        const TopPartial p = row_top[r];
        am = p.idx;
        cf = 1.0f / p.s;
        mg = p.m - p.m2;
        um = cf > threshold ? 1 : 0;
        if (um) any_pass = true;
        if (cf > best_c) { best_c = cf; best_b = b; best_am = am; }
      }
      argmax[m] = am;
      conf[m] = cf;
      unmask[m] = um;
      if (margin) margin[m] = mg;
      if (target) target[m] = um ? am : t;
    }
  }
  const bool any = __ballot(any_pass) != 0ull;
  if (force_one && !any) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const float oc = __shfl_xor(best_c, o, 64);
      const int ob = __shfl_xor(best_b, o, 64);
      const int oa = __shfl_xor(best_am, o, 64);
      if (oc > best_c || (oc == best_c && ob < best_b)) { best_c = oc; best_b = ob; best_am = oa; }
    }
    if (best_c >= 0.f && lane == (best_b & 63)) {   // the lane that wrote this position rewrites it
      const int m = g * B + best_b;
      unmask[m] = 1;
      if (target) target[m] = best_am;
    }
  }
}

hipError_t launch_head_finalize(const TopPartial* row_top, const int32_t* row_idx, const int32_t* count,
                                const int32_t* tok, const uint8_t* mask, int mask_id, int G, int B, float threshold,
                                int force_one, int32_t* argmax, float* conf, uint8_t* unmask, float* margin,
                                int32_t* target, hipStream_t st) {
  head_finalize_kernel<<<G, 64, 0, st>>>(row_top, row_idx, count, tok, mask, mask_id, B, threshold, force_one,
                                         argmax, conf, unmask, margin, target);
  return hipGetLastError();
}

}  // namespace spiffy

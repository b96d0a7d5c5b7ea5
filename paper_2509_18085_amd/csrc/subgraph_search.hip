// Offline calibration, part 3 (Alg. 2; App. D.1): the optimal connected subgraph of the candidate graph.
//
//   G' = all node sets Q of size D in which every node is of level 1 or 2 or has a parent in Q
//   G* = argmax over G' of the summed counts; equal sums go to the smaller bit mask sum_q 2^q
//
// Every one of the C(N, D) node sets is tried (the paper's brute force), N <= 64.  A set is a 64-bit mask
// x; with child[p] = mask of the children of p, x is connected iff  x & ~(root | OR_{p in x} child[p]) == 0.
//
// Work split: the h = min(N, 12) lowest nodes are the "low" part.  Each workgroup tabulates in LDS, for every
// subset A of the low nodes, (sum of counts, ~OR of child masks, A), grouped by |A|.  A set is B | A with B a
// subset of the N - h high nodes and |B| = D - |A|.  For each size a = |A| the C(N-h, D-a) high subsets are
// shared out evenly over all threads of the grid as contiguous ranges of colexicographic ranks; a thread
// unranks the first, steps to the next with the same-popcount successor, computes (sum, cover) of B once and
// then runs over all C(h, a) table entries of the group: per tried set two 64-bit adds/ands, one OR, a zero
// test and a compare.  All lanes of a wavefront read the same table entry (LDS broadcast) and loop counts are
// uniform, so lanes diverge only at the end of a range.
#include "kernels.h"

namespace spiffy {

namespace {

constexpr int kLow = 12;                       // tabulated low nodes (2^12 entries)
constexpr int kThreads = 1024;
constexpr int kBinomN = 65;                    // binomials C(n, k), 0 <= n, k <= 64, saturating
constexpr unsigned long long kSat = ~0ull;

struct SgWorkspace {                           // device memory, filled by the prepare kernel
  unsigned long long child[64];
  unsigned long long root;
  unsigned long long binom[kBinomN * kBinomN];
};
struct SgPartial {
  long long best_sum;
  unsigned long long best_mask;
  unsigned long long n_connected;
};

// child masks, root mask, binomial table; one wavefront
__global__ __launch_bounds__(64) void sg_prepare_kernel(const int32_t* __restrict__ level, int N,
                                                        const int32_t* __restrict__ edges, int E, SgWorkspace* ws) {
  __shared__ unsigned long long s_child[64];
  __shared__ unsigned long long s_row[2][kBinomN];
  const int lane = threadIdx.x;
  s_child[lane] = 0ull;
  __syncthreads();
  for (int e = lane; e < E; e += 64) {
    const int p = edges[2 * e], q = edges[2 * e + 1];
    if (p >= 0 && p < N && q >= 0 && q < N) atomicOr(&s_child[p], 1ull << q);
  }
  const bool is_root = lane < N && (level[lane] == 1 || level[lane] == 2);
  const unsigned long long root = __ballot(is_root);
  __syncthreads();
  ws->child[lane] = s_child[lane];
  if (lane == 0) ws->root = root;
  // Pascal's triangle, one row per step; sums that do not fit 64 bits stick at the maximum
  for (int k = lane; k < kBinomN; k += 64) s_row[0][k] = k == 0 ? 1ull : 0ull;
  __syncthreads();
  for (int n = 0; n < kBinomN; ++n) {
    const unsigned long long* cur = s_row[n & 1];
    unsigned long long* nxt = s_row[(n + 1) & 1];
    for (int k = lane; k < kBinomN; k += 64) {
      ws->binom[n * kBinomN + k] = cur[k];
      const unsigned long long a = cur[k], b = k > 0 ? cur[k - 1] : 0ull;
      const unsigned long long s = a + b;
      nxt[k] = (a == kSat || b == kSat || s < a) ? kSat : s;
    }
    __syncthreads();
  }
}

__device__ __forceinline__ bool better(long long s, unsigned long long x, long long s2, unsigned long long x2) {
  return s > s2 || (s == s2 && x < x2);
}

__global__ __launch_bounds__(kThreads) void sg_search_kernel(const long long* __restrict__ count, int N, int D,
                                                             const SgWorkspace* __restrict__ ws,
                                                             SgPartial* __restrict__ partial) {
  extern __shared__ __align__(16) unsigned char sg_smem[];
  unsigned long long* binom = reinterpret_cast<unsigned long long*>(sg_smem);            // [65][65]
  long long* tab_sum = reinterpret_cast<long long*>(binom + kBinomN * kBinomN);          // [2^h]
  unsigned long long* tab_ncov = reinterpret_cast<unsigned long long*>(tab_sum + (1 << kLow));
  unsigned short* tab_low = reinterpret_cast<unsigned short*>(tab_ncov + (1 << kLow));
  __shared__ unsigned long long s_child[64];
  __shared__ long long s_cnt[64];
  __shared__ int s_off[kLow + 2];
  __shared__ SgPartial s_red[kThreads / 64];

  const int tid = threadIdx.x;
  const int h = N < kLow ? N : kLow;
  const int nH = N - h;
  for (int i = tid; i < kBinomN * kBinomN; i += kThreads) binom[i] = ws->binom[i];
  if (tid < 64) {
    s_child[tid] = ws->child[tid];
    s_cnt[tid] = tid < N ? count[tid] : 0;
  }
  __syncthreads();
  if (tid == 0) {
    int o = 0;
    for (int a = 0; a <= h; ++a) {
      s_off[a] = o;
      o += (int)binom[h * kBinomN + a];
    }
    s_off[h + 1] = o;
  }
  __syncthreads();
  // table of the low subsets, grouped by size, colexicographic inside a group
  for (int v = tid; v < (1 << h); v += kThreads) {
    long long s = 0;
    unsigned long long cov = 0ull;
    int r = 0, i = 0;
    for (int m = v; m; m &= m - 1) {
      const int c = __ffs(m) - 1;
      ++i;
      r += (int)binom[c * kBinomN + i];
      s += s_cnt[c];
      cov |= s_child[c];
    }
    const int idx = s_off[i] + r;
    tab_sum[idx] = s;
    tab_ncov[idx] = ~cov;
    tab_low[idx] = (unsigned short)v;
  }
  __syncthreads();

  const unsigned long long root = ws->root;
  const unsigned long long gtid = (unsigned long long)blockIdx.x * kThreads + tid;
  const unsigned long long nth = (unsigned long long)gridDim.x * kThreads;
  long long best = (long long)(1ull << 63);      // below any reachable sum
  unsigned long long bestx = ~0ull;
  unsigned int n_conn = 0;
  unsigned long long n_conn_hi = 0;              // flushed from n_conn once per high subset

  for (int a = 0; a <= h; ++a) {
    const int kB = D - a;
    if (kB < 0 || kB > nH) continue;
    const unsigned long long nb = binom[nH * kBinomN + kB];
    const int nE = (int)binom[h * kBinomN + a];
    const int e0 = s_off[a];
    const unsigned long long per = (nb + nth - 1) / nth;
    const unsigned long long r0 = gtid * per;
    const unsigned long long r1 = r0 + per < nb ? r0 + per : nb;     // my ranks: [r0, r1)
    unsigned long long Bh = 0ull;                                    // high subset, bit c = node h + c
    if (r0 < nb) {
      unsigned long long r = r0;
      int c = nH - 1;
      for (int i = kB; i >= 1; --i) {
        while (binom[c * kBinomN + i] > r) --c;
        Bh |= 1ull << c;
        r -= binom[c * kBinomN + i];
        --c;
      }
    }
    for (unsigned long long it = 0; it < per; ++it) {
      const bool valid = r0 + it < r1;
      long long sumB = 0;
      unsigned long long covB = root;
      for (unsigned long long m = valid ? Bh : 0ull; m; m &= m - 1) {
        const int c = h + __ffsll((long long)m) - 1;
        sumB += s_cnt[c];
        covB |= s_child[c];
      }
      if (!__any(valid)) continue;                 // the whole wavefront is past its ranges
      const unsigned long long B = Bh << h;        // h <= 12
      const unsigned long long nB = ~covB;
      for (int e = 0; e < nE; ++e) {
        const long long s = sumB + tab_sum[e0 + e];
        const unsigned long long x = B | tab_low[e0 + e];
        const bool ok = valid && (x & nB & tab_ncov[e0 + e]) == 0ull;
        n_conn += ok ? 1u : 0u;
        if (ok && s >= best) {
          if (better(s, x, best, bestx)) {
            best = s;
            bestx = x;
          }
        }
      }
      n_conn_hi += n_conn;
      n_conn = 0;
      if (valid && r0 + it + 1 < r1) {             // successor with the same number of bits
        const unsigned long long lo = Bh & (0ull - Bh);
        const unsigned long long rp = Bh + lo;
        Bh = (((rp ^ Bh) >> 2) >> (__ffsll((long long)Bh) - 1)) | rp;
      }
    }
  }

  // workgroup reduction
  const int lane = tid & 63, wave = tid >> 6;
  for (int o = 32; o >= 1; o >>= 1) {
    const long long s2 = __shfl_xor(best, o, 64);
    const unsigned long long x2 = __shfl_xor(bestx, o, 64);
    n_conn_hi += __shfl_xor(n_conn_hi, o, 64);
    if (better(s2, x2, best, bestx)) {
      best = s2;
      bestx = x2;
    }
  }
  if (lane == 0) {
    s_red[wave].best_sum = best;
    s_red[wave].best_mask = bestx;
    s_red[wave].n_connected = n_conn_hi;
  }
  __syncthreads();
  if (tid == 0) {
    SgPartial p = s_red[0];
    for (int w = 1; w < kThreads / 64; ++w) {
      p.n_connected += s_red[w].n_connected;
      if (better(s_red[w].best_sum, s_red[w].best_mask, p.best_sum, p.best_mask)) {
        p.best_sum = s_red[w].best_sum;
        p.best_mask = s_red[w].best_mask;
      }
    }
    partial[blockIdx.x] = p;
  }
}

__global__ __launch_bounds__(64) void sg_final_kernel(const SgPartial* __restrict__ partial, int n_partial, int D,
                                                      unsigned long long* best_mask, long long* best_sum,
                                                      unsigned long long* n_connected, int32_t* nodes_out) {
  const int lane = threadIdx.x;
  long long best = (long long)(1ull << 63);
  unsigned long long bestx = ~0ull, n = 0ull;
  for (int i = lane; i < n_partial; i += 64) {
    n += partial[i].n_connected;
    if (better(partial[i].best_sum, partial[i].best_mask, best, bestx)) {
      best = partial[i].best_sum;
      bestx = partial[i].best_mask;
    }
  }
  for (int o = 32; o >= 1; o >>= 1) {
    const long long s2 = __shfl_xor(best, o, 64);
    const unsigned long long x2 = __shfl_xor(bestx, o, 64);
    n += __shfl_xor(n, o, 64);
    if (better(s2, x2, best, bestx)) {
      best = s2;
      bestx = x2;
    }
  }
  if (n == 0ull) {            // no connected set of this size
    best = 0;
    bestx = 0ull;
  }
  if (lane == 0) {
    *best_mask = bestx;
    *best_sum = best;
    *n_connected = n;
  }
  if (nodes_out && lane < D) {      // ascending node ids, -1 when there is no set
    int node = -1;
    if (n != 0ull) {
      unsigned long long m = bestx;
      for (int i = 0; i < lane; ++i) m &= m - 1;
      node = __ffsll((long long)m) - 1;
    }
    nodes_out[lane] = node;
  }
}

constexpr size_t kSgSmem = sizeof(unsigned long long) * kBinomN * kBinomN + (sizeof(long long) + sizeof(unsigned long long)) * (1 << kLow) +
                           sizeof(unsigned short) * (1 << kLow);

}  // namespace

int subgraph_search_max_blocks() { return 1024; }

size_t subgraph_search_workspace_bytes() {
  return align_up(sizeof(SgWorkspace), 256) + align_up(sizeof(SgPartial) * subgraph_search_max_blocks(), 256);
}

hipError_t launch_subgraph_search(const SubgraphArgs& a, hipStream_t st) {
  static int n_cu = 0;
  if (n_cu == 0) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    hipDeviceProp_t prop;
    e = hipGetDeviceProperties(&prop, dev);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void*)sg_search_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kSgSmem);
    if (e != hipSuccess) return e;
    n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  }
  // one workgroup per compute unit (the table fills most of the LDS), fewer when there is little to share out
  int blocks = n_cu < subgraph_search_max_blocks() ? n_cu : subgraph_search_max_blocks();
  const unsigned long long per_block = 64ull * kThreads;
  if (a.total_sets < (unsigned long long)blocks * per_block)
    blocks = (int)((a.total_sets + per_block - 1) / per_block);
  if (blocks < 1) blocks = 1;
  unsigned char* w = reinterpret_cast<unsigned char*>(a.workspace);
  SgWorkspace* ws = reinterpret_cast<SgWorkspace*>(w);
  SgPartial* partial = reinterpret_cast<SgPartial*>(w + align_up(sizeof(SgWorkspace), 256));
  sg_prepare_kernel<<<1, 64, 0, st>>>(a.level, a.N, a.edges, a.E, ws);
  sg_search_kernel<<<blocks, kThreads, kSgSmem, st>>>((const long long*)a.count, a.N, a.D, ws, partial);
  sg_final_kernel<<<1, 64, 0, st>>>(partial, blocks, a.D, (unsigned long long*)a.best_mask, (long long*)a.best_sum,
                                    (unsigned long long*)a.n_connected, a.nodes_out);
  return hipGetLastError();
}

}  // namespace spiffy

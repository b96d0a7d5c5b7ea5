// Offline calibration, part 3 (Alg. 2; App. D.1): the optimal connected subgraph of the candidate graph.
//
//   G' = all node sets Q of size D in which every node is of level 1 or 2 or has a parent in Q
//   G* = argmax over G' of the summed counts; equal sums go to the smaller bit mask sum_q 2^q
//
// Every one of the C(N, D) node sets is tried (the paper's brute force), N <= 64.  A set is a 64-bit mask
// x; with child[p] = mask of the children of p, x is connected iff  x & ~(root | OR_{p in x} child[p]) == 0.
//
// Work split: the h = min(N, 12) lowest nodes are the "low" part.  A one-workgroup kernel tabulates, for every
// subset A of the low nodes, (sum of counts, a cover word P, A), grouped by |A|.  A set is B | A with B a subset
// of the N - h high nodes and |B| = D - |A|.  For each size a = |A| the C(N-h, D-a) high subsets are shared out
// evenly over all threads of the grid as contiguous ranges of colexicographic ranks; a thread unranks the
// first, steps to the next with the same-popcount successor, computes (sum, cover) of B once and then runs
// over all C(h, a) table entries of the group.  P holds, above bit h, the nodes A does not cover and, below
// it, the nodes of A that neither A nor a root level covers; with TB = (B | low bits) & ~(root | cover of B)
// the set B | A is connected iff P & TB == 0.  Per tried set: two ANDs, a zero test, a 64-bit add and a compare
// against the lane's best; the connected sets are counted per wavefront from the lane mask.  Every lane of a
// wavefront needs the same table entry and loop counts are uniform, so the entries are read once per
// wavefront through the scalar data path and lanes diverge only at the end of a range.
#include "kernels.h"

namespace spiffy {

namespace {

constexpr int kLow = 12;                       // tabulated low nodes (2^12 entries)
constexpr int kThreads = 1024;
constexpr int kBinomN = 65;                    // binomials C(n, k), 0 <= n, k <= 64, saturating
constexpr unsigned long long kSat = ~0ull;

struct __align__(16) SgEntry {
  long long sum;
  unsigned long long P;
};
struct SgWorkspace {                           // device memory, filled by the prepare kernel
  SgEntry tab[(1 << kLow) + 1];                // low subsets grouped by size; one spare entry for the read-ahead
  unsigned long long child[64];
  unsigned long long root;
  unsigned long long binom[kBinomN * kBinomN];
  int off[kLow + 2];                           // first table entry of each size group
  unsigned short tab_low[1 << kLow];           // the subset itself
};
struct SgPartial {
  long long best_sum;
  unsigned long long best_mask;
  unsigned long long n_connected;
};

// child masks, root mask, binomial table, table of the low subsets; one workgroup
__global__ __launch_bounds__(kThreads) void sg_prepare_kernel(const long long* __restrict__ count,
                                                              const int32_t* __restrict__ level, int N,
                                                              const int32_t* __restrict__ edges, int E, SgWorkspace* ws) {
  __shared__ unsigned long long s_child[64];
  __shared__ long long s_cnt[64];
  __shared__ unsigned long long s_binom[kBinomN * kBinomN];
  __shared__ int s_off[kLow + 2];
  __shared__ unsigned long long s_root;
  const int tid = threadIdx.x;
  const int h = N < kLow ? N : kLow;
  if (tid < 64) {
    s_child[tid] = 0ull;
    s_cnt[tid] = tid < N ? count[tid] : 0;
  }
  __syncthreads();
  for (int e = tid; e < E; e += kThreads) {
    const int p = edges[2 * e], q = edges[2 * e + 1];
    if (p >= 0 && p < N && q >= 0 && q < N) atomicOr(&s_child[p], 1ull << q);
  }
  if (tid < 64) {
    const bool is_root = tid < N && (level[tid] == 1 || level[tid] == 2);
    const unsigned long long root = __ballot(is_root);
    if (tid == 0) s_root = root;
  }
  // Pascal's triangle row by row; sums that do not fit 64 bits stick at the maximum
  for (int k = tid; k < kBinomN; k += kThreads) s_binom[k] = k == 0 ? 1ull : 0ull;
  __syncthreads();
  for (int n = 1; n < kBinomN; ++n) {
    if (tid < kBinomN) {
      const unsigned long long a = s_binom[(n - 1) * kBinomN + tid], b = tid > 0 ? s_binom[(n - 1) * kBinomN + tid - 1] : 0ull;
      const unsigned long long sum = a + b;
      s_binom[n * kBinomN + tid] = (a == kSat || b == kSat || sum < a) ? kSat : sum;
    }
    __syncthreads();
  }
  if (tid == 0) {
    int o = 0;
    for (int a = 0; a <= h; ++a) {
      s_off[a] = o;
      o += (int)s_binom[h * kBinomN + a];
    }
    s_off[h + 1] = o;
  }
  __syncthreads();
  for (int i = tid; i < kBinomN * kBinomN; i += kThreads) ws->binom[i] = s_binom[i];
  if (tid < 64) ws->child[tid] = s_child[tid];
  if (tid < kLow + 2) ws->off[tid] = tid <= h + 1 ? s_off[tid] : 0;
  const unsigned long long root = s_root;
  if (tid == 0) ws->root = root;
  // Low subsets grouped by size, colexicographic inside a group.  Entry of subset A: the sum of its counts and
  // the word P: above bit h the nodes A does not cover, below it the nodes of A that neither A nor a root
  // level covers.
  const unsigned long long lowall = (1ull << h) - 1ull;
  for (int v = tid; v < (1 << h); v += kThreads) {
    long long s = 0;
    unsigned long long cov = 0ull;
    int r = 0, i = 0;
    for (int m = v; m; m &= m - 1) {
      const int c = __ffs(m) - 1;
      ++i;
      r += (int)s_binom[c * kBinomN + i];
      s += s_cnt[c];
      cov |= s_child[c];
    }
    const int idx = s_off[i] + r;
    SgEntry en;
    en.sum = s;
    en.P = (~cov & ~lowall) | ((unsigned long long)v & ~cov & ~root);
    ws->tab[idx] = en;
    ws->tab_low[idx] = (unsigned short)v;
  }
  if (tid == 0) {
    SgEntry z;
    z.sum = 0;
    z.P = 0ull;
    ws->tab[1 << h] = z;
  }
}

__device__ __forceinline__ bool better(long long s, unsigned long long x, long long s2, unsigned long long x2) {
  return s > s2 || (s == s2 && x < x2);
}

// `ws` is read-only here and every table read has a wavefront-uniform address, so the entries travel through
// the scalar data path and the vector units only see the arithmetic.
__global__ __launch_bounds__(kThreads) void sg_search_kernel(const long long* __restrict__ count, int N, int D,
                                                             const SgWorkspace* __restrict__ ws,
                                                             SgPartial* __restrict__ partial) {
  __shared__ unsigned long long s_child[64];
  __shared__ long long s_cnt[64];
  __shared__ SgPartial s_red[kThreads / 64];

  const int tid = threadIdx.x;
  const int h = N < kLow ? N : kLow;
  const int nH = N - h;
  if (tid < 64) {
    s_child[tid] = ws->child[tid];
    s_cnt[tid] = tid < N ? count[tid] : 0;
  }
  __syncthreads();
  const unsigned long long* __restrict__ binom = ws->binom;
  const SgEntry* __restrict__ tab = ws->tab;
  const unsigned short* __restrict__ tab_low = ws->tab_low;
  const unsigned long long root = ws->root;
  const unsigned long long lowall = (1ull << h) - 1ull;

  const unsigned long long gtid = (unsigned long long)blockIdx.x * kThreads + tid;
  const unsigned long long nth = (unsigned long long)gridDim.x * kThreads;
  long long best = (long long)(1ull << 63);      // below any reachable sum
  unsigned long long bestx = ~0ull;
  unsigned long long n_wave = 0ull;              // connected sets seen by this wavefront (uniform)

  for (int a = 0; a <= h; ++a) {
    const int kB = D - a;
    if (kB < 0 || kB > nH) continue;
    const unsigned long long nb = binom[nH * kBinomN + kB];
    const int nE = (int)binom[h * kBinomN + a];
    const int e0 = ws->off[a];
    const unsigned long long per = (nb + nth - 1) / nth;
    // small groups start at different threads, so that no thread collects the tails of all of them
    const unsigned long long vt = (gtid + (unsigned long long)a * 64ull * 1543ull) % nth;
    const unsigned long long r0 = vt * per;
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
      const unsigned long long vmask = __ballot(valid);
      if (vmask == 0ull) break;                    // ranks ascend in every lane: nothing more in this wavefront
      long long sumB = 0;
      unsigned long long covB = root;
      for (unsigned long long m = valid ? Bh : 0ull; m; m &= m - 1) {
        const int c = h + __ffsll((long long)m) - 1;
        sumB += s_cnt[c];
        covB |= s_child[c];
      }
      const unsigned long long B = Bh << h;        // h <= 12
      const unsigned long long TB = (B | lowall) & ~covB;
      // lanes without work run along on an empty B and get their best back afterwards
      const long long best_in = best;
      const unsigned long long bestx_in = bestx;
      unsigned int n_ok = 0;
      SgEntry next = tab[e0];
      for (int e = 0; e < nE; ++e) {
        const SgEntry en = next;
        next = tab[e0 + e + 1];                    // one entry ahead (the table has a spare entry at its end)
        const bool ok = (en.P & TB) == 0ull;
        n_ok += (unsigned int)__popcll(__ballot(ok) & vmask);
        const long long s = sumB + en.sum;
        if (ok && s >= best) {                     // rare once a good set is known
          const unsigned long long x = B | tab_low[e0 + e];
          if (better(s, x, best, bestx)) {
            best = s;
            bestx = x;
          }
        }
      }
      n_wave += n_ok;
      if (!valid) {
        best = best_in;
        bestx = bestx_in;
      }
      if (r0 + it + 1 < r1) {                      // successor with the same number of bits
        const unsigned long long lo = Bh & (0ull - Bh);
        const unsigned long long rp = Bh + lo;
        Bh = (((rp ^ Bh) >> 2) >> (__ffsll((long long)Bh) - 1)) | rp;
      }
    }
  }

  const int lane = tid & 63, wave = tid >> 6;
  unsigned long long n_conn_hi = lane == 0 ? n_wave : 0ull;
  // workgroup reduction
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
    n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  }
  // two workgroups of 16 wavefronts per compute unit, fewer when there is little to share out
  int blocks = 2 * n_cu < subgraph_search_max_blocks() ? 2 * n_cu : subgraph_search_max_blocks();
  const unsigned long long per_block = 64ull * kThreads;
  if (a.total_sets < (unsigned long long)blocks * per_block)
    blocks = (int)((a.total_sets + per_block - 1) / per_block);
  if (blocks < 1) blocks = 1;
  unsigned char* w = reinterpret_cast<unsigned char*>(a.workspace);
  SgWorkspace* ws = reinterpret_cast<SgWorkspace*>(w);
  SgPartial* partial = reinterpret_cast<SgPartial*>(w + align_up(sizeof(SgWorkspace), 256));
  sg_prepare_kernel<<<1, kThreads, 0, st>>>((const long long*)a.count, a.level, a.N, a.edges, a.E, ws);
  sg_search_kernel<<<blocks, kThreads, 0, st>>>((const long long*)a.count, a.N, a.D, ws, partial);
  sg_final_kernel<<<1, 64, 0, st>>>(partial, blocks, a.D, (unsigned long long*)a.best_mask, (long long*)a.best_sum,
                                    (unsigned long long*)a.n_connected, a.nodes_out);
  return hipGetLastError();
}

}  // namespace spiffy

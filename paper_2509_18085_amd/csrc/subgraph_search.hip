// Offline calibration, part 3 (Alg. 2; App. D.1): the optimal connected subgraph of the candidate graph.
//
//   G' = all node sets Q of size D in which every node is of level 1 or 2 or has a parent in Q
//   G* = argmax over G' of the summed counts; equal sums go to the smaller bit mask sum_q 2^q
//
// Every one of the C(N, D) node sets is tried (the paper's brute force), N <= 64.  A set is a 64-bit mask
// x; with child[p] = mask of the children of p, x is connected iff  x & ~(root | OR_{p in x} child[p]) == 0.
//
// Work split: the nodes are cut into a low part (the h = min(N, 12) lowest nodes), a middle part (the next
// hm <= 11) and a top part (the rest).  A one-workgroup kernel tabulates every subset of the low part (sum of
// counts, a cover word P, the subset) and of the middle part (sum, cover mask, the subset), grouped by size.
// A set is T | M | A.  For each pair of sizes (a, b) = (|A|, |M|) the C(nT, D-a-b) x C(hm, b) pairs (T, M) are
// shared out evenly over all threads of the grid as contiguous ranges; a lane steps through the middle
// entries of its range (one table read per pair), moves to the next top subset with the same-popcount
// successor when they wrap (unranked once at the start), and for every pair runs over all C(h, a) low
// entries of the group.  P holds, above bit h, the nodes A does not cover and, below it, the nodes of A
// that neither A nor a root level covers; with B = T | M and TB = (B | low bits) & ~(root | cover of B) the
// set B | A is connected iff P & TB == 0.  Per tried set: an AND and an AND-OR on 32-bit halves, a zero test,
// an add and a compare against the lane's best (32-bit sums when the counts allow: 64-bit integer adds and
// compares run at a fraction of the 32-bit rate), and the lane's count of connected sets.  Every lane of a
// wavefront needs the same low entry and loop counts are uniform, so those entries are read four at a time
// through the scalar data path, one trip ahead, and lanes diverge only at the end of a range or when a top
// subset changes.  All 64-bit divisions (ranges per thread, starting threads) are done once by the table
// kernel; size pairs with fewer pairs than threads are cut into runs of low entries so that no wavefront is
// left with a lump of work.
#include "kernels.h"

namespace spiffy {

namespace {

constexpr int kLow = 12;                       // tabulated low nodes (2^12 entries)
constexpr int kMid = 11;                       // tabulated middle nodes (2^11 entries)
constexpr int kThreads = 1024;
constexpr int kMaxGroups = 2048;              // (a, b) size pairs, the small ones cut into runs of low entries
constexpr int kBinomN = 65;                    // binomials C(n, k), 0 <= n, k <= 64, saturating
constexpr unsigned long long kSat = ~0ull;

struct __align__(16) SgEntry {
  long long sum;
  unsigned long long P;
};
struct SgGroup {
  unsigned long long npair;                    // (top subset, middle subset) pairs
  unsigned long long per;                      // pairs per thread
  unsigned long long start;                    // thread that takes the first range (groups start at different threads)
  unsigned int nM;                             // middle subsets of this size
  int kT, nE, e0, m0;                          // top nodes in the set; low entries: count, first; first middle entry
};
struct SgWorkspace {                           // device memory, filled by the prepare kernel
  SgEntry tab[(1 << kLow) + 8];                // low subsets grouped by size; spare entries for the read-ahead
  unsigned long long child[64];
  unsigned long long root;
  unsigned long long binom[kBinomN * kBinomN];
  int off[kLow + 2];                           // first table entry of each size group
  unsigned short tab_low[1 << kLow];           // the subset itself
  // middle subsets (nodes h .. h+hm-1), grouped by size: sum of counts, cover (OR of child masks), the subset
  long long mid_sum[1 << kMid];
  unsigned long long mid_cov[1 << kMid];
  unsigned short mid_bits[1 << kMid];
  int mid_off[kMid + 2];
  // the (a, b) size pairs that have sets, with everything the search needs about them
  int n_groups;
  int narrow;                                  // the sum of |count| is below 2^30: sums fit 32-bit arithmetic
  SgGroup groups[kMaxGroups];
};
struct SgPartial {
  long long best_sum;
  unsigned long long best_mask;
  unsigned long long n_connected;
};

// child masks, root mask, binomial table, table of the low subsets; one workgroup
__global__ __launch_bounds__(kThreads) void sg_prepare_kernel(const long long* __restrict__ count,
                                                              const int32_t* __restrict__ level, int N,
                                                              const int32_t* __restrict__ edges, int E, int D,
                                                              unsigned long long n_threads, SgWorkspace* ws) {
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
    const long long c = s_cnt[tid];
    unsigned long long mag = (unsigned long long)(c < 0 ? -c : c);
    bool small = mag < (1ull << 30);
    if (!small) mag = 0ull;
    for (int o = 32; o >= 1; o >>= 1) mag += __shfl_xor(mag, o, 64);
    const bool all_small = __ballot(!small) == 0ull;
    if (tid == 0) ws->narrow = (all_small && mag < (1ull << 30)) ? 1 : 0;
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
  if (tid < 8) {
    SgEntry z;
    z.sum = 0;
    z.P = 0ull;
    ws->tab[(1 << h) + tid] = z;
  }
  // middle subsets, same order
  const int hm = N - h < kMid ? N - h : kMid;
  __shared__ int s_moff[kMid + 2];
  if (tid == 0) {
    int o = 0;
    for (int b = 0; b <= hm; ++b) {
      s_moff[b] = o;
      o += (int)s_binom[hm * kBinomN + b];
    }
    s_moff[hm + 1] = o;
  }
  __syncthreads();
  if (tid < kMid + 2) ws->mid_off[tid] = tid <= hm + 1 ? s_moff[tid] : 0;
  for (int v = tid; v < (1 << hm); v += kThreads) {
    long long sm = 0;
    unsigned long long cov = 0ull;
    int r = 0, i = 0;
    for (int m = v; m; m &= m - 1) {
      const int c = __ffs(m) - 1;
      ++i;
      r += (int)s_binom[c * kBinomN + i];
      sm += s_cnt[h + c];
      cov |= s_child[h + c];
    }
    const int idx = s_moff[i] + r;
    ws->mid_sum[idx] = sm;
    ws->mid_cov[idx] = cov;
    ws->mid_bits[idx] = (unsigned short)v;
  }
  // Size pairs; the 64-bit divisions are done here once instead of by every thread of the search.  Thread
  // a*(hm+1)+b owns pair (a, b).  A pair with fewer (top, middle) pairs than threads gives each of its lanes
  // one pair and all its low entries, a lump that unbalances the wavefronts: it is cut into runs of at least
  // 128 low entries (at most 8: the low table's largest group has 924), each a group of its own with the same
  // pairs and its own starting thread, as many as it takes to give every thread about one unit.
  __shared__ int s_runs[(kLow + 1) * (kMid + 1)], s_first[(kLow + 1) * (kMid + 1) + 1];
  const int nT = N - h - hm;
  const int n_ab = (h + 1) * (hm + 1);
  SgGroup g;
  int runs = 0, nE = 0, ga = 0;
  if (tid < n_ab) {
    ga = tid / (hm + 1);
    const int gb = tid % (hm + 1);
    const int kT = D - ga - gb;
    if (kT >= 0 && kT <= nT) {
      g.nM = (unsigned int)s_binom[hm * kBinomN + gb];
      g.npair = s_binom[nT * kBinomN + kT] * g.nM;
      g.per = (g.npair + n_threads - 1) / n_threads;
      g.kT = kT;
      g.m0 = s_moff[gb];
      nE = (int)s_binom[h * kBinomN + ga];
      runs = 1;
      if (g.npair < n_threads) {
        const unsigned long long fill = n_threads / g.npair;
        runs = (nE + 127) / 128;
        if ((unsigned long long)runs > fill) runs = (int)fill;
        if (runs < 1) runs = 1;
      }
    }
    s_runs[tid] = runs;
  }
  __syncthreads();
  if (tid == 0) {
    int n = 0;
    for (int i = 0; i < n_ab; ++i) {
      s_first[i] = n;
      n += s_runs[i];
    }
    ws->n_groups = n;
  }
  __syncthreads();
  for (int c = 0; c < runs; ++c) {
    const int lo = (int)((long long)nE * c / runs), hi = (int)((long long)nE * (c + 1) / runs);
    const int n = s_first[tid] + c;
    g.e0 = s_off[ga] + lo;
    g.nE = hi - lo;
    g.start = ((unsigned long long)n * 64ull * 1543ull) % n_threads;
    ws->groups[n] = g;
  }
}

__device__ __forceinline__ bool better(long long s, unsigned long long x, long long s2, unsigned long long x2) {
  return s > s2 || (s == s2 && x < x2);
}

// The enumeration proper.  S is the type sums are kept in: 32-bit when the counts allow it (64-bit integer adds
// and compares run at a fraction of the 32-bit rate), else 64-bit.  `ws` is read-only here and every low-table
// read has a wavefront-uniform address, so those entries travel through the scalar data path and the vector
// units only see the arithmetic.
template <typename S>
__device__ __forceinline__ void sg_enumerate(const SgWorkspace* __restrict__ ws, int N, int D, const long long* s_cnt,
                                             const unsigned long long* s_child, unsigned long long gtid,
                                             unsigned long long nth, long long& best_out, unsigned long long& bestx_out,
                                             unsigned long long& n_lane_out) {
  const int h = N < kLow ? N : kLow;
  const int nH = N - h;
  const unsigned long long* __restrict__ binom = ws->binom;
  const SgEntry* __restrict__ tab = ws->tab;
  const unsigned short* __restrict__ tab_low = ws->tab_low;
  const unsigned long long root = ws->root;
  const unsigned long long lowall = (1ull << h) - 1ull;
  constexpr S kLowest = sizeof(S) == 4 ? (S)(1u << 31) : (S)(1ull << 63);      // below any reachable sum
  S best = kLowest;
  unsigned long long bestx = ~0ull;
  unsigned long long n_lane = 0ull;              // connected sets seen by this lane

  const int hm = nH < kMid ? nH : kMid;          // middle nodes h .. h+hm-1
  const int nT = nH - hm;                         // top nodes h+hm .. N-1
  const long long* __restrict__ mid_sum = ws->mid_sum;
  const unsigned long long* __restrict__ mid_cov = ws->mid_cov;
  const unsigned short* __restrict__ mid_bits = ws->mid_bits;

  // One group per (a, b) = (low nodes, middle nodes) in the set.  A lane's unit of work is a pair (top subset,
  // middle subset): the middle part comes from its table, the top part is summed when it changes.
  const int n_groups = ws->n_groups;
  for (int gi = 0; gi < n_groups; ++gi) {
    const SgGroup grp = ws->groups[gi];
    const int kT = grp.kT, nE = grp.nE, e0 = grp.e0, m0 = grp.m0;
    const unsigned long long npair = grp.npair, per = grp.per, nM = grp.nM;
    unsigned long long vt = gtid + grp.start;
    if (vt >= nth) vt -= nth;
    const unsigned long long r0 = vt * per;
    const unsigned long long r1 = r0 + per < npair ? r0 + per : npair;     // my pairs: [r0, r1)
    if (__ballot(r0 < npair) == 0ull) continue;                            // nothing for this wavefront here
    unsigned long long Th = 0ull;                                          // top subset, bit c = node h+hm+c
    unsigned long long mi = 0ull;                                          // middle entry inside its group
    S sumT = 0;
    unsigned long long covT = root;
    auto top_sums = [&]() {
      sumT = 0;
      covT = root;
      for (unsigned long long m = Th; m; m &= m - 1) {
        const int c = h + hm + __ffsll((long long)m) - 1;
        sumT += (S)s_cnt[c];
        covT |= s_child[c];
      }
    };
    if (r0 < npair) {
      // r0 < 2^40 and nM < 2^12: the quotient through one double division, corrected by at most one
      unsigned long long r = (unsigned long long)((double)r0 / (double)nM);
      if (r * nM > r0) --r;
      else if ((r + 1) * nM <= r0) ++r;
      mi = r0 - r * nM;
      int c = nT - 1;
      for (int i = kT; i >= 1; --i) {
        while (binom[c * kBinomN + i] > r) --c;
        Th |= 1ull << c;
        r -= binom[c * kBinomN + i];
        --c;
      }
      top_sums();
    }
    for (unsigned long long it = 0; it < per; ++it) {
      const bool valid = r0 + it < r1;
      const unsigned long long vmask = __ballot(valid);
      if (vmask == 0ull) break;                    // ranks ascend in every lane: nothing more in this wavefront
      const S sumB = sumT + (S)mid_sum[m0 + mi];
      const unsigned long long covB = covT | mid_cov[m0 + mi];
      const unsigned long long B = (Th << (h + hm)) | ((unsigned long long)mid_bits[m0 + mi] << h);
      const unsigned long long TB = (B | lowall) & ~covB;
      const unsigned int TBl = (unsigned int)TB, TBh = (unsigned int)(TB >> 32);   // 64-bit compares are slow: test halves
      auto uncovered = [&](const SgEntry& en) {
        // two instructions on 32-bit halves; the entry is wavefront-uniform (scalar registers).  Left to the
        // compiler this becomes a 64-bit compare, which runs at a fraction of the 32-bit rate.
        unsigned int t;
        asm("v_and_b32 %0, %1, %2\n\tv_and_or_b32 %0, %3, %4, %0"
            : "=&v"(t)
            : "s"((unsigned int)(en.P >> 32)), "v"(TBh), "s"((unsigned int)en.P), "v"(TBl));
        return t != 0u;
      };
      // lanes without work run along on a stale pair and get their best back afterwards
      const S best_in = best;
      const unsigned long long bestx_in = bestx;
      unsigned int n_ok = 0;                       // per lane: the scalar unit is the busier one in this loop
      // four low entries per trip: one 64-byte read through the scalar path, fetched one trip ahead (the table
      // has spare entries at its end), one branch for the rare case that any of the four may beat the lane's best
      auto try_entry = [&](const SgEntry& en, int e) {
        const unsigned long long x = B | tab_low[e0 + e];
        const S s = sumB + (S)en.sum;
        if (!uncovered(en) && (s > best || (s == best && x < bestx))) {
          best = s;
          bestx = x;
        }
      };
      SgEntry n0 = tab[e0], n1 = tab[e0 + 1], n2 = tab[e0 + 2], n3 = tab[e0 + 3];
      int e = 0;
      for (; e + 4 <= nE; e += 4) {
        const SgEntry cur[4] = {n0, n1, n2, n3};
        n0 = tab[e0 + e + 4];
        n1 = tab[e0 + e + 5];
        n2 = tab[e0 + e + 6];
        n3 = tab[e0 + e + 7];
        unsigned long long cand = 0ull;              // lanes for which one of the four may beat their best
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const bool ok = !uncovered(cur[j]);
          n_ok += ok ? 1u : 0u;
          cand |= __ballot(ok) & __ballot(sumB + (S)cur[j].sum >= best);
        }
        if (cand != 0ull) {
#pragma unroll
          for (int j = 0; j < 4; ++j) try_entry(cur[j], e + j);
        }
      }
      {                                              // the last one to three entries of the group
        const SgEntry last[3] = {n0, n1, n2};
#pragma unroll
        for (int j = 0; j < 3; ++j)
          if (e + j < nE) {
            n_ok += !uncovered(last[j]) ? 1u : 0u;
            try_entry(last[j], e + j);
          }
      }
      if (valid) n_lane += n_ok;
      if (!valid) {
        best = best_in;
        bestx = bestx_in;
      }
      if (r0 + it + 1 < r1) {                      // next pair: next middle subset, then the next top subset
        if (++mi == nM) {
          mi = 0ull;
          const unsigned long long lo = Th & (0ull - Th);
          const unsigned long long rp = Th + lo;
          Th = (((rp ^ Th) >> 2) >> (__ffsll((long long)Th) - 1)) | rp;   // same number of bits, next in value
          top_sums();
        }
      }
    }
  }

  best_out = best == kLowest ? (long long)(1ull << 63) : (long long)best;
  bestx_out = bestx;
  n_lane_out = n_lane;
}

__global__ __launch_bounds__(kThreads) void sg_search_kernel(const long long* __restrict__ count, int N, int D,
                                                             const SgWorkspace* __restrict__ ws,
                                                             SgPartial* __restrict__ partial) {
  __shared__ unsigned long long s_child[64];
  __shared__ long long s_cnt[64];
  __shared__ SgPartial s_red[kThreads / 64];

  const int tid = threadIdx.x;
  if (tid < 64) {
    s_child[tid] = ws->child[tid];
    s_cnt[tid] = tid < N ? count[tid] : 0;
  }
  __syncthreads();
  const unsigned long long gtid = (unsigned long long)blockIdx.x * kThreads + tid;
  const unsigned long long nth = (unsigned long long)gridDim.x * kThreads;
  long long best;
  unsigned long long bestx, n_lane;
  if (ws->narrow) sg_enumerate<int>(ws, N, D, s_cnt, s_child, gtid, nth, best, bestx, n_lane);
  else sg_enumerate<long long>(ws, N, D, s_cnt, s_child, gtid, nth, best, bestx, n_lane);

  const int lane = tid & 63, wave = tid >> 6;
  unsigned long long n_conn_hi = n_lane;
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
  // compute units of the current device (asked once per device id; the answer decides only how the work is cut)
  static std::atomic<int> cu_of_device[64];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  int n_cu = cu_of_device[dev & 63].load(std::memory_order_acquire);
  if (n_cu == 0) {
    e = hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return e;
    if (n_cu <= 0) n_cu = 256;
    cu_of_device[dev & 63].store(n_cu, std::memory_order_release);
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
  sg_prepare_kernel<<<1, kThreads, 0, st>>>((const long long*)a.count, a.level, a.N, a.edges, a.E, a.D,
                                            (unsigned long long)blocks * kThreads, ws);
  sg_search_kernel<<<blocks, kThreads, 0, st>>>((const long long*)a.count, a.N, a.D, ws, partial);
  sg_final_kernel<<<1, 64, 0, st>>>(partial, blocks, a.D, (unsigned long long*)a.best_mask, (long long*)a.best_sum,
                                    (unsigned long long*)a.n_connected, a.nodes_out);
  return hipGetLastError();
}

}  // namespace spiffy

// Drafting from the current distribution and pruning of the draft graph (Sec. 4.4.2, 4.4.4) on one
// wavefront.
//
//   token position rank i  = position in the sort of the masked positions by confidence, most confident
//                            first, equal confidences to the lower position (first relation of Sec. 4.4.2)
//   vocabulary rank j      = column of the per-position top-K lists
//   draft formula m        = set {(i, j)}: block m is the current block with c_ij unmasked at the position of
//                            rank i (Sec. 4.4.3); a formula that names a rank beyond the masked positions, a
//                            vocabulary rank beyond K, or one position twice cannot be built
//   localScore, childScore, score: geometric means (Sec. 4.4.4), computed as exp2 of mean log2;
//                            children = buildable children in the edge list; no children -> local score
//   the d_star best scores are kept (equal scores to the lower node), node 0 always; surviving edges are
//   renumbered to the kept list, in their original order
//
// Lane m stands for node m (at most 64 nodes, like the acceptance walk); the O(B^2) counting rank and the
// O(E) scans are spread over the lanes.
#include "kernels.h"

namespace spiffy {

namespace {

constexpr int kMaxB = 4096;

__global__ __launch_bounds__(64) void draft_prune_kernel(DraftPruneArgs a) {
  __shared__ int order[kMaxB];              // order[i-1] = position of rank i
  __shared__ float s_local[64], s_score[64];
  __shared__ unsigned char s_ok[64];
  __shared__ unsigned long long s_kids[64];
  __shared__ int s_pos[64];                 // node -> index in the kept list, or -1
  __shared__ int s_nmasked;
  const int lane = threadIdx.x;
  const int D = a.D, B = a.B, K = a.K;

  // ---- token position ranks by counting ------------------------------------------------------------
  if (lane == 0) s_nmasked = 0;
  s_kids[lane] = 0ull;
  __syncthreads();
  for (int b = lane; b < B; b += 64) {
    if (a.state[b] != a.mask_id) continue;
    const float pb = a.topk_probs[(size_t)b * K];
    int beat = 0;
    for (int c = 0; c < B; ++c) {
      if (a.state[c] != a.mask_id) continue;
      const float pc = a.topk_probs[(size_t)c * K];
      beat += (pc > pb || (pc == pb && c < b)) ? 1 : 0;
    }
    order[beat] = b;
    atomicAdd(&s_nmasked, 1);
  }
  __syncthreads();
  const int n_masked = s_nmasked;

  // ---- every block starts as a copy of the current one ---------------------------------------------
  for (int e = lane; e < (D + 1) * B; e += 64) a.drafts[e] = a.state[e % B];

  // ---- formulas: validate, then local score -------------------------------------------------------
  bool ok = false;
  float loc = __builtin_nanf("");
  int f0 = 0, f1 = 0;
  if (lane >= 1 && lane <= D) {
    f0 = a.formula_offsets[lane - 1];
    f1 = a.formula_offsets[lane];
    ok = f0 >= 0 && f1 > f0 && f1 <= a.nnz;
    float sum_log = 0.f;
    for (int e = f0; ok && e < f1; ++e) {
      const int i = a.formula_pairs[2 * e], j = a.formula_pairs[2 * e + 1];
      if (i < 1 || i > n_masked || j < 1 || j > K) { ok = false; break; }
      for (int e2 = f0; e2 < e; ++e2)
        if (a.formula_pairs[2 * e2] == i) ok = false;        // the same position twice
      if (ok) sum_log += __log2f(a.topk_probs[(size_t)order[i - 1] * K + (j - 1)]);
    }
    if (ok) loc = exp2f(sum_log / (float)(f1 - f0));
  } else if (lane == 0) {
    ok = true;
  }
  s_ok[lane] = ok ? 1 : 0;
  s_local[lane] = loc;
  __syncthreads();     // copies of the current block are in place before any lane writes its tokens
  if (ok && lane >= 1) {
    for (int e = f0; e < f1; ++e) {
      const int i = a.formula_pairs[2 * e], j = a.formula_pairs[2 * e + 1];
      const int b = order[i - 1];
      a.drafts[(size_t)lane * B + b] = a.topk_tokens[(size_t)b * K + (j - 1)];
    }
  }

  // ---- children sets, child score, score ----------------------------------------------------------------
  for (int e = lane; e < a.E; e += 64) {
    const int p = a.edges[2 * e], c = a.edges[2 * e + 1];
    if (p >= 1 && p <= D && c >= 1 && c <= D && s_ok[c]) atomicOr(&s_kids[p], 1ull << c);
  }
  __syncthreads();
  float sc = __builtin_nanf("");
  if (ok && lane >= 1) {
    unsigned long long kids = s_kids[lane];
    if (kids) {
      float sum_log = 0.f;
      int n = 0;
      while (kids) {
        const int c = __ffsll((long long)kids) - 1;
        kids &= kids - 1;
        sum_log += __log2f(s_local[c]);
        ++n;
      }
      const float child = exp2f(sum_log / (float)n);
      sc = sqrtf(loc * child);
    } else {
      sc = loc;
    }
  }
  if (lane <= D) {
    a.buildable[lane] = ok ? 1 : 0;
    a.local[lane] = loc;
    a.score[lane] = sc;
  }

  // ---- keep the d_star best ---------------------------------------------------------------------------
  s_score[lane] = sc;
  __syncthreads();
  bool keep = lane == 0;
  if (ok && lane >= 1) {
    int beat = 0;
    for (int m = 1; m <= D; ++m) {
      const float other = s_score[m];
      beat += (s_ok[m] && (other > sc || (other == sc && m < lane))) ? 1 : 0;
    }
    keep = beat < a.d_star;
  }
  const unsigned long long kept_mask = __ballot(keep);
  const int my_pos = __popcll(kept_mask & ((1ull << lane) - 1ull));
  s_pos[lane] = keep ? my_pos : -1;
  const int n_kept = __popcll(kept_mask);
  if (keep) a.kept[my_pos] = lane;
  __syncthreads();
  // kept blocks, in node order: a copy of the current block, then the formula's tokens
  for (int r = 0; r < 64; ++r) {
    if (!((kept_mask >> r) & 1ull)) continue;
    const int dst = s_pos[r];
    for (int b = lane; b < B; b += 64) a.states_out[(size_t)dst * B + b] = a.state[b];
  }
  __syncthreads();
  if (keep && lane >= 1) {
    for (int e = f0; e < f1; ++e) {
      const int i = a.formula_pairs[2 * e], j = a.formula_pairs[2 * e + 1];
      const int b = order[i - 1];
      a.states_out[(size_t)my_pos * B + b] = a.topk_tokens[(size_t)b * K + (j - 1)];
    }
  }
  // surviving edges, original order, renumbered
  int n_out = 0;
  for (int e0 = 0; e0 < a.E; e0 += 64) {
    const int e = e0 + lane;
    bool live = false;
    int p = 0, c = 0;
    if (e < a.E) {
      p = a.edges[2 * e];
      c = a.edges[2 * e + 1];
      live = p >= 0 && p <= D && c >= 0 && c <= D && s_pos[p] >= 0 && s_pos[c] >= 0;
    }
    const unsigned long long m = __ballot(live);
    if (live) {
      const int o = n_out + __popcll(m & ((1ull << lane) - 1ull));
      a.edges_out[2 * o] = s_pos[p];
      a.edges_out[2 * o + 1] = s_pos[c];
    }
    n_out += __popcll(m);
  }
  if (lane == 0) {
    a.counts[0] = n_kept;
    a.counts[1] = n_out;
  }
}

}  // namespace

hipError_t launch_draft_prune(const DraftPruneArgs& a, hipStream_t st) {
  if (a.B > kMaxB || a.D > 63) return hipErrorInvalidValue;
  draft_prune_kernel<<<1, 64, 0, st>>>(a);
  return hipGetLastError();
}

}  // namespace spiffy

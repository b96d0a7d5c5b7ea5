// Acceptance walk over the draft graph (Alg. 1 step 5, children by Eqs. (4)-(6)) on one
// wavefront: lane c stands for node c, the children of every node are a 64-bit mask in LDS,
// "does draft c equal the current target" is evaluated by all lanes at once and the lowest
// matching child is picked with a ballot.
#include "kernels.h"

namespace spiffy {

__global__ __launch_bounds__(64) void graph_accept_kernel(const int32_t* __restrict__ edges, int E,
                                                          const int32_t* __restrict__ draft,
                                                          const int32_t* __restrict__ target, int G, int B, int root,
                                                          spiffy_accept_result* __restrict__ res,
                                                          int32_t* __restrict__ state) {
  __shared__ unsigned long long child[64];
  __shared__ int bad;
  const int lane = threadIdx.x;
  child[lane] = 0ull;
  if (lane == 0) bad = 0;
  __syncthreads();
  for (int e = lane; e < E; e += 64) {
    const int p = edges[2 * e], c = edges[2 * e + 1];
    if (p < 0 || p >= G || c < 0 || c >= G) {
      atomicOr(&bad, 1);
    } else {
      atomicOr(&child[p], 1ull << c);
    }
  }
  __syncthreads();
  int cur = root, depth = 0;
  unsigned long long seen = 1ull << root;
  while (depth < G) {                      // at most G-1 moves: every move marks a new node
    const unsigned long long cand = child[cur] & ~seen;
    bool match = lane < G && ((cand >> lane) & 1ull);
    if (match) {
      const int32_t* dr = draft + (size_t)lane * B;
      const int32_t* tg = target + (size_t)cur * B;
      for (int b = 0; b < B; ++b) {
        if (dr[b] != tg[b]) { match = false; break; }
      }
    }
    const unsigned long long hit = __ballot(match);
    if (hit == 0ull) break;
    cur = __ffsll((long long)hit) - 1;     // lowest matching node id
    seen |= 1ull << cur;
    ++depth;
  }
  if (lane == 0) {
    res->node = cur;
    res->depth = depth;
    res->n_steps = depth + 1;
    res->flags = bad ? 1 : 0;
  }
  if (state) {
    for (int b = lane; b < B; b += 64) state[b] = target[(size_t)cur * B + b];
  }
}

hipError_t launch_graph_accept(const int32_t* edges, int E, const int32_t* draft, const int32_t* target, int G,
                               int B, int root, spiffy_accept_result* res, int32_t* state, hipStream_t st) {
  graph_accept_kernel<<<1, 64, 0, st>>>(edges, E, draft, target, G, B, root, res, state);
  return hipGetLastError();
}

}  // namespace spiffy

// Launchers implemented by the kernel translation units; called only by api.hip.
// Every launcher enqueues on `st` and returns hipGetLastError() of its launches.
#pragma once
#include "common.h"

namespace spiffy {

// ---- generic (any shape, T = float or bf16 storage, fp32 math) ---------------------------------
hipError_t launch_embed(int dtype, const void* w_embed, const int32_t* tokens, int M, int d, int V,
                        void* out, hipStream_t st);
// out[r,:] = rmsnorm(x[src(r),:]) * gain, src(r) = row_idx ? row_idx[r] : r, rows r < *n_rows_dev
// (or < M when n_rows_dev is NULL).
hipError_t launch_rmsnorm(int dtype, const void* x, const void* gain, float eps, int M, int d,
                          const int32_t* row_idx, const int32_t* n_rows_dev, void* out, hipStream_t st);
hipError_t launch_gemm_generic(int dtype, int epi, const GemmArgs& a, hipStream_t st);
// a_out[r,:] = a[row_idx[r],:] and b_out[r,:] = b[row_idx[r],:] for r < *count; row sizes in bytes, multiples of 16
hipError_t launch_scatter_rows(const void* in, size_t row_bytes, const int32_t* row_idx, const int32_t* count, int M,
                               void* out, hipStream_t st);     // out[row_idx[r],:] = in[r,:] for r < *count
hipError_t launch_gather_rows2(const void* a, size_t a_row_bytes, const void* b, size_t b_row_bytes,
                               const int32_t* row_idx, const int32_t* count, int M, void* a_out, void* b_out,
                               hipStream_t st);

struct AttnArgs {
  const void* qkv;       // [M, (Hq+2Hkv)*hd]: q | k | v columns, not yet rotated
  const void* prefix_k;  // [Hkv,P,hd]
  const void* prefix_v;
  void* out;             // [M, Hq*hd]
  void* partial;         // MFMA path: split partials (fp32)
  int G, B, Hq, Hkv, hd, P, pos0;
  int ldp;               // rows allocated per KV head in prefix_k / prefix_v (0 = P)
  int S;                 // dual cache: rows P+B .. P+B+S-1 of the same arrays hold the tokens after the block
  int own;               // 1: every state also attends to its own B rows (keys / values from qkv); 0: cache rows only
  float rope_base;
  int rope_ready;        // MFMA path: the rotary table at the start of `partial` is already filled
};
hipError_t launch_attn_generic(int dtype, const AttnArgs& a, hipStream_t st);
// Prefix-cache extension (Sec. 3.1): the K rows (rotated at positions pos0 .. pos0+B-1) and V rows of the
// first B rows of the fused qkv activations go to rows P .. P+B-1 of every KV head of the cache
// ([Hkv][ldp][hd]).  Must run before the attention of the same layer reads the cache only up to row P.
// rows 0 .. B-1 of the appended range come from qkv rows 0 .. B0-1 and B0+skip .. (B0 <= 0: one run of B rows).
// tab_a / tab_b: optional rotary tables [hd/2][n] (cos, sin) for the first B0 rows (n = B0) and for the rest
// (n = B - B0), as the attention kernels use them; NULL = the same values computed in the kernel.
hipError_t launch_kv_append(int dtype, const void* qkv, int Hq, int Hkv, int hd, int B, int pos0, float rope_base,
                            void* cache_k, void* cache_v, int P, int ldp, hipStream_t st, int B0 = 0, int skip = 0,
                            const void* tab_a = nullptr, const void* tab_b = nullptr);

// masked-row list: row_idx[0..count) = flattened (g,b) with mask set, ascending; *count.
hipError_t launch_compact_rows(const int32_t* tokens, const uint8_t* mask, int mask_id, int M,
                               int32_t* row_idx, int32_t* count, hipStream_t st);
// per compacted row r: summary over the whole vocabulary of scale * (n[r,:] . w_vocab[v,:])
hipError_t launch_lmhead_generic(int dtype, const void* n, const void* w_vocab, int d, int V,
                                 float scale, const int32_t* count, int M, TopPartial* row_top,
                                 hipStream_t st);
// merge n_part partials per row; part is [n_part][m_cap]; tmp is [kLmheadCombineSlices][m_cap] scratch
constexpr int kLmheadCombineSlices = 16;
hipError_t launch_lmhead_combine(const TopPartial* part, int n_part, int m_cap, const int32_t* count, int M,
                                 TopPartial* tmp, TopPartial* row_top, hipStream_t st);
// scatter row summaries to [G,B] outputs, apply threshold / force_one, build next states
hipError_t launch_head_finalize(const TopPartial* row_top, const int32_t* row_idx, const int32_t* count,
                                const int32_t* tokens, const uint8_t* mask, int mask_id, int G, int B,
                                float threshold, int force_one, int32_t* argmax, float* conf,
                                uint8_t* unmask, float* margin, int32_t* target, hipStream_t st);

// top-K tokens of the accepted node's rows from what the head pass left behind; all pointers device memory
struct HeadTopkArgs {
  int dtype;
  const void* nf;                 // gathered normalised rows [count][d]
  const void* w_vocab;            // [V][d]
  int d, V;
  float scale;
  const TopPartial* part;         // [n_part][m_cap] per-128-token summaries (MFMA head), or unused
  int n_part, m_cap;
  const TopPartial* row_top;      // [count] merged summaries
  const int32_t* row_idx;         // [count] flattened (g,b) of every compacted row, ascending
  const int32_t* count;
  const int32_t* tokens;          // [G*B] block tokens
  const spiffy_accept_result* result;   // node read on the device; NULL: use `node`
  int node, G, B, K;
  float* cand_val;                // [B][SPIFFY_MAX_TOPK][SPIFFY_MAX_TOPK]
  int32_t* cand_idx;
  int32_t* out_tokens;            // [B][K]
  float* out_probs;               // [B][K]
};
hipError_t launch_head_topk(const HeadTopkArgs& a, hipStream_t st);

// drafting + pruning (one wavefront); all pointers device memory
struct DraftPruneArgs {
  const int32_t* state;            // [B]
  const int32_t* topk_tokens;      // [B][K]
  const float* topk_probs;         // [B][K], column 0 = confidence
  const int32_t* formula_offsets;  // [D+1]
  const int32_t* formula_pairs;    // [nnz][2]: (i, j), 1-based
  const int32_t* edges;            // [E][2] over nodes 0..D
  int32_t* drafts;                 // [D+1][B]
  uint8_t* buildable;              // [D+1]
  float* local;                    // [D+1]
  float* score;                    // [D+1]
  int32_t* kept;                   // [d_star+1]
  int32_t* states_out;             // [d_star+1][B]
  int32_t* edges_out;              // [E][2]
  int32_t* counts;                 // [2]: kept nodes, surviving edges
  int B, K, D, nnz, E, d_star, mask_id;
};
hipError_t launch_draft_prune(const DraftPruneArgs& a, hipStream_t st);

hipError_t launch_graph_accept(const int32_t* edges, int E, const int32_t* draft, const int32_t* target,
                               int G, int B, int root, spiffy_accept_result* res, int32_t* state,
                               hipStream_t st);

// ---- MFMA (bf16, gfx950) -----------------------------------------------------------------------
bool mfma_gemm_supported(int epi, const GemmArgs& a);
hipError_t launch_gemm_mfma(int epi, const GemmArgs& a, hipStream_t st);
// what launch_gemm_mfma launches for a shape: tile rows x columns (SWIGLU: a tile of w columns holds w/2 features), the
// range of output columns (features) and the number of workgroups of each launch
struct GemmPlan {
  int n_parts;
  struct { int bm, bn, col0, ncols, workgroups; } part[2];
};
GemmPlan plan_gemm_mfma(int epi, int M, int N, int ksplit);
int mfma_lmhead_partials_per_row(int V);
int mfma_ksplit(int N, int K);          // K slices used for a [M,K]x[N,K] projection with residual (depends on N, K only)
// out = R + sum of the K-slice partials P[ksplit][M][N] (fixed order); if normed != NULL also RMSNorm(out)*gain.
// n_rows_dev (optional): only rows below *n_rows_dev exist; out_rows (optional): row m of the result goes to row
// out_rows[m] of `out` (the partials, R and normed keep row m).
hipError_t launch_splitk_reduce(const float* P, int ksplit, const void* R, void* out, const void* gain, float eps,
                                void* normed, int M, int N, hipStream_t st, const int32_t* n_rows_dev = nullptr,
                                const int32_t* out_rows = nullptr);
bool mfma_attn_supported(const AttnArgs& a);
size_t mfma_attn_partial_bytes(int G, int B, int Hq, int hd, int P);
hipError_t launch_attn_mfma(const AttnArgs& a, hipStream_t st);
const void* launch_rope_table(void* partial, int B, int pos0, float rope_base, hipStream_t st);   // head_dim 128 only
hipError_t launch_attn_mfma_pair(const AttnArgs& a, const AttnArgs& b, hipStream_t st);   // two problems, one launch

// Calibration, part 3 (Alg. 2; App. D.1): best connected node set of size D.  All pointers device memory.
struct SubgraphArgs {
  const int64_t* count;          // [N]
  const int32_t* level;          // [N], 1-based
  const int32_t* edges;          // [E][2] (parent, child)
  int N, E, D;
  unsigned long long total_sets; // C(N, D), for the launch size
  uint64_t* best_mask;
  int64_t* best_sum;
  uint64_t* n_connected;
  int32_t* nodes_out;            // [D] or NULL
  void* workspace;
};
size_t subgraph_search_workspace_bytes();
hipError_t launch_subgraph_search(const SubgraphArgs& a, hipStream_t st);

}  // namespace spiffy

/*
 * spiffy.h - C ABI of the MI355X (gfx950) draft-graph verification library.
 *
 * One verification step of Spiffy (arxiv 2509.18085): G states of one B-token block (node 0 is
 * the current true state X_k(t), the others are draft blocks, Sec. 4.2) go through ONE forward
 * pass (Sec. 4.3, Eqs. (2),(3)); each state attends to the shared cached context and to itself
 * only (Fig. 4); every masked position is reduced to top-1 token, top-1 probability and the
 * threshold-unmask decision (Alg. 1 steps 1-4, threshold rule of Sec. 3.1); then the draft graph
 * (Eqs. (4)-(6)) is walked to the deepest accepted state (Alg. 1 step 5).
 *
 * Conventions for every call
 *   - Kernel choice is by shape: bf16 with head_dim 128, d % 128 == 0, ffn % 64 == 0 runs the MFMA
 *     kernels (LM head: d % 64 == 0); anything else runs shape-agnostic fp32-math kernels.  The
 *     choice depends on the arguments of the call only (no environment variable, no global state).
 *     On the MFMA kernels a layer takes d <= 16384 (a row in fp32 is kept in 64 KB of on-chip memory by
 *     the reduction behind the output and down projections); wider models get SPIFFY_ESHAPE.
 *   - All data pointers are DEVICE pointers owned by the caller unless a parameter says "host".
 *     The library never frees or keeps them.  Structs (cfg, weights, prefix) are HOST structs
 *     that hold device pointers.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue work
 *     and return; they never synchronise and never allocate.  Scratch memory comes from the
 *     caller: `workspace` of at least spiffy_workspace_bytes(...) bytes, 256-byte aligned.
 *   - Matrices are row-major.  Weights are [out, in].  dtype (SPIFFY_BF16 / SPIFFY_F32) is the
 *     storage type of weights, hidden states and KV; accumulation is fp32 in both cases.
 *   - Outputs are fully overwritten; inputs are never modified; hidden_in == hidden_out is allowed.
 *   - Errors are return codes; every argument check happens on the host before any launch, so
 *     a failing call launches nothing.  Null required pointer, G<1, B<1, bad threshold, bad root
 *     -> SPIFFY_EINVAL; unsupported shape -> SPIFFY_ESHAPE; pointer not 16-byte aligned ->
 *     SPIFFY_EALIGN; workspace too small -> SPIFFY_EWORKSPACE; a failed launch -> SPIFFY_EDEVICE.
 */
#ifndef SPIFFY_H
#define SPIFFY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SPIFFY_OK = 0,
  SPIFFY_EINVAL = -1,
  SPIFFY_ESHAPE = -2,
  SPIFFY_EALIGN = -3,
  SPIFFY_EWORKSPACE = -4,
  SPIFFY_EDEVICE = -5,
  SPIFFY_ELIMIT = -6   /* spiffy_decode_head_static only: the call needs more scratch than the library holds */
} spiffy_status;

enum { SPIFFY_BF16 = 0, SPIFFY_F32 = 1 };

/* Limits checked by the host: G <= SPIFFY_MAX_G for the walk (one node per lane of a 64-wide
 * wavefront, 64-bit child masks); rows G*B <= SPIFFY_MAX_ROWS. */
#define SPIFFY_MAX_G 64
#define SPIFFY_MAX_TOPK 8   /* vocabulary ranks per position that spiffy_head_topk can return */
#define SPIFFY_MAX_ROWS 16384

typedef struct {
  int32_t d;           /* model width */
  int32_t n_q_heads;   /* query heads Hq */
  int32_t n_kv_heads;  /* key/value heads Hkv, divides Hq */
  int32_t head_dim;    /* hd, even, <= 256 */
  int32_t ffn;         /* SwiGLU width F */
  int32_t vocab;       /* V */
  int32_t mask_id;     /* token id of MASK (Sec. 3.1) */
  int32_t dtype;       /* SPIFFY_BF16 or SPIFFY_F32 */
  float rms_eps;
  float rope_base;
} spiffy_model_cfg;

/* One transformer layer.  wq [Hq*hd, d], wk/wv [Hkv*hd, d], wo [d, Hq*hd], w_gate/w_up [F, d],
 * w_down [d, F], norm1/norm2 [d]; bq/bk/bv optional biases ([Hq*hd], [Hkv*hd], [Hkv*hd]),
 * NULL = none. */
typedef struct {
  const void *wq, *wk, *wv, *wo;
  const void *w_gate, *w_up, *w_down;
  const void *norm1, *norm2;
  const void *bq, *bk, *bv;
} spiffy_layer_weights;

/* Cached context of one layer (prefix caching, Sec. 3.1; dual cache, Sec. 4.3 / App. A.2): k and v are each
 * [Hkv, capacity, hd] and row j holds sequence position j; k rows are already rotated at their positions.
 * Rows 0 .. P-1 are the prefix.  P may be 0 (then, with S = 0, k and v may be NULL).  With S > 0 rows
 * P+B .. P+B+S-1 hold the S tokens after the block (B = the block size of the call): every block, true or
 * draft, attends to prefix, itself and suffix (Fig. 4).  Rows P .. P+B-1, the slot of the block being decoded,
 * are never read; spiffy_commit_block writes them. */
typedef struct {
  const void *k, *v;
  int32_t P;
  int32_t capacity; /* rows allocated per KV head (the stride between heads); 0 means P.  A cache that
                     * spiffy_commit_block extends, or that holds a suffix, has capacity >= P + B + S. */
  int32_t S;        /* suffix rows; 0 = prefix cache only */
} spiffy_prefix_kv;

/* Result of the walk: accepted node id, number of accepted drafts (depth), decode steps covered
 * by this forward (depth+1), and a flag word (bit 0: an edge endpoint was outside [0,G) and
 * that edge was ignored). */
typedef struct {
  int32_t node, depth, n_steps, flags;
} spiffy_accept_result;

const char *spiffy_status_str(int status);

/* 1 if the cfg/B combination runs on the MFMA kernels, 0 if on the generic kernels, <0 = status. */
int spiffy_uses_mfma(const spiffy_model_cfg *cfg, int32_t B);

/* Bytes of caller-provided scratch needed by verify_layer / decode_head / verify_step for up to
 * G states of B tokens and up to P_max cached rows per layer (prefix and suffix together, P + S).
 * 0 on invalid arguments. */
size_t spiffy_workspace_bytes(const spiffy_model_cfg *cfg, int32_t G, int32_t B, int32_t P_max);

/* Token embedding of the G states: hidden_out[g,b,:] = w_embed[block_tokens[g,b],:]; masked
 * positions carry the MASK id's row (Sec. 3.1).  w_embed [V,d]; block_tokens [G,B] int32 with
 * values in [0,V) (out-of-range ids are clamped); hidden_out [G,B,d]. */
int spiffy_embed(const spiffy_model_cfg *cfg, const void *w_embed, const int32_t *block_tokens,
                 int32_t G, int32_t B, void *hidden_out, void *stream);

/* One transformer layer over the G states in one pass (Sec. 4.3; mask of Fig. 4 is implicit:
 * the rows of state g attend to the P cached keys and to the B keys of state g, bidirectionally,
 * and to nothing else).  pre-norm RMSNorm, QKV projection (+bias), rotary embedding at positions
 * pos0..pos0+B-1 for every g (pos0 = P normally), attention, output projection + residual,
 * RMSNorm, SwiGLU FFN + residual.  hidden_in, hidden_out [G,B,d]. */
int spiffy_verify_layer(const spiffy_model_cfg *cfg, const spiffy_layer_weights *w,
                        const spiffy_prefix_kv *prefix, const void *hidden_in, int32_t G, int32_t B,
                        int32_t pos0, void *hidden_out, void *workspace, size_t workspace_bytes,
                        void *stream);

/* The last layer of a step.  Only masked positions are decoded (Alg. 1 steps 1-4 rank and fill masked positions
 * only; Sec. 3.1), so behind the attention, where every row of a state still supplies keys and values to the
 * others, only the rows of masked positions are computed: output projection, FFN and residuals run on those rows.
 * mask [G,B] uint8 (1 = masked) may be NULL, then mask = (block_tokens == cfg.mask_id).  hidden_out rows of
 * masked positions receive exactly what spiffy_verify_layer writes there (bit for bit: a row's arithmetic does
 * not depend on the rows computed with it); the other rows of hidden_out are not written.  Other arguments,
 * workspace and errors as for spiffy_verify_layer.  spiffy_verify_step runs its last layer this way when
 * the caller passes hidden_out = NULL. */
int spiffy_verify_layer_last(const spiffy_model_cfg *cfg, const spiffy_layer_weights *w,
                             const spiffy_prefix_kv *prefix, const void *hidden_in, const int32_t *block_tokens,
                             const uint8_t *mask, int32_t G, int32_t B, int32_t pos0, void *hidden_out,
                             void *workspace, size_t workspace_bytes, void *stream);

/* LM head reduced to decisions (Alg. 1 steps 1-4 with the threshold rule of Sec. 3.1), for all G
 * states.  mask [G,B] uint8 (1 = masked) may be NULL, then mask = (block_tokens == cfg.mask_id).
 * For every masked position: logits = logit_scale *
 * RMSNorm(hidden) * w_vocab^T over the whole vocabulary, argmax = lowest-index top-1 token,
 * conf = its softmax probability, top2_margin = top-1 logit minus second logit,
 * unmask = conf > threshold (strict, fp32).  If force_one != 0 and a state has masked positions
 * but none passes, its highest-conf masked position (lowest index on ties) is unmasked.
 * target_states = Next(state): the state with its unmasked positions filled by argmax.
 * At positions that are not masked: argmax = the token, conf = 0, unmask = 0, margin = +inf.
 * Logits are never written to memory.  final_norm [d]; w_vocab [V,d];
 * argmax/target_states [G,B] int32; conf/top2_margin [G,B] float; unmask [G,B] uint8.
 * top2_margin and target_states may be NULL.  The bf16 matrix-core head (d % 64 == 0) addresses the vocabulary
 * matrix with 32-bit byte offsets and keeps at most 2048 chunk summaries per row: vocab * d * 2 >= 2^32 or
 * vocab > 262144 -> SPIFFY_ESHAPE. */
int spiffy_decode_head(const spiffy_model_cfg *cfg, const void *hidden, const void *final_norm,
                       const void *w_vocab, const int32_t *block_tokens, const uint8_t *mask,
                       int32_t G, int32_t B, float threshold, float logit_scale, int32_t force_one, int32_t *argmax,
                       float *conf, uint8_t *unmask, float *top2_margin, int32_t *target_states,
                       void *workspace, size_t workspace_bytes, void *stream);

/* spiffy_decode_head for callers that cannot allocate and have no workspace to pass: code recorded into a HIP
 * graph, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (without the workspace), same
 * kernels and bit-identical outputs; the scratch is a device array of SPIFFY_STATIC_SCRATCH_BYTES that the library
 * holds on every GPU it runs on until the process ends.  The call allocates nothing and frees nothing.  Limits:
 * G*B <= SPIFFY_STATIC_MAX_ROWS (the paper's operating point, four states of a 32-token block, Sec. 5) and a head
 * scratch (gathered rows G*B x d, one 16-byte summary per row and 128-token chunk of the vocabulary) within the
 * array: bf16 with d <= 8192 and vocab <= 262144 always fits.  Anything larger returns SPIFFY_ELIMIT before any
 * launch.  All calls on one GPU share that GPU's array (each call overwrites what the last one left; nothing in it
 * has to be cleared), so calls that overlap on one GPU, on different streams or from different threads, race:
 * serialise them.  The first call on a device looks up the array's address (not inside a graph capture). */
#define SPIFFY_STATIC_SCRATCH_BYTES (8u << 20)
#define SPIFFY_STATIC_MAX_ROWS 128
int spiffy_decode_head_static(const spiffy_model_cfg *cfg, const void *hidden, const void *final_norm,
                              const void *w_vocab, const int32_t *block_tokens, const uint8_t *mask,
                              int32_t G, int32_t B, float threshold, float logit_scale, int32_t force_one,
                              int32_t *argmax, float *conf, uint8_t *unmask, float *top2_margin,
                              int32_t *target_states, void *stream);

/* The projection GEMM that verify_layer is made of, exposed for unit tests and for kernel-level
 * timing.  A [M,K], weights [N,K] row-major, C [M,N] (SPIFFY_GEMM_SWIGLU: W0 = gate, W1 = up,
 * both [N,K], C = silu(A W0^T) * (A W1^T)); SPIFFY_GEMM_RESID: C = R + A W0^T with R [M,N];
 * SPIFFY_GEMM_STORE: C = A W0^T.  bf16 with K % 64 == 0 and N % 64 == 0 (SWIGLU: N % 32 == 0)
 * runs the MFMA kernel, anything else the generic kernel.  workspace (256-byte aligned, at least
 * 4*M*N*sizeof(float) bytes) may be NULL; with it, SPIFFY_GEMM_RESID slices K exactly as
 * verify_layer does for its output and down projections (the slice count depends on N and K only). */
enum { SPIFFY_GEMM_STORE = 0, SPIFFY_GEMM_RESID = 1, SPIFFY_GEMM_SWIGLU = 2 };
int spiffy_gemm(int32_t dtype, int32_t epilogue, const void *A, const void *W0, const void *W1,
                const void *R, void *C, int32_t M, int32_t N, int32_t K, void *workspace,
                size_t workspace_bytes, void *stream);

/* How spiffy_gemm / verify_layer would launch a bf16 projection of M rows, N output columns (SPIFFY_GEMM_SWIGLU: N
 * features) and inner size K on the MFMA kernel: host arithmetic only, nothing is launched and no device is touched.
 * The choice is scheduling: the order of the K sum of an output element does not depend on it (Sec. 4.3: states of one
 * step are independent rows), only k_slices does, and k_slices depends on (N, K) alone.  with_workspace: as for
 * spiffy_gemm, SPIFFY_GEMM_RESID slices K only when scratch is given.  Returns SPIFFY_ESHAPE for shapes the MFMA
 * kernel does not take (see spiffy_gemm), SPIFFY_EINVAL for a NULL plan or an unknown epilogue. */
typedef struct {
  int32_t n_launches;       /* 1, or 2 when the columns are split into a wide-tile part and a rest */
  int32_t k_slices;         /* K slices (partial sums in fp32 scratch, reduced in a fixed order) */
  struct {
    int32_t tile_rows, tile_cols;   /* SWIGLU: a tile of w columns holds w/2 features (gate and up interleaved) */
    int32_t col0, n_cols;           /* output columns (features) [col0, col0 + n_cols) */
    int32_t workgroups;
  } launch[2];
} spiffy_gemm_plan_t;
int spiffy_gemm_plan(int32_t epilogue, int32_t M, int32_t N, int32_t K, int32_t with_workspace,
                     spiffy_gemm_plan_t *plan);

/* Acceptance walk (Alg. 1 step 5).  graph_edges [E,2] int32 (parent, child), E >= 0;
 * draft_states, target_states [G,B] int32; 0 <= root < G <= SPIFFY_MAX_G.  Starting at root, move
 * to the lowest-id child (by the edge list only) whose draft state equals the current node's
 * target state at all B positions; stop when none matches or a node would repeat.  result
 * (device) receives the node, depth and n_steps; accepted_state [B] (device, may be NULL)
 * receives target_states[node].  Edges with an endpoint outside [0,G) are ignored and flagged. */
int spiffy_graph_accept(const int32_t *graph_edges, int32_t E, const int32_t *draft_states,
                        const int32_t *target_states, int32_t G, int32_t B, int32_t root,
                        spiffy_accept_result *result, int32_t *accepted_state, void *stream);

/* Drafting source (Sec. 4.4.2, vocabulary sort): the K most likely tokens and their probabilities at every
 * masked position of one node's block, most likely first (equal logits to the lower token id), from the
 * distribution the preceding head pass computed for that node.  Must follow, on the same stream, a
 * spiffy_decode_head, spiffy_verify_step, spiffy_verify_step_seq or spiffy_verify_step_commit call with the same cfg, G, B,
 * block_tokens, logit_scale, w_vocab and workspace (after_step says which kind, 0 = decode_head; every step
 * keeps the head's scratch at the start of its workspace, so the flag does not change where it is looked
 * for): it reads what that call left in the workspace (the
 * gathered normalised rows and the per-row / per-vocabulary-chunk summaries) and recomputes only the logits
 * of the K best 128-token chunks of every row.  The node is result->node read on the device (result may be
 * NULL: then `node`, 0 <= node < G).  1 <= K <= SPIFFY_MAX_TOPK.
 * Outputs (device): topk_tokens [B,K] int32, topk_probs [B,K] float.  Column 0 is exactly the argmax / conf
 * of that node's rows.  Positions that are not masked get their own token and probability 0; ranks that do
 * not exist (K > vocab) get token -1 and probability 0.  These are the inputs of spiffy_draft_prune. */
int spiffy_head_topk(const spiffy_model_cfg *cfg, const void *w_vocab, const int32_t *block_tokens, int32_t G,
                     int32_t B, const spiffy_accept_result *result, int32_t node, int32_t K, float logit_scale,
                     int32_t after_step, int32_t *topk_tokens, float *topk_probs, void *workspace,
                     size_t workspace_bytes, void *stream);

/* Drafting and pruning for the NEXT step (Sec. 4.4.2 drafting source, 4.4.3 draft formulas, 4.4.4 pruning),
 * one launch, no host synchronisation.  All pointers are device memory.
 *   state [B] int32: the current block X_k(t); positions equal to mask_id are masked.
 *   topk_tokens [B,K] int32, topk_probs [B,K] float: per position the K most likely tokens of the current
 *     distribution and their probabilities, most likely first (column 0 = the confidence); only rows of
 *     masked positions are read.  With K = 1 these are the argmax / conf rows that spiffy_decode_head wrote
 *     for the accepted node.
 *   formula_offsets [D+1], formula_pairs [nnz,2] int32: draft formula m (1..D) is the set of pairs
 *     (i, j), 1-based, i = token position rank (masked positions sorted by confidence, most confident
 *     first, ties to the lower position), j = vocabulary rank; pairs formula_offsets[m-1] ..
 *     formula_offsets[m]-1.  Node 0 of the graph is the current block (empty formula).
 *   edges [E,2] int32 (parent, child) over nodes 0..D;  0 <= D <= SPIFFY_MAX_G-1, 1 <= B <= 4096,
 *     1 <= K <= 16, 0 <= d_star.
 * Outputs: drafts [D+1,B] (row m = the current block with c_ij unmasked at the position of rank i for every
 * pair of formula m; a formula that names a rank beyond the masked positions, a vocabulary rank beyond K or
 * one position twice, or whose offsets are not increasing within [0,nnz], cannot be built: its row is the
 * current block and buildable[m] = 0); local [D+1], score [D+1] float (geometric means of Sec. 4.4.4 over the
 * buildable children in `edges`; no children: the local score; NaN for node 0 and unbuildable nodes);
 * kept [d_star+1]: node 0 and the d_star best-scoring buildable nodes (equal scores to the lower index), in
 * ascending node order; states_out [d_star+1,B]: their blocks in that order; edges_out [E,2]: the edges whose
 * two ends are kept, original order, renumbered to positions in `kept`; counts [2]: number of kept nodes and
 * of surviving edges.  states_out / edges_out / counts are the block_tokens / graph_edges of the next
 * spiffy_verify_step. */
int spiffy_draft_prune(const int32_t *state, int32_t B, int32_t mask_id, const int32_t *topk_tokens,
                       const float *topk_probs, int32_t K, const int32_t *formula_offsets,
                       const int32_t *formula_pairs, int32_t D, int32_t nnz, const int32_t *edges, int32_t E,
                       int32_t d_star, int32_t *drafts, uint8_t *buildable, float *local, float *score,
                       int32_t *kept, int32_t *states_out, int32_t *edges_out, int32_t *counts, void *stream);

/* The whole step on one stream with no host synchronisation: embed, n_layers x verify_layer,
 * decode_head, graph_accept.  layers / prefix are HOST arrays of n_layers structs.
 * hidden_out [G,B,d] receives the last layer's output.  It may be NULL: the hidden states then stay in the
 * workspace, and the last layer computes only the rows of masked positions behind its attention (see
 * spiffy_verify_layer_last; every output of the step is the same, bit for bit). */
int spiffy_verify_step(const spiffy_model_cfg *cfg, int32_t n_layers,
                       const spiffy_layer_weights *layers, const spiffy_prefix_kv *prefix,
                       const void *w_embed, const void *final_norm, const void *w_vocab,
                       const int32_t *block_tokens, int32_t G, int32_t B, int32_t pos0,
                       const int32_t *graph_edges, int32_t E, int32_t root, float threshold,
                       float logit_scale, int32_t force_one, void *hidden_out, int32_t *argmax,
                       float *conf, uint8_t *unmask, float *top2_margin, int32_t *target_states,
                       spiffy_accept_result *result, int32_t *accepted_state, void *workspace,
                       size_t workspace_bytes, void *stream);

/* The whole step for a full-sequence bidirectional model that caches only the prefix (Sec. 4.3, Fig. 4, App. A.2):
 * the true sequence after the prefix, i.e. the true block (state 0) and the S tokens after it (suffix_tokens [S],
 * device memory), is recomputed in the call and attends to itself; every draft block attends to the prefix, to
 * itself and to the true suffix, never to the block it drafts for.  In every layer the rotated keys and the values
 * of the true block and of the suffix are WRITTEN to rows P .. P+B+S-1 of that layer's cache (prefix[l].k / .v must
 * have capacity >= P + B + S; prefix[l].S must be 0: the suffix is computed here, not cached), from where the
 * blocks read the suffix and the suffix rows read the whole true sequence.  The suffix sits at positions
 * pos0+B .. pos0+B+S-1.  Head and walk run on the G blocks only.  hidden_out [G*B + S, d] (block rows, then
 * suffix rows; may be NULL).  Workspace from spiffy_workspace_bytes_seq.  S <= SPIFFY_MAX_SUFFIX; S = 0 is
 * spiffy_verify_step.  Other arguments and errors as for spiffy_verify_step. */
#define SPIFFY_MAX_SUFFIX 4096
size_t spiffy_workspace_bytes_seq(const spiffy_model_cfg *cfg, int32_t G, int32_t B, int32_t S, int32_t P_max);
int spiffy_verify_step_seq(const spiffy_model_cfg *cfg, int32_t n_layers, const spiffy_layer_weights *layers,
                           const spiffy_prefix_kv *prefix, const void *w_embed, const void *final_norm,
                           const void *w_vocab, const int32_t *block_tokens, const int32_t *suffix_tokens,
                           int32_t G, int32_t B, int32_t S, int32_t pos0, const int32_t *graph_edges, int32_t E,
                           int32_t root, float threshold, float logit_scale, int32_t force_one, void *hidden_out,
                           int32_t *argmax, float *conf, uint8_t *unmask, float *top2_margin,
                           int32_t *target_states, spiffy_accept_result *result, int32_t *accepted_state,
                           void *workspace, size_t workspace_bytes, void *stream);

/* Prefix-cache extension when a block is complete (prefix caching, Sec. 3.1: the keys and values of everything
 * before the block being decoded stay fixed).  One forward pass of the finished block (B tokens, no MASK
 * expected but not checked) through the n_layers layers; in every layer the block's keys (rotated at positions
 * pos0 .. pos0+B-1) and values are written to rows P .. P+B-1 of every KV head of that layer's cache, where
 * P = prefix[l].P.  prefix[l].k / .v must have capacity >= P + B rows per head; the structs themselves are not
 * modified: the caller adds B to every P before the next block.  layers / prefix are HOST arrays.  Workspace as
 * for spiffy_verify_step with G = 1. */
int spiffy_commit_block(const spiffy_model_cfg *cfg, int32_t n_layers, const spiffy_layer_weights *layers,
                        const spiffy_prefix_kv *prefix, const void *w_embed, const int32_t *block_tokens,
                        int32_t B, int32_t pos0, void *workspace, size_t workspace_bytes, void *stream);

/* spiffy_commit_block of the block just finished and spiffy_verify_step of the first state(s) of the next block
 * in ONE pass over the weights (with few states the step only streams weights, so two passes cost twice one;
 * prefix caching, Sec. 3.1, and the step of Alg. 1).  prev_block_tokens [B] (device) is the finished block, at
 * positions pos0-B .. pos0-1, with prefix[l].P rows in front of it; its keys / values are written to cache rows
 * P .. P+B-1 of every layer (capacity >= P + B), exactly as spiffy_commit_block writes them.  block_tokens [G,B]
 * are the states of the block at positions pos0 .. pos0+B-1: they attend to the P + B rows that are the prefix
 * once the call has written them (and, with prefix[l].S > 0, to the S - B suffix rows behind their own slot, while
 * the finished block attends to all S, as in the two separate calls).  Results: those of spiffy_commit_block
 * followed by spiffy_verify_step with P + B (and S - B), bit for bit.  The structs are not modified: the caller
 * adds B to every P (and takes B off every S) afterwards.  hidden_out [G*B + B, d] (the states' rows, then the
 * finished block's; may be NULL).  pos0 >= B; (G + 1) * B <= SPIFFY_MAX_ROWS.  Workspace from
 * spiffy_workspace_bytes_commit (P_max = the largest P + S).  Other arguments and errors as for
 * spiffy_verify_step. */
size_t spiffy_workspace_bytes_commit(const spiffy_model_cfg *cfg, int32_t G, int32_t B, int32_t P_max);
int spiffy_verify_step_commit(const spiffy_model_cfg *cfg, int32_t n_layers, const spiffy_layer_weights *layers,
                              const spiffy_prefix_kv *prefix, const void *w_embed, const void *final_norm,
                              const void *w_vocab, const int32_t *prev_block_tokens, const int32_t *block_tokens,
                              int32_t G, int32_t B, int32_t pos0, const int32_t *graph_edges, int32_t E,
                              int32_t root, float threshold, float logit_scale, int32_t force_one, void *hidden_out,
                              int32_t *argmax, float *conf, uint8_t *unmask, float *top2_margin,
                              int32_t *target_states, spiffy_accept_result *result, int32_t *accepted_state,
                              void *workspace, size_t workspace_bytes, void *stream);

/* Offline calibration, part 3 (Alg. 2; App. D.1): the optimal subgraph of the candidate graph.  The graph has
 * N <= 64 nodes (draft formulas q_kv); count [N] is each node's frequency, level [N] its 1-based level k, edges
 * [E,2] rows (p, q): p is a parent of q (rows with an end outside 0..N-1 are ignored).  A node is connected to a
 * set if its level is 1 or 2 or one of its parents is in the set; G' is every set of D nodes all of which are
 * connected to it; the result is the set of G' with the largest summed count, equal sums going to the smaller
 * bit mask sum_q 2^q.  Every one of the C(N, D) sets is tried; more than SPIFFY_SUBGRAPH_MAX_SETS is refused
 * (SPIFFY_ESHAPE).  Outputs: *best_mask, *best_sum, *n_connected = |G'|, nodes_out [D] (optional) the chosen
 * nodes ascending.  When G' is empty (also D > N): mask 0, sum 0, nodes -1.  |count| must stay below 2^56 so the
 * sums cannot wrap.  All arrays and outputs are device memory; workspace (256-byte aligned) of
 * spiffy_subgraph_search_workspace_bytes() bytes.  Enqueues three kernels; no host synchronisation. */
#define SPIFFY_SUBGRAPH_MAX_SETS (1ull << 40)
size_t spiffy_subgraph_search_workspace_bytes(void);
int spiffy_subgraph_search(const int64_t *count, const int32_t *level, int32_t N, const int32_t *edges, int32_t E,
                           int32_t D, uint64_t *best_mask, int64_t *best_sum, uint64_t *n_connected,
                           int32_t *nodes_out, void *workspace, size_t workspace_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SPIFFY_H */

// C ABI of the verification library: argument checks, workspace carving, kernel selection by
// shape, launch order.  No kernel lives here.  Every check runs before the first launch.
#include <cmath>
#include <cstring>

#include <mutex>

#include "kernels.h"

using namespace spiffy;

// Scratch of the allocation-free entry point (spiffy_decode_head_static): every GPU the library runs on holds its own
// copy of this array until the process ends.  In host code the name is only a handle for hipGetSymbolAddress; kernels
// get the device address that call returns.
static __device__ __align__(256) unsigned char scratch[SPIFFY_STATIC_SCRATCH_BYTES];

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t esize(int dtype) { return dtype == SPIFFY_F32 ? 4 : 2; }

int check_cfg(const spiffy_model_cfg* c) {
  if (!c) return SPIFFY_EINVAL;
  if (c->dtype != SPIFFY_BF16 && c->dtype != SPIFFY_F32) return SPIFFY_EINVAL;
  if (c->d < 8 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->head_dim < 2 || c->ffn < 8 || c->vocab < 2)
    return SPIFFY_EINVAL;
  if (c->mask_id < 0 || c->mask_id >= c->vocab) return SPIFFY_EINVAL;
  if (!(c->rms_eps >= 0.f) || !(c->rope_base > 0.f)) return SPIFFY_EINVAL;
  if (c->n_q_heads % c->n_kv_heads != 0) return SPIFFY_ESHAPE;
  if (c->head_dim % 8 != 0 || c->head_dim > 256) return SPIFFY_ESHAPE;
  if (c->d % 8 != 0 || c->ffn % 8 != 0) return SPIFFY_ESHAPE;
  return SPIFFY_OK;
}

int check_gb(int32_t G, int32_t B) {
  if (G < 1 || B < 1) return SPIFFY_EINVAL;
  if ((int64_t)G * B > SPIFFY_MAX_ROWS) return SPIFFY_ESHAPE;
  return SPIFFY_OK;
}

bool layer_mfma(const spiffy_model_cfg* c) {
  if (c->dtype != SPIFFY_BF16 || c->head_dim != 128) return false;
  return c->d % 128 == 0 && c->ffn % 64 == 0;
}
bool head_mfma(const spiffy_model_cfg* c) {
  if (c->dtype != SPIFFY_BF16) return false;
  return c->d % 64 == 0;
}

// Limits of the MFMA LM head: per-lane byte offsets into the vocabulary matrix and into the gathered rows are 32-bit,
// and the top-K refinement holds at most 2048 per-chunk summaries of a row (V <= 262144).
bool head_shape_ok(const spiffy_model_cfg* c) {
  if (!head_mfma(c)) return true;
  const size_t lim = (size_t)1 << 32;
  if ((size_t)c->vocab * c->d * 2 >= lim || (size_t)SPIFFY_MAX_ROWS * c->d * 2 >= lim) return false;
  return mfma_lmhead_partials_per_row(c->vocab) <= 2048;
}

// generic attention keeps all scores of one row in LDS
size_t generic_attn_smem(const spiffy_model_cfg* c, int B, int P) {
  const int hd = c->head_dim;
  const int nchunk = 256 / hd > 0 ? 256 / hd : 1;
  return sizeof(float) * ((size_t)hd + (size_t)B * hd + (size_t)(P + B) + (size_t)nchunk * hd);
}
constexpr size_t kMaxGenericSmem = 150 * 1024;

struct Carve {
  unsigned char* base;
  size_t off;
  explicit Carve(void* p) : base(reinterpret_cast<unsigned char*>(p)), off(0) {}
  void* take(size_t bytes) {
    void* r = base ? base + off : nullptr;
    off += align_up(bytes, 256);
    return r;
  }
};

struct LayerWs {
  void *n, *qkv, *attn, *h, *act, *attn_partial, *attn_partial_seq, *splitk;
  void *gat_attn, *gat_x;        // last layer, masked rows only: gathered attention rows and residual rows
  int32_t *rows, *count;         // ... and their row list
  size_t bytes;
};
// P = cached rows (prefix and suffix together).  S_seq > 0: full-sequence step, S_seq true suffix rows ride along
// after the G*B block rows and have an attention scratch of their own (queries over the P + B + S_seq cache rows).
LayerWs carve_layer(const spiffy_model_cfg* c, int G, int B, int P, void* base, int S_seq = 0) {
  const size_t M = (size_t)G * B + S_seq, es = esize(c->dtype);
  const size_t qkv_cols = (size_t)(c->n_q_heads + 2 * c->n_kv_heads) * c->head_dim;
  Carve cv(base);
  LayerWs w;
  w.n = cv.take(M * c->d * es);
  w.qkv = cv.take(M * qkv_cols * es);
  w.attn = cv.take(M * (size_t)c->n_q_heads * c->head_dim * es);
  w.h = cv.take(M * c->d * es);
  w.act = cv.take(M * c->ffn * es);
  w.attn_partial = cv.take(layer_mfma(c) ? mfma_attn_partial_bytes(G, B, c->n_q_heads, c->head_dim, P + S_seq) : 0);
  w.attn_partial_seq = cv.take(layer_mfma(c) && S_seq ? mfma_attn_partial_bytes(1, S_seq, c->n_q_heads, c->head_dim, P + B + S_seq) : 0);
  w.splitk = cv.take(layer_mfma(c) ? sizeof(float) * 4 * M * c->d : 0);   // up to 4 K slices of [M,d] fp32
  w.gat_attn = cv.take(M * (size_t)c->n_q_heads * c->head_dim * es);
  w.gat_x = cv.take(M * c->d * es);
  w.rows = (int32_t*)cv.take(sizeof(int32_t) * M);
  w.count = (int32_t*)cv.take(sizeof(int32_t) * 4);
  w.bytes = cv.off;
  return w;
}

struct HeadWs {
  int32_t *row_idx, *count;
  void* nf;
  TopPartial *part, *part2, *row_top;
  float* cand_val;       // top-K refinement candidates [B][SPIFFY_MAX_TOPK][SPIFFY_MAX_TOPK]
  int32_t* cand_idx;
  int m_cap, n_part;
  size_t bytes;
};
HeadWs carve_head(const spiffy_model_cfg* c, int G, int B, void* base) {
  const int M = G * B;
  Carve cv(base);
  HeadWs w;
  w.m_cap = (int)align_up((size_t)M, 128);
  w.n_part = head_mfma(c) ? mfma_lmhead_partials_per_row(c->vocab) : 0;
  w.row_idx = (int32_t*)cv.take(sizeof(int32_t) * w.m_cap);
  w.count = (int32_t*)cv.take(sizeof(int32_t) * 4);
  w.nf = cv.take((size_t)w.m_cap * c->d * esize(c->dtype));
  w.part = (TopPartial*)cv.take(sizeof(TopPartial) * (size_t)w.n_part * w.m_cap);
  w.part2 = (TopPartial*)cv.take(sizeof(TopPartial) * (size_t)kLmheadCombineSlices * w.m_cap);
  w.row_top = (TopPartial*)cv.take(sizeof(TopPartial) * w.m_cap);
  w.cand_val = (float*)cv.take(sizeof(float) * (size_t)B * SPIFFY_MAX_TOPK * SPIFFY_MAX_TOPK);
  w.cand_idx = (int32_t*)cv.take(sizeof(int32_t) * (size_t)B * SPIFFY_MAX_TOPK * SPIFFY_MAX_TOPK);
  w.bytes = cv.off;
  return w;
}

// layer and head scratch alias each other (used one after the other); the step adds a hidden
// buffer and a next-state buffer in front.
struct StepWs {
  void* hidden;
  int32_t* target;
  void* rest;
  size_t rest_bytes, bytes;
};
StepWs carve_step(const spiffy_model_cfg* c, int G, int B, int P, void* base, int S_seq = 0) {
  const size_t M = (size_t)G * B;
  Carve cv(base);
  StepWs w;
  // the layer / head scratch comes first, so that the head's leftovers sit at the start of the workspace whatever
  // G, B, P and S_seq were (spiffy_head_topk finds them there after a step)
  const size_t lb = carve_layer(c, G, B, P, nullptr, S_seq).bytes, hb = carve_head(c, G, B, nullptr).bytes;
  w.rest_bytes = lb > hb ? lb : hb;
  w.rest = cv.take(w.rest_bytes);
  w.hidden = cv.take((M + S_seq) * c->d * esize(c->dtype));
  w.target = (int32_t*)cv.take(sizeof(int32_t) * M);
  w.bytes = cv.off;
  return w;
}

int dev(hipError_t e) { return e == hipSuccess ? SPIFFY_OK : SPIFFY_EDEVICE; }

int check_layer_args(const spiffy_model_cfg* cfg, const spiffy_layer_weights* w, const spiffy_prefix_kv* prefix,
                     int32_t G, int32_t B) {
  if (!w || !prefix) return SPIFFY_EINVAL;
  if (!w->wq || !w->wk || !w->wv || !w->wo || !w->w_gate || !w->w_up || !w->w_down || !w->norm1 || !w->norm2)
    return SPIFFY_EINVAL;
  if (prefix->P < 0 || (prefix->P > 0 && (!prefix->k || !prefix->v))) return SPIFFY_EINVAL;
  if (prefix->capacity != 0 && prefix->capacity < prefix->P) return SPIFFY_EINVAL;
  if (prefix->S < 0 || (prefix->S > 0 && (!prefix->k || !prefix->v))) return SPIFFY_EINVAL;
  if (prefix->S > 0 && (int64_t)prefix->P + B + prefix->S > prefix->capacity) return SPIFFY_ESHAPE;  // suffix rows sit after the block's slot
  const void* ptrs[] = {w->wq, w->wk, w->wv, w->wo, w->w_gate, w->w_up, w->w_down, w->norm1, w->norm2,
                        w->bq, w->bk, w->bv, prefix->k, prefix->v};
  for (const void* p : ptrs)
    if (p && !aligned16(p)) return SPIFFY_EALIGN;
  if (!layer_mfma(cfg) && generic_attn_smem(cfg, B, prefix->P + prefix->S) > kMaxGenericSmem) return SPIFFY_ESHAPE;
  // the reduction behind the split-K projections keeps a row of d fp32 values in 64 KB of LDS for its RMSNorm
  if (layer_mfma(cfg) && (size_t)cfg->d * sizeof(float) > 64 * 1024) return SPIFFY_ESHAPE;
  return SPIFFY_OK;
}

// Chaining hints used by the whole-step driver: `normed_in` = ws.n already holds RMSNorm-1 of hidden_in
// (written by the previous layer's last kernel); `next_norm1` = gain of the next layer's RMSNorm-1, to be
// produced into ws.n by this layer's last kernel; `rope_ready` = the rotary table is already in place.
struct LayerChain {
  bool normed_in = false;
  const void* next_norm1 = nullptr;
  bool rope_ready = false;
  bool normed_out = false;   // set when ws.n holds the next layer's normalised input on return
  bool append_kv = false;    // write the (rotated) K and V rows of state 0 into the cache at rows P .. P+B-1
  int seq_S = 0;             // full-sequence step: this many true suffix rows follow the G*B block rows
  bool rope_ready_seq = false;
  // commit-and-verify step (seq_S == B): the trailing B rows are the finished block BEFORE the one being decoded.
  // prefix->P counts the rows in front of that finished block; its keys / values are written to cache rows
  // P .. P+B-1 and the G states (positions pos0 = that block's + B) attend to P + B cached rows.
  bool tail_is_prev_block = false;
  // Last layer of a step: only masked positions are decoded (Alg. 1 steps 1-4 look at masked positions only), so
  // beyond the attention, where every row still supplies keys and values, only their rows are computed.  rows /
  // count: the device-side list of those rows (ascending) in the layer scratch; the other rows of hidden_out are
  // left as they are.
  bool masked_rows_only = false;
  const int32_t* tokens = nullptr;    // [G,B] block tokens and optional explicit mask, for the row list
  const uint8_t* mask = nullptr;
};

// The same product as two launches over the row ranges [0, rows_a) and [rows_a, rows_a + rows_b): each range gets the
// tile shape that suits its height (a ragged total would otherwise pay a whole extra round of the tall tiles).
// Rows are independent and the K order of an element does not depend on the shape, so nothing else changes.
hipError_t launch_gemm_mfma_rows(int epi, GemmArgs g, int rows_a, int rows_b, int dtype, hipStream_t st) {
  const size_t es = esize(dtype), ces = epi == EPI_PARTIAL ? sizeof(float) : es;
  g.Mz = rows_a + rows_b;
  // one launch when there are few rows in all (weight streaming sets the time: stream them once, not twice) or
  // when the second range adds no 256-row tile
  if (rows_a + rows_b <= 512 || cdiv(rows_a + rows_b, 256) == cdiv(rows_a, 256)) {
    g.M = rows_a + rows_b;
    return launch_gemm_mfma(epi, g, st);
  }
  GemmArgs a = g;
  a.M = rows_a;
  hipError_t e = launch_gemm_mfma(epi, a, st);
  if (e != hipSuccess || rows_b == 0) return e;
  GemmArgs b = g;
  b.M = rows_b;
  b.A = reinterpret_cast<const char*>(g.A) + (size_t)rows_a * g.lda * es;
  b.C = reinterpret_cast<char*>(g.C) + (size_t)rows_a * g.ldc * ces;
  if (g.R) b.R = reinterpret_cast<const char*>(g.R) + (size_t)rows_a * g.ldc * es;
  return launch_gemm_mfma(epi, b, st);
}

int run_layer(const spiffy_model_cfg* cfg, const spiffy_layer_weights* w, const spiffy_prefix_kv* prefix,
              const void* hidden_in, int G, int B, int pos0, void* hidden_out, void* workspace, hipStream_t st,
              LayerChain* chain = nullptr) {
  // S_seq > 0 (full-sequence step): rows G*B .. G*B+S_seq-1 of every activation matrix are the true suffix.  It is
  // recomputed like the blocks; its fresh keys / values, and those of the true block (state 0), go to the cache
  // rows behind the prefix, where the blocks find the suffix (as in the dual-cache layout) and the suffix rows
  // find the whole true sequence.
  const int S_seq = chain ? chain->seq_S : 0;
  const bool prev = chain && chain->tail_is_prev_block;
  const int M = G * B + S_seq, d = cfg->d, dt = cfg->dtype;
  const int qd = cfg->n_q_heads * cfg->head_dim, kvd = cfg->n_kv_heads * cfg->head_dim;
  const bool mf = layer_mfma(cfg);
  const LayerWs ws = carve_layer(cfg, G, B, prefix->P + prefix->S, workspace, S_seq);
  int rc;
  auto mfma_rows = [&](int epi, const GemmArgs& ga) {
    return S_seq ? launch_gemm_mfma_rows(epi, ga, G * B, S_seq, dt, st) : launch_gemm_mfma(epi, ga, st);
  };
  if (chain) chain->normed_out = false;
  if (!(chain && chain->normed_in) &&
      (rc = dev(launch_rmsnorm(dt, hidden_in, w->norm1, cfg->rms_eps, M, d, nullptr, nullptr, ws.n, st))))
    return rc;

  GemmArgs g;
  std::memset(&g, 0, sizeof(g));
  g.A = ws.n; g.lda = d; g.M = M; g.K = d;
  g.W[0] = w->wq; g.W[1] = w->wk; g.W[2] = w->wv;
  g.bias[0] = w->bq; g.bias[1] = w->bk; g.bias[2] = w->bv;
  g.Nseg[0] = qd; g.Nseg[1] = kvd; g.Nseg[2] = kvd;
  g.N = qd + 2 * kvd; g.C = ws.qkv; g.ldc = g.N; g.scale = 1.f;
  const bool mf_qkv = mf && mfma_gemm_supported(EPI_STORE, g);
  if ((rc = dev(mf_qkv ? mfma_rows(EPI_STORE, g) : launch_gemm_generic(dt, EPI_STORE, g, st)))) return rc;

  AttnArgs a;
  a.qkv = ws.qkv; a.prefix_k = prefix->k; a.prefix_v = prefix->v; a.out = ws.attn; a.partial = ws.attn_partial;
  a.G = G; a.B = B; a.Hq = cfg->n_q_heads; a.Hkv = cfg->n_kv_heads; a.hd = cfg->head_dim; a.P = prefix->P;
  a.ldp = prefix->capacity;
  a.S = S_seq ? S_seq : prefix->S;
  if (prev) {                // the finished block has joined the prefix; a cached suffix loses the current block's slot
    a.P = prefix->P + B;
    a.S = prefix->S > B ? prefix->S - B : 0;
  }
  a.own = 1;
  a.pos0 = pos0; a.rope_base = cfg->rope_base; a.rope_ready = chain && chain->rope_ready;
  const int ldp = prefix->capacity ? prefix->capacity : prefix->P;
  // The appends rotate keys with the tables the attention kernels use (built here, once per step, when the MFMA
  // attention will run; otherwise the append computes the same values itself).
  const bool mfa = mf && mfma_attn_supported(a);
  const int tail_pos0 = prev ? pos0 - B : pos0 + B;
  bool tail_rope_ready = chain && chain->rope_ready_seq;
  const void *tab = nullptr, *tab_tail = nullptr;
  if (mfa && chain && (chain->append_kv || S_seq)) {
    if (!a.rope_ready) {
      launch_rope_table(ws.attn_partial, B, pos0, cfg->rope_base, st);
      a.rope_ready = 1;
    }
    tab = ws.attn_partial;
    if (S_seq) {
      if (!tail_rope_ready) {
        launch_rope_table(ws.attn_partial_seq, S_seq, tail_pos0, cfg->rope_base, st);
        tail_rope_ready = true;
      }
      tab_tail = ws.attn_partial_seq;
    }
  }
  if (S_seq && !prev) {
    // the true block (state 0: qkv rows 0 .. B-1) and the suffix (qkv rows G*B ..) land next to each other in the cache,
    // at consecutive positions: one launch over the two runs of rows
    if ((rc = dev(launch_kv_append(dt, ws.qkv, a.Hq, a.Hkv, a.hd, B + S_seq, pos0, cfg->rope_base,
                                   const_cast<void*>(prefix->k), const_cast<void*>(prefix->v), prefix->P, ldp, st, B,
                                   (G - 1) * B, tab, tab_tail))))
      return rc;
  } else {
    if (chain && chain->append_kv &&
        (rc = dev(launch_kv_append(dt, ws.qkv, a.Hq, a.Hkv, a.hd, B, pos0, cfg->rope_base,
                                   const_cast<void*>(prefix->k), const_cast<void*>(prefix->v), prefix->P, ldp, st, 0, 0,
                                   tab))))
      return rc;
    if (S_seq) {     // the finished block in front of the states
      const size_t es = esize(dt);
      const char* qkv_seq = reinterpret_cast<const char*>(ws.qkv) + (size_t)G * B * g.N * es;
      if ((rc = dev(launch_kv_append(dt, qkv_seq, a.Hq, a.Hkv, a.hd, S_seq, tail_pos0, cfg->rope_base,
                                     const_cast<void*>(prefix->k), const_cast<void*>(prefix->v), prefix->P, ldp, st, 0, 0,
                                     tab_tail))))
        return rc;
    }
  }
  if (!(S_seq && mfa) &&      // with rows riding along, the MFMA path runs both groups in one launch below
      (rc = dev(mfa ? launch_attn_mfma(a, st) : launch_attn_generic(dt, a, st))))
    return rc;
  if (S_seq) {      // the suffix rows: queries at positions pos0+B .., keys = cache rows 0 .. P+B+S_seq-1, no block of their own
    const size_t es = esize(dt);
    AttnArgs b = a;
    b.qkv = reinterpret_cast<const char*>(ws.qkv) + (size_t)G * B * g.N * es;
    b.out = reinterpret_cast<char*>(ws.attn) + (size_t)G * B * qd * es;
    b.partial = ws.attn_partial_seq;
    b.G = 1; b.B = S_seq; b.P = prefix->P + B + S_seq; b.S = 0; b.own = 0;
    b.pos0 = tail_pos0; b.rope_ready = tail_rope_ready;
    if (prev) {     // the finished block: one state at the positions before pos0, over the rows in front of it
      b.P = prefix->P; b.S = prefix->S; b.own = 1;
    }
    if (mfa) {       // (b differs from a in row counts and lengths only)
      if ((rc = dev(launch_attn_mfma_pair(a, b, st)))) return rc;
    } else if ((rc = dev(launch_attn_generic(dt, b, st)))) return rc;
  }

  // Masked rows only (last layer): from here on row r of every matrix is row ws.rows[r] of the block rows, r < *ws.count.
  // The row count is known on the device only: the launches cover all M rows and skip what lies beyond it.  A row's
  // arithmetic does not depend on where it sits, so the results are those of the full layer, bit for bit.
  const bool cm = chain && chain->masked_rows_only && !S_seq;
  const int32_t* n_rows = cm ? ws.count : nullptr;
  const void* attn_rows = ws.attn;
  const void* resid = hidden_in;
  if (cm) {
    const size_t es = esize(dt);
    if ((rc = dev(launch_compact_rows(chain->tokens, chain->mask, cfg->mask_id, M, ws.rows, ws.count, st)))) return rc;
    if ((rc = dev(launch_gather_rows2(ws.attn, (size_t)qd * es, hidden_in, (size_t)d * es, ws.rows, ws.count, M, ws.gat_attn,
                                      ws.gat_x, st))))
      return rc;
    attn_rows = ws.gat_attn;
    resid = ws.gat_x;
  }

  // output projection + residual (+ RMSNorm-2 fused into the split-K reduction when K is sliced)
  std::memset(&g, 0, sizeof(g));
  g.A = attn_rows; g.lda = qd; g.M = M; g.M_dev = n_rows; g.K = qd; g.W[0] = w->wo; g.Nseg[0] = d; g.N = d;
  g.C = ws.h; g.ldc = d; g.R = resid; g.scale = 1.f;
  bool normed = false;
  if (mf && mfma_gemm_supported(EPI_RESID, g)) {
    const int ks = mfma_ksplit(d, qd);
    if (ks > 1) {
      g.C = ws.splitk; g.ksplit = ks;
      if ((rc = dev(mfma_rows(EPI_PARTIAL, g)))) return rc;
      if ((rc = dev(launch_splitk_reduce((const float*)ws.splitk, ks, resid, ws.h, w->norm2, cfg->rms_eps, ws.n, M,
                                         d, st, n_rows))))
        return rc;
      normed = true;
    } else if ((rc = dev(mfma_rows(EPI_RESID, g)))) return rc;
  } else if ((rc = dev(launch_gemm_generic(dt, EPI_RESID, g, st)))) return rc;

  if (!normed && (rc = dev(launch_rmsnorm(dt, ws.h, w->norm2, cfg->rms_eps, M, d, nullptr, n_rows, ws.n, st))))
    return rc;

  std::memset(&g, 0, sizeof(g));
  g.A = ws.n; g.lda = d; g.M = M; g.M_dev = n_rows; g.K = d; g.W[0] = w->w_gate; g.W[1] = w->w_up; g.N = cfg->ffn;
  g.C = ws.act; g.ldc = cfg->ffn; g.scale = 1.f;
  if ((rc = dev(mf && mfma_gemm_supported(EPI_SWIGLU, g) ? mfma_rows(EPI_SWIGLU, g)
                                                          : launch_gemm_generic(dt, EPI_SWIGLU, g, st))))
    return rc;

  // down projection + residual; compacted rows go back to their places in hidden_out (by the reduction when K is
  // sliced, else through ws.gat_x, which is free once the output projection has read it)
  std::memset(&g, 0, sizeof(g));
  g.A = ws.act; g.lda = cfg->ffn; g.M = M; g.M_dev = n_rows; g.K = cfg->ffn; g.W[0] = w->w_down; g.Nseg[0] = d; g.N = d;
  g.C = cm ? ws.gat_x : hidden_out; g.ldc = d; g.R = ws.h; g.scale = 1.f;
  if (mf && mfma_gemm_supported(EPI_RESID, g)) {
    const int ks = mfma_ksplit(d, cfg->ffn);
    if (ks > 1) {
      g.C = ws.splitk; g.ksplit = ks;
      if ((rc = dev(mfma_rows(EPI_PARTIAL, g)))) return rc;
      const void* ng = chain ? chain->next_norm1 : nullptr;
      if (chain && ng) chain->normed_out = true;
      return dev(launch_splitk_reduce((const float*)ws.splitk, ks, ws.h, hidden_out, ng, cfg->rms_eps,
                                      ng ? ws.n : nullptr, M, d, st, n_rows, cm ? ws.rows : nullptr));
    }
    if ((rc = dev(mfma_rows(EPI_RESID, g)))) return rc;
  } else if ((rc = dev(launch_gemm_generic(dt, EPI_RESID, g, st)))) return rc;
  if (cm) return dev(launch_scatter_rows(ws.gat_x, (size_t)d * esize(dt), ws.rows, ws.count, M, hidden_out, st));
  return SPIFFY_OK;
}

int run_head(const spiffy_model_cfg* cfg, const void* hidden, const void* final_norm, const void* w_vocab,
             const int32_t* tokens, const uint8_t* mask, int G, int B, float threshold, float logit_scale,
             int force_one, int32_t* argmax, float* conf, uint8_t* unmask, float* margin, int32_t* target,
             void* workspace, hipStream_t st) {
  const int M = G * B, dt = cfg->dtype;
  const HeadWs ws = carve_head(cfg, G, B, workspace);
  int rc;
  if ((rc = dev(launch_compact_rows(tokens, mask, cfg->mask_id, M, ws.row_idx, ws.count, st)))) return rc;
  if ((rc = dev(launch_rmsnorm(dt, hidden, final_norm, cfg->rms_eps, M, cfg->d, ws.row_idx, ws.count, ws.nf, st))))
    return rc;
  if (head_mfma(cfg)) {
    GemmArgs g;
    std::memset(&g, 0, sizeof(g));
    g.A = ws.nf; g.lda = cfg->d; g.M = M; g.M_dev = ws.count; g.K = cfg->d;
    g.W[0] = w_vocab; g.Nseg[0] = cfg->vocab; g.N = cfg->vocab;
    g.C = ws.part; g.ldc = ws.m_cap; g.scale = logit_scale;
    if ((rc = dev(launch_gemm_mfma(EPI_LMHEAD, g, st)))) return rc;
    if ((rc = dev(launch_lmhead_combine(ws.part, ws.n_part, ws.m_cap, ws.count, M, ws.part2, ws.row_top, st)))) return rc;
  } else {
    if ((rc = dev(launch_lmhead_generic(dt, ws.nf, w_vocab, cfg->d, cfg->vocab, logit_scale, ws.count, M,
                                        ws.row_top, st))))
      return rc;
  }
  return dev(launch_head_finalize(ws.row_top, ws.row_idx, ws.count, tokens, mask, cfg->mask_id, G, B, threshold,
                                  force_one, argmax, conf, unmask, margin, target, st));
}

int check_head_args(const spiffy_model_cfg* cfg, const void* hidden, const void* final_norm, const void* w_vocab,
                    const int32_t* tokens, float threshold, float logit_scale, const int32_t* argmax,
                    const float* conf, const uint8_t* unmask) {
  if (!hidden || !final_norm || !w_vocab || !tokens || !argmax || !conf || !unmask) return SPIFFY_EINVAL;
  if (!(threshold >= 0.f && threshold <= 1.f) || !(logit_scale > 0.f) || !std::isfinite(logit_scale))
    return SPIFFY_EINVAL;
  if (!aligned16(hidden) || !aligned16(final_norm) || !aligned16(w_vocab)) return SPIFFY_EALIGN;
  if ((size_t)cfg->d * sizeof(float) > 64 * 1024 && !head_mfma(cfg)) return SPIFFY_ESHAPE;
  return head_shape_ok(cfg) ? SPIFFY_OK : SPIFFY_ESHAPE;
}

int check_accept_args(const int32_t* edges, int32_t E, const int32_t* draft, const int32_t* target, int32_t G,
                      int32_t B, int32_t root, const spiffy_accept_result* res) {
  if (G < 1 || B < 1 || E < 0 || (E > 0 && !edges) || !draft || !target || !res) return SPIFFY_EINVAL;
  if (root < 0 || root >= G) return SPIFFY_EINVAL;
  if (G > SPIFFY_MAX_G) return SPIFFY_ESHAPE;
  return SPIFFY_OK;
}

// Device address of `scratch` on the current device: looked up once per device, with that device current.
int static_scratch_ptr(void** out) {
  static std::mutex mu;
  static void* ptr[64] = {};
  int d = 0;
  if (hipGetDevice(&d) != hipSuccess || d < 0 || d >= 64) return SPIFFY_EDEVICE;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr[d]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return SPIFFY_EDEVICE;
    ptr[d] = p;
  }
  *out = ptr[d];
  return SPIFFY_OK;
}

}  // namespace

extern "C" {
#pragma GCC visibility push(default)

const char* spiffy_status_str(int s) {
  switch (s) {
    case SPIFFY_OK: return "ok";
    case SPIFFY_EINVAL: return "invalid argument";
    case SPIFFY_ESHAPE: return "unsupported shape";
    case SPIFFY_EALIGN: return "pointer not 16-byte aligned";
    case SPIFFY_EWORKSPACE: return "workspace too small";
    case SPIFFY_EDEVICE: return "device launch failed";
    case SPIFFY_ELIMIT: return "size beyond the limit of the allocation-free entry point";
    default: return "unknown status";
  }
}

int spiffy_uses_mfma(const spiffy_model_cfg* cfg, int32_t B) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  if (B < 1) return SPIFFY_EINVAL;
  return layer_mfma(cfg) ? 1 : 0;
}

size_t spiffy_workspace_bytes(const spiffy_model_cfg* cfg, int32_t G, int32_t B, int32_t P_max) {
  if (check_cfg(cfg) || check_gb(G, B) || P_max < 0) return 0;
  return carve_step(cfg, G, B, P_max, nullptr).bytes;
}

int spiffy_embed(const spiffy_model_cfg* cfg, const void* w_embed, const int32_t* block_tokens, int32_t G,
                 int32_t B, void* hidden_out, void* stream) {
  int rc;
  if ((rc = check_cfg(cfg)) || (rc = check_gb(G, B))) return rc;
  if (!w_embed || !block_tokens || !hidden_out) return SPIFFY_EINVAL;
  if (!aligned16(w_embed) || !aligned16(hidden_out)) return SPIFFY_EALIGN;
  return dev(launch_embed(cfg->dtype, w_embed, block_tokens, G * B, cfg->d, cfg->vocab, hidden_out,
                          (hipStream_t)stream));
}

int spiffy_verify_layer(const spiffy_model_cfg* cfg, const spiffy_layer_weights* w, const spiffy_prefix_kv* prefix,
                        const void* hidden_in, int32_t G, int32_t B, int32_t pos0, void* hidden_out,
                        void* workspace, size_t workspace_bytes, void* stream) {
  int rc;
  if ((rc = check_cfg(cfg)) || (rc = check_gb(G, B))) return rc;
  if (!hidden_in || !hidden_out || !workspace || pos0 < 0) return SPIFFY_EINVAL;
  if ((rc = check_layer_args(cfg, w, prefix, G, B))) return rc;
  if (!aligned16(hidden_in) || !aligned16(hidden_out) || (reinterpret_cast<uintptr_t>(workspace) & 255u))
    return SPIFFY_EALIGN;
  if (workspace_bytes < carve_layer(cfg, G, B, prefix->P + prefix->S, nullptr).bytes) return SPIFFY_EWORKSPACE;
  return run_layer(cfg, w, prefix, hidden_in, G, B, pos0, hidden_out, workspace, (hipStream_t)stream);
}

int spiffy_verify_layer_last(const spiffy_model_cfg* cfg, const spiffy_layer_weights* w, const spiffy_prefix_kv* prefix,
                             const void* hidden_in, const int32_t* block_tokens, const uint8_t* mask, int32_t G, int32_t B,
                             int32_t pos0, void* hidden_out, void* workspace, size_t workspace_bytes, void* stream) {
  int rc;
  if ((rc = check_cfg(cfg)) || (rc = check_gb(G, B))) return rc;
  if (!hidden_in || !hidden_out || !workspace || !block_tokens || pos0 < 0) return SPIFFY_EINVAL;
  if ((rc = check_layer_args(cfg, w, prefix, G, B))) return rc;
  if (!aligned16(hidden_in) || !aligned16(hidden_out) || (reinterpret_cast<uintptr_t>(workspace) & 255u))
    return SPIFFY_EALIGN;
  if (workspace_bytes < carve_layer(cfg, G, B, prefix->P + prefix->S, nullptr).bytes) return SPIFFY_EWORKSPACE;
  LayerChain chain;
  chain.masked_rows_only = true;
  chain.tokens = block_tokens;
  chain.mask = mask;
  return run_layer(cfg, w, prefix, hidden_in, G, B, pos0, hidden_out, workspace, (hipStream_t)stream, &chain);
}

int spiffy_decode_head(const spiffy_model_cfg* cfg, const void* hidden, const void* final_norm, const void* w_vocab,
                       const int32_t* block_tokens, const uint8_t* mask, int32_t G, int32_t B, float threshold,
                       float logit_scale, int32_t force_one, int32_t* argmax, float* conf, uint8_t* unmask,
                       float* top2_margin, int32_t* target_states, void* workspace, size_t workspace_bytes,
                       void* stream) {
  int rc;
  if ((rc = check_cfg(cfg)) || (rc = check_gb(G, B))) return rc;
  if (!workspace) return SPIFFY_EINVAL;
  if ((rc = check_head_args(cfg, hidden, final_norm, w_vocab, block_tokens, threshold, logit_scale, argmax, conf,
                            unmask)))
    return rc;
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return SPIFFY_EALIGN;
  if (workspace_bytes < carve_head(cfg, G, B, nullptr).bytes) return SPIFFY_EWORKSPACE;
  return run_head(cfg, hidden, final_norm, w_vocab, block_tokens, mask, G, B, threshold, logit_scale, force_one,
                  argmax, conf, unmask, top2_margin, target_states, workspace, (hipStream_t)stream);
}

int spiffy_decode_head_static(const spiffy_model_cfg* cfg, const void* hidden, const void* final_norm,
                              const void* w_vocab, const int32_t* block_tokens, const uint8_t* mask, int32_t G,
                              int32_t B, float threshold, float logit_scale, int32_t force_one, int32_t* argmax,
                              float* conf, uint8_t* unmask, float* top2_margin, int32_t* target_states, void* stream) {
  int rc;
  if ((rc = check_cfg(cfg)) || (rc = check_gb(G, B))) return rc;
  if ((rc = check_head_args(cfg, hidden, final_norm, w_vocab, block_tokens, threshold, logit_scale, argmax, conf,
                            unmask)))
    return rc;
  if ((int64_t)G * B > SPIFFY_STATIC_MAX_ROWS) return SPIFFY_ELIMIT;
  if (carve_head(cfg, G, B, nullptr).bytes > (size_t)SPIFFY_STATIC_SCRATCH_BYTES) return SPIFFY_ELIMIT;
  void* ws = nullptr;
  if ((rc = static_scratch_ptr(&ws))) return rc;
  // every kernel of the head writes what it later reads (row list and count, gathered rows, summaries): nothing in
  // the scratch has to start at zero, and what the previous call left there is never read
  return run_head(cfg, hidden, final_norm, w_vocab, block_tokens, mask, G, B, threshold, logit_scale, force_one,
                  argmax, conf, unmask, top2_margin, target_states, ws, (hipStream_t)stream);
}

int spiffy_gemm(int32_t dtype, int32_t epilogue, const void* A, const void* W0, const void* W1, const void* R,
                void* C, int32_t M, int32_t N, int32_t K, void* workspace, size_t workspace_bytes, void* stream) {
  if (dtype != SPIFFY_BF16 && dtype != SPIFFY_F32) return SPIFFY_EINVAL;
  if (epilogue < SPIFFY_GEMM_STORE || epilogue > SPIFFY_GEMM_SWIGLU) return SPIFFY_EINVAL;
  if (!A || !W0 || !C || M < 1 || N < 1 || K < 1) return SPIFFY_EINVAL;
  if (epilogue == SPIFFY_GEMM_SWIGLU && !W1) return SPIFFY_EINVAL;
  if (epilogue == SPIFFY_GEMM_RESID && !R) return SPIFFY_EINVAL;
  if (K % 8 != 0 || N % 8 != 0) return SPIFFY_ESHAPE;
  if (!aligned16(A) || !aligned16(W0) || !aligned16(C) || (W1 && !aligned16(W1)) || (R && !aligned16(R)))
    return SPIFFY_EALIGN;
  GemmArgs g;
  std::memset(&g, 0, sizeof(g));
  g.A = A; g.lda = K; g.M = M; g.K = K; g.N = N; g.C = C; g.ldc = N; g.R = R; g.scale = 1.f;
  g.W[0] = W0;
  if (epilogue == SPIFFY_GEMM_SWIGLU) g.W[1] = W1; else g.Nseg[0] = N;
  const bool mf = dtype == SPIFFY_BF16 && mfma_gemm_supported(epilogue, g);
  hipStream_t st = (hipStream_t)stream;
  if (mf && epilogue == SPIFFY_GEMM_RESID) {     // same K slicing as verify_layer when scratch is given
    const int ks = mfma_ksplit(N, K);
    if (ks > 1 && workspace) {
      if (reinterpret_cast<uintptr_t>(workspace) & 255u) return SPIFFY_EALIGN;
      if (workspace_bytes < sizeof(float) * (size_t)ks * M * N) return SPIFFY_EWORKSPACE;
      g.C = workspace; g.ksplit = ks;
      int rc = dev(launch_gemm_mfma(EPI_PARTIAL, g, st));
      if (rc) return rc;
      return dev(launch_splitk_reduce((const float*)workspace, ks, R, C, nullptr, 0.f, nullptr, M, N, st));
    }
  }
  return dev(mf ? launch_gemm_mfma(epilogue, g, st) : launch_gemm_generic(dtype, epilogue, g, st));
}

int spiffy_gemm_plan(int32_t epilogue, int32_t M, int32_t N, int32_t K, int32_t with_workspace,
                     spiffy_gemm_plan_t* plan) {
  if (!plan || epilogue < SPIFFY_GEMM_STORE || epilogue > SPIFFY_GEMM_SWIGLU) return SPIFFY_EINVAL;
  if (M < 1 || N < 1 || K < 1) return SPIFFY_ESHAPE;
  GemmArgs g;
  std::memset(&g, 0, sizeof(g));
  g.M = M; g.N = N; g.K = K; g.lda = K; g.ldc = N;
  if (epilogue != SPIFFY_GEMM_SWIGLU) g.Nseg[0] = N;
  if (!mfma_gemm_supported(epilogue, g)) return SPIFFY_ESHAPE;
  int epi = epilogue, ks = 1;
  if (epilogue == SPIFFY_GEMM_RESID && with_workspace && mfma_ksplit(N, K) > 1) { epi = EPI_PARTIAL; ks = mfma_ksplit(N, K); }
  const GemmPlan p = plan_gemm_mfma(epi, M, N, ks);
  std::memset(plan, 0, sizeof(*plan));
  plan->n_launches = p.n_parts;
  plan->k_slices = ks;
  for (int i = 0; i < p.n_parts; ++i) {
    plan->launch[i].tile_rows = p.part[i].bm;
    plan->launch[i].tile_cols = p.part[i].bn;
    plan->launch[i].col0 = p.part[i].col0;
    plan->launch[i].n_cols = p.part[i].ncols;
    plan->launch[i].workgroups = p.part[i].workgroups;
  }
  return SPIFFY_OK;
}

int spiffy_graph_accept(const int32_t* graph_edges, int32_t E, const int32_t* draft_states,
                        const int32_t* target_states, int32_t G, int32_t B, int32_t root,
                        spiffy_accept_result* result, int32_t* accepted_state, void* stream) {
  int rc = check_accept_args(graph_edges, E, draft_states, target_states, G, B, root, result);
  if (rc) return rc;
  return dev(launch_graph_accept(graph_edges, E, draft_states, target_states, G, B, root, result, accepted_state,
                                 (hipStream_t)stream));
}

int spiffy_head_topk(const spiffy_model_cfg* cfg, const void* w_vocab, const int32_t* block_tokens, int32_t G,
                     int32_t B, const spiffy_accept_result* result, int32_t node, int32_t K, float logit_scale,
                     int32_t after_step, int32_t* topk_tokens, float* topk_probs, void* workspace,
                     size_t workspace_bytes, void* stream) {
  int rc;
  if ((rc = check_cfg(cfg)) || (rc = check_gb(G, B))) return rc;
  if (!w_vocab || !block_tokens || !topk_tokens || !topk_probs || !workspace) return SPIFFY_EINVAL;
  if (!(logit_scale > 0.f) || !std::isfinite(logit_scale)) return SPIFFY_EINVAL;
  if (!result && (node < 0 || node >= G)) return SPIFFY_EINVAL;
  if (K < 1 || K > SPIFFY_MAX_TOPK) return SPIFFY_ESHAPE;
  if (cfg->dtype == SPIFFY_BF16 && cfg->d % 8 != 0) return SPIFFY_ESHAPE;
  if (!head_shape_ok(cfg)) return SPIFFY_ESHAPE;
  if (!aligned16(w_vocab)) return SPIFFY_EALIGN;
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return SPIFFY_EALIGN;
  // a step keeps its layer / head scratch at the start of its workspace, so the head's leftovers are found at the
  // same place after spiffy_decode_head and after a whole step
  (void)after_step;
  void* head_base = workspace;
  if (workspace_bytes < carve_head(cfg, G, B, nullptr).bytes) return SPIFFY_EWORKSPACE;
  const HeadWs ws = carve_head(cfg, G, B, head_base);
  HeadTopkArgs a;
  a.dtype = cfg->dtype; a.nf = ws.nf; a.w_vocab = w_vocab; a.d = cfg->d; a.V = cfg->vocab; a.scale = logit_scale;
  a.part = ws.part; a.n_part = ws.n_part; a.m_cap = ws.m_cap; a.row_top = ws.row_top; a.row_idx = ws.row_idx;
  a.count = ws.count; a.tokens = block_tokens; a.result = result; a.node = node; a.G = G; a.B = B; a.K = K;
  a.cand_val = ws.cand_val; a.cand_idx = ws.cand_idx; a.out_tokens = topk_tokens; a.out_probs = topk_probs;
  return dev(launch_head_topk(a, (hipStream_t)stream));
}

int spiffy_draft_prune(const int32_t* state, int32_t B, int32_t mask_id, const int32_t* topk_tokens,
                       const float* topk_probs, int32_t K, const int32_t* formula_offsets,
                       const int32_t* formula_pairs, int32_t D, int32_t nnz, const int32_t* edges, int32_t E,
                       int32_t d_star, int32_t* drafts, uint8_t* buildable, float* local, float* score,
                       int32_t* kept, int32_t* states_out, int32_t* edges_out, int32_t* counts, void* stream) {
  if (!state || !topk_tokens || !topk_probs || !formula_offsets || !drafts || !buildable || !local || !score ||
      !kept || !states_out || !counts)
    return SPIFFY_EINVAL;
  if ((nnz > 0 && !formula_pairs) || (E > 0 && (!edges || !edges_out))) return SPIFFY_EINVAL;
  if (B < 1 || B > 4096 || K < 1 || K > 16 || D < 0 || D > SPIFFY_MAX_G - 1 || nnz < 0 || E < 0 || d_star < 0)
    return SPIFFY_ESHAPE;
  DraftPruneArgs a;
  a.state = state; a.topk_tokens = topk_tokens; a.topk_probs = topk_probs;
  a.formula_offsets = formula_offsets; a.formula_pairs = formula_pairs; a.edges = edges;
  a.drafts = drafts; a.buildable = buildable; a.local = local; a.score = score; a.kept = kept;
  a.states_out = states_out; a.edges_out = edges_out; a.counts = counts;
  a.B = B; a.K = K; a.D = D; a.nnz = nnz; a.E = E; a.d_star = d_star; a.mask_id = mask_id;
  return dev(launch_draft_prune(a, (hipStream_t)stream));
}

int spiffy_verify_step(const spiffy_model_cfg* cfg, int32_t n_layers, const spiffy_layer_weights* layers,
                       const spiffy_prefix_kv* prefix, const void* w_embed, const void* final_norm,
                       const void* w_vocab, const int32_t* block_tokens, int32_t G, int32_t B, int32_t pos0,
                       const int32_t* graph_edges, int32_t E, int32_t root, float threshold, float logit_scale,
                       int32_t force_one, void* hidden_out, int32_t* argmax, float* conf, uint8_t* unmask,
                       float* top2_margin, int32_t* target_states, spiffy_accept_result* result,
                       int32_t* accepted_state, void* workspace, size_t workspace_bytes, void* stream) {
  int rc;
  if ((rc = check_cfg(cfg)) || (rc = check_gb(G, B))) return rc;
  if (n_layers < 0 || (n_layers > 0 && (!layers || !prefix)) || !w_embed || !workspace || pos0 < 0)
    return SPIFFY_EINVAL;
  if (!aligned16(w_embed) || (hidden_out && !aligned16(hidden_out)) || (reinterpret_cast<uintptr_t>(workspace) & 255u))
    return SPIFFY_EALIGN;
  int P_max = 0;
  for (int l = 0; l < n_layers; ++l) {
    if ((rc = check_layer_args(cfg, &layers[l], &prefix[l], G, B))) return rc;
    if (prefix[l].P + prefix[l].S > P_max) P_max = prefix[l].P + prefix[l].S;
  }
  if ((rc = check_head_args(cfg, workspace, final_norm, w_vocab, block_tokens, threshold, logit_scale, argmax, conf,
                            unmask)))
    return rc;
  const int32_t* tgt_probe = target_states ? target_states : reinterpret_cast<const int32_t*>(workspace);
  if ((rc = check_accept_args(graph_edges, E, block_tokens, tgt_probe, G, B, root, result))) return rc;
  const StepWs ws = carve_step(cfg, G, B, P_max, workspace);
  if (workspace_bytes < ws.bytes) return SPIFFY_EWORKSPACE;

  hipStream_t st = (hipStream_t)stream;
  void* hid = hidden_out ? hidden_out : ws.hidden;
  int32_t* tgt = target_states ? target_states : ws.target;
  if ((rc = dev(launch_embed(cfg->dtype, w_embed, block_tokens, G * B, cfg->d, cfg->vocab, hid, st)))) return rc;
  LayerChain chain;
  chain.tokens = block_tokens;
  for (int l = 0; l < n_layers; ++l) {
    chain.normed_in = chain.normed_out;
    chain.next_norm1 = (l + 1 < n_layers) ? layers[l + 1].norm1 : nullptr;
    // a caller that does not ask for the hidden states gets the last layer on the masked rows only: the head reads
    // nothing else
    chain.masked_rows_only = !hidden_out && l + 1 == n_layers;
    if ((rc = run_layer(cfg, &layers[l], &prefix[l], hid, G, B, pos0, hid, ws.rest, st, &chain))) return rc;
    chain.rope_ready = true;      // same pos0 / B / base for every layer: the table is computed once
  }
  if ((rc = run_head(cfg, hid, final_norm, w_vocab, block_tokens, nullptr, G, B, threshold, logit_scale, force_one,
                     argmax, conf, unmask, top2_margin, tgt, ws.rest, st)))
    return rc;
  return dev(launch_graph_accept(graph_edges, E, block_tokens, tgt, G, B, root, result, accepted_state, st));
}

size_t spiffy_workspace_bytes_seq(const spiffy_model_cfg* cfg, int32_t G, int32_t B, int32_t S, int32_t P_max) {
  if (check_cfg(cfg) || check_gb(G, B) || P_max < 0 || S < 0 || S > SPIFFY_MAX_SUFFIX) return 0;
  return carve_step(cfg, G, B, P_max, nullptr, S).bytes;
}

int spiffy_verify_step_seq(const spiffy_model_cfg* cfg, int32_t n_layers, const spiffy_layer_weights* layers,
                           const spiffy_prefix_kv* prefix, const void* w_embed, const void* final_norm,
                           const void* w_vocab, const int32_t* block_tokens, const int32_t* suffix_tokens, int32_t G,
                           int32_t B, int32_t S, int32_t pos0, const int32_t* graph_edges, int32_t E, int32_t root,
                           float threshold, float logit_scale, int32_t force_one, void* hidden_out, int32_t* argmax,
                           float* conf, uint8_t* unmask, float* top2_margin, int32_t* target_states,
                           spiffy_accept_result* result, int32_t* accepted_state, void* workspace,
                           size_t workspace_bytes, void* stream) {
  int rc;
  if ((rc = check_cfg(cfg)) || (rc = check_gb(G, B))) return rc;
  if (n_layers < 1 || !layers || !prefix || !w_embed || !workspace || pos0 < 0 || S < 0 || (S > 0 && !suffix_tokens))
    return SPIFFY_EINVAL;
  if (S > SPIFFY_MAX_SUFFIX) return SPIFFY_ESHAPE;
  if (!aligned16(w_embed) || (hidden_out && !aligned16(hidden_out)) || (reinterpret_cast<uintptr_t>(workspace) & 255u))
    return SPIFFY_EALIGN;
  int P_max = 0;
  for (int l = 0; l < n_layers; ++l) {
    if ((rc = check_layer_args(cfg, &layers[l], &prefix[l], G, B))) return rc;
    if (prefix[l].S != 0) return SPIFFY_EINVAL;                       // the suffix is computed here, not cached
    if (S > 0) {
      if (!prefix[l].k || !prefix[l].v) return SPIFFY_EINVAL;         // rows behind the prefix are written
      if ((int64_t)prefix[l].P + B + S > prefix[l].capacity) return SPIFFY_ESHAPE;
      if (!layer_mfma(cfg) && generic_attn_smem(cfg, S, prefix[l].P + B + S) > kMaxGenericSmem) return SPIFFY_ESHAPE;
    }
    if (prefix[l].P > P_max) P_max = prefix[l].P;
  }
  if ((rc = check_head_args(cfg, workspace, final_norm, w_vocab, block_tokens, threshold, logit_scale, argmax, conf,
                            unmask)))
    return rc;
  const int32_t* tgt_probe = target_states ? target_states : reinterpret_cast<const int32_t*>(workspace);
  if ((rc = check_accept_args(graph_edges, E, block_tokens, tgt_probe, G, B, root, result))) return rc;
  const StepWs ws = carve_step(cfg, G, B, P_max, workspace, S);
  if (workspace_bytes < ws.bytes) return SPIFFY_EWORKSPACE;

  hipStream_t st = (hipStream_t)stream;
  void* hid = hidden_out ? hidden_out : ws.hidden;
  int32_t* tgt = target_states ? target_states : ws.target;
  if ((rc = dev(launch_embed(cfg->dtype, w_embed, block_tokens, G * B, cfg->d, cfg->vocab, hid, st)))) return rc;
  if (S > 0) {
    void* hid_seq = reinterpret_cast<char*>(hid) + (size_t)G * B * cfg->d * esize(cfg->dtype);
    if ((rc = dev(launch_embed(cfg->dtype, w_embed, suffix_tokens, S, cfg->d, cfg->vocab, hid_seq, st)))) return rc;
  }
  LayerChain chain;
  chain.seq_S = S;
  for (int l = 0; l < n_layers; ++l) {
    chain.normed_in = chain.normed_out;
    chain.next_norm1 = (l + 1 < n_layers) ? layers[l + 1].norm1 : nullptr;
    if ((rc = run_layer(cfg, &layers[l], &prefix[l], hid, G, B, pos0, hid, ws.rest, st, &chain))) return rc;
    chain.rope_ready = true;
    chain.rope_ready_seq = true;
  }
  if ((rc = run_head(cfg, hid, final_norm, w_vocab, block_tokens, nullptr, G, B, threshold, logit_scale, force_one,
                     argmax, conf, unmask, top2_margin, tgt, ws.rest, st)))
    return rc;
  return dev(launch_graph_accept(graph_edges, E, block_tokens, tgt, G, B, root, result, accepted_state, st));
}

size_t spiffy_workspace_bytes_commit(const spiffy_model_cfg* cfg, int32_t G, int32_t B, int32_t P_max) {
  if (check_cfg(cfg) || check_gb(G, B) || check_gb(G + 1, B) || P_max < 0) return 0;
  return carve_step(cfg, G, B, P_max, nullptr, B).bytes;
}

int spiffy_verify_step_commit(const spiffy_model_cfg* cfg, int32_t n_layers, const spiffy_layer_weights* layers,
                              const spiffy_prefix_kv* prefix, const void* w_embed, const void* final_norm,
                              const void* w_vocab, const int32_t* prev_block_tokens, const int32_t* block_tokens,
                              int32_t G, int32_t B, int32_t pos0, const int32_t* graph_edges, int32_t E, int32_t root,
                              float threshold, float logit_scale, int32_t force_one, void* hidden_out, int32_t* argmax,
                              float* conf, uint8_t* unmask, float* top2_margin, int32_t* target_states,
                              spiffy_accept_result* result, int32_t* accepted_state, void* workspace,
                              size_t workspace_bytes, void* stream) {
  int rc;
  if ((rc = check_cfg(cfg)) || (rc = check_gb(G, B)) || (rc = check_gb(G + 1, B))) return rc;
  if (n_layers < 1 || !layers || !prefix || !w_embed || !workspace || !prev_block_tokens || pos0 < B) return SPIFFY_EINVAL;
  if (!aligned16(w_embed) || (hidden_out && !aligned16(hidden_out)) || (reinterpret_cast<uintptr_t>(workspace) & 255u))
    return SPIFFY_EALIGN;
  int P_max = 0;
  for (int l = 0; l < n_layers; ++l) {
    if ((rc = check_layer_args(cfg, &layers[l], &prefix[l], G, B))) return rc;
    if (!prefix[l].k || !prefix[l].v) return SPIFFY_EINVAL;            // the finished block's rows are written
    const int cap = prefix[l].capacity ? prefix[l].capacity : prefix[l].P;
    if ((int64_t)prefix[l].P + B > cap) return SPIFFY_ESHAPE;
    if (!layer_mfma(cfg) && generic_attn_smem(cfg, B, prefix[l].P + B + prefix[l].S) > kMaxGenericSmem) return SPIFFY_ESHAPE;
    if (prefix[l].P + prefix[l].S > P_max) P_max = prefix[l].P + prefix[l].S;
  }
  if ((rc = check_head_args(cfg, workspace, final_norm, w_vocab, block_tokens, threshold, logit_scale, argmax, conf,
                            unmask)))
    return rc;
  const int32_t* tgt_probe = target_states ? target_states : reinterpret_cast<const int32_t*>(workspace);
  if ((rc = check_accept_args(graph_edges, E, block_tokens, tgt_probe, G, B, root, result))) return rc;
  const StepWs ws = carve_step(cfg, G, B, P_max, workspace, B);
  if (workspace_bytes < ws.bytes) return SPIFFY_EWORKSPACE;

  hipStream_t st = (hipStream_t)stream;
  void* hid = hidden_out ? hidden_out : ws.hidden;
  int32_t* tgt = target_states ? target_states : ws.target;
  void* hid_prev = reinterpret_cast<char*>(hid) + (size_t)G * B * cfg->d * esize(cfg->dtype);
  if ((rc = dev(launch_embed(cfg->dtype, w_embed, block_tokens, G * B, cfg->d, cfg->vocab, hid, st)))) return rc;
  if ((rc = dev(launch_embed(cfg->dtype, w_embed, prev_block_tokens, B, cfg->d, cfg->vocab, hid_prev, st)))) return rc;
  LayerChain chain;
  chain.seq_S = B;
  chain.tail_is_prev_block = true;
  for (int l = 0; l < n_layers; ++l) {
    chain.normed_in = chain.normed_out;
    chain.next_norm1 = (l + 1 < n_layers) ? layers[l + 1].norm1 : nullptr;
    if ((rc = run_layer(cfg, &layers[l], &prefix[l], hid, G, B, pos0, hid, ws.rest, st, &chain))) return rc;
    chain.rope_ready = true;
    chain.rope_ready_seq = true;
  }
  if ((rc = run_head(cfg, hid, final_norm, w_vocab, block_tokens, nullptr, G, B, threshold, logit_scale, force_one,
                     argmax, conf, unmask, top2_margin, tgt, ws.rest, st)))
    return rc;
  return dev(launch_graph_accept(graph_edges, E, block_tokens, tgt, G, B, root, result, accepted_state, st));
}

int spiffy_commit_block(const spiffy_model_cfg* cfg, int32_t n_layers, const spiffy_layer_weights* layers,
                        const spiffy_prefix_kv* prefix, const void* w_embed, const int32_t* block_tokens, int32_t B,
                        int32_t pos0, void* workspace, size_t workspace_bytes, void* stream) {
  int rc;
  if ((rc = check_cfg(cfg)) || (rc = check_gb(1, B))) return rc;
  if (n_layers < 1 || !layers || !prefix || !w_embed || !block_tokens || !workspace || pos0 < 0)
    return SPIFFY_EINVAL;
  if (!aligned16(w_embed)) return SPIFFY_EALIGN;
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return SPIFFY_EALIGN;
  int P_max = 0;
  for (int l = 0; l < n_layers; ++l) {
    if ((rc = check_layer_args(cfg, &layers[l], &prefix[l], 1, B))) return rc;
    if (!prefix[l].k || !prefix[l].v) return SPIFFY_EINVAL;
    const int cap = prefix[l].capacity ? prefix[l].capacity : prefix[l].P;
    if ((int64_t)prefix[l].P + B > cap) return SPIFFY_ESHAPE;      // no room for the block's rows
    if (prefix[l].P + prefix[l].S > P_max) P_max = prefix[l].P + prefix[l].S;
  }
  const StepWs ws = carve_step(cfg, 1, B, P_max, workspace);
  if (workspace_bytes < ws.bytes) return SPIFFY_EWORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  if ((rc = dev(launch_embed(cfg->dtype, w_embed, block_tokens, B, cfg->d, cfg->vocab, ws.hidden, st)))) return rc;
  LayerChain chain;
  chain.append_kv = true;
  for (int l = 0; l < n_layers; ++l) {
    chain.normed_in = chain.normed_out;
    chain.next_norm1 = (l + 1 < n_layers) ? layers[l + 1].norm1 : nullptr;
    if ((rc = run_layer(cfg, &layers[l], &prefix[l], ws.hidden, 1, B, pos0, ws.hidden, ws.rest, st, &chain))) return rc;
    chain.rope_ready = true;
  }
  return SPIFFY_OK;
}

size_t spiffy_subgraph_search_workspace_bytes(void) { return subgraph_search_workspace_bytes(); }

int spiffy_subgraph_search(const int64_t* count, const int32_t* level, int32_t N, const int32_t* edges, int32_t E,
                           int32_t D, uint64_t* best_mask, int64_t* best_sum, uint64_t* n_connected,
                           int32_t* nodes_out, void* workspace, size_t workspace_bytes, void* stream) {
  if (!count || !level || !best_mask || !best_sum || !n_connected || !workspace || (E > 0 && !edges))
    return SPIFFY_EINVAL;
  if (N < 1 || N > 64 || D < 1 || D > 64 || E < 0) return SPIFFY_ESHAPE;
  // C(N, D) sets are tried one by one: refuse what would run for minutes
  unsigned long long total = 1;
  if (D > N) {
    total = 0;
  } else {
    const int k = D < N - D ? D : N - D;
    for (int i = 1; i <= k; ++i) {
      total = total * (unsigned long long)(N - k + i) / (unsigned long long)i;     // exact: a product of i consecutive integers
      if (total > SPIFFY_SUBGRAPH_MAX_SETS) return SPIFFY_ESHAPE;
    }
  }
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return SPIFFY_EALIGN;
  if (workspace_bytes < subgraph_search_workspace_bytes()) return SPIFFY_EWORKSPACE;
  SubgraphArgs a;
  a.count = count; a.level = level; a.edges = edges; a.N = N; a.E = E; a.D = D; a.total_sets = total;
  a.best_mask = best_mask; a.best_sum = best_sum; a.n_connected = n_connected; a.nodes_out = nodes_out;
  a.workspace = workspace;
  return dev(launch_subgraph_search(a, (hipStream_t)stream));
}

#pragma GCC visibility pop
}  // extern "C"

"""CPU oracle for the draft-graph verification step of Spiffy (arxiv 2509.18085).

TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, fp64 definition of what the
GPU library computes.  Only the tests, the smoke check and the benchmark's CPU-baseline
leg may import it; the product (the HIP library and its Python binding) never does, and
this file imports nothing from the product.  It shares no code, table or helper with
the HIP path.

Everything is written as the definition reads, one draft at a time, one head at a time,
in float64 (inputs that are bf16 on the GPU arrive here as the same values widened).
numpy's matrix product is used as a library step; there is no blocking, fusion, caching
trick or reordering.

What the paper fixes and where:
  * batched verification = the model evaluated on (context ; one state of the block) for
    the true state and every draft, all in one call                       Sec. 4.3, Eqs. (2),(3)
  * a draft block attends to itself and to the true context, never to another draft or to
    the block it drafts for; attention inside a block is bidirectional    Fig. 4 caption
  * keys/values of everything before the block are cached and fixed       Sec. 3.1 (prefix caching)
  * exactness holds with fixed context KV / blockwise-causal context      Sec. 4.3, App. A.2
  * dual cache: the fixed context also holds the tokens after the block   Sec. 4.3, App. A.2
  * full-sequence models with a prefix cache only: the true sequence (block ; suffix) is
    recomputed in the call and attends to itself; a draft block attends to the context, to
    itself and to the true suffix, not to the block it drafts for           Sec. 4.3, Fig. 4, App. A.2
  * Next(X, p): per-position top-1 probability and token, unmask the chosen positions
                                                                          Alg. 1 steps 1-4, App. A
  * threshold rule: unmask every masked position whose top-1 probability exceeds tau
                                                                          Sec. 3.1
  * acceptance walk over children of the last accepted node               Alg. 1 step 5, Eqs. (4)-(6)
  * the accepted draft's own distribution (same forward pass) yields the next state
                                                                          App. A, case 2
  * draft blocks = current block + tokens c_ij named by draft formulas {(i, j)}, i = token
    position rank, j = vocabulary rank                                    Sec. 4.4.2, 4.4.3
  * pruning score: geometric means of token probabilities, of the children's local scores,
    and of the two                                                        Sec. 4.4.4
  * calibration, optimal subgraph: among all size-D node sets of the candidate graph in which
    every node is of level 1 or 2 or has a parent in the set, the one with the largest total
    count                                                                 Alg. 2 part 3, App. D.1

Readings taken where the paper is silent (architecture details are not in the paper at
all; the shapes come from the workload configurations):
  pre-norm RMSNorm with learnable gain, rotary embedding with rotate-half pairing
  (i, i+hd/2) and angle pos * base^(-2i/hd), SwiGLU FFN, optional QKV bias, untied
  embedding / vocabulary matrices; every one of the G blocks sits at positions
  pos0 .. pos0+B-1; only still-masked positions may be unmasked; ties go to the lowest
  index; the threshold comparison is strict ">" on the float32 value of the confidence;
  if no masked position of a state exceeds tau and force_one is set, the single
  highest-confidence masked position is unmasked (progress guarantee needed by Alg. 1).

Pins (tests/test_oracle_pins.py): closed forms, rotary invariances, agreement of the
cached formulation with a dense-mask single-sequence formulation (two independent
formulations of Sec. 4.3), torch's CPU scaled-dot-product attention, brute-force
enumeration of all walks on small graphs, the losslessness theorem on a tiny model; for
drafting and pruning a hand-worked example, an independent loop implementation on exact
fractions, the graph conditions of Eqs. (4)-(6), and the link to Next(X, p): the formula
"ranks 1..s, vocabulary rank 1" reproduces the threshold rule's next state and is accepted;
for the dual cache (tests/test_oracle_suffix_pins.py) the mean-of-values closed form over
P + B + S rows, torch's attention, the block rows of a full bidirectional one-layer forward,
the dense-mask formulation with the suffix in the context, and a scalar brute force; for the
full-sequence step (tests/test_oracle_fullseq_pins.py) the dense-mask single-sequence
formulation, the reduction to a plain cached forward for one state, and draft isolation; for the
subgraph search (tests/test_oracle_subgraph_pins.py) a hand-worked example, the paper's
breadth-first growth from the root levels as a second formulation, and closed forms for the
number of connected sets and the optimum on structured graphs.
No function here is "parity unpinned".
"""
from __future__ import annotations

from typing import Callable, Dict, List, Optional, Sequence, Tuple

import numpy as np

F64 = np.float64


# ----------------------------------------------------------------------------------------
# elementwise pieces
# ----------------------------------------------------------------------------------------

def rms_norm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """Row-wise x / sqrt(mean(x^2) + eps) * gain."""
    x = np.asarray(x, F64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(gain, F64)


def rope(x: np.ndarray, positions: np.ndarray, base: float) -> np.ndarray:
    """Rotary embedding on the last axis (size hd) of x[..., T, hd]; positions[T].
    Pair (i, i + hd/2) is rotated by angle pos * base^(-2 i / hd)."""
    x = np.asarray(x, F64)
    hd = x.shape[-1]
    half = hd // 2
    i = np.arange(half, dtype=F64)
    inv_freq = base ** (-2.0 * i / hd)
    ang = np.asarray(positions, F64)[:, None] * inv_freq[None, :]      # [T, half]
    c, s = np.cos(ang), np.sin(ang)
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def softmax_rows(s: np.ndarray) -> np.ndarray:
    s = s - np.max(s, axis=-1, keepdims=True)
    e = np.exp(s)
    return e / np.sum(e, axis=-1, keepdims=True)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round to the nearest bfloat16 (ties to even), returned as float64.  Used only where a
    float decides an integer and the GPU kernel's operand precision has to be mirrored."""
    b = np.ascontiguousarray(np.asarray(x, np.float32)).view(np.uint32).astype(np.uint64)
    b = ((b + 0x7FFF + ((b >> 16) & 1)) >> 16) << 16
    return b.astype(np.uint32).view(np.float32).astype(F64).reshape(np.shape(x))


def _w(d: Dict, k: str) -> Optional[np.ndarray]:
    v = d.get(k)
    return None if v is None else np.asarray(v, F64)


# ----------------------------------------------------------------------------------------
# O1: one transformer layer over G independent block states with a shared cached prefix
# ----------------------------------------------------------------------------------------

def verify_layer(w: Dict[str, np.ndarray], prefix_k: np.ndarray, prefix_v: np.ndarray,
                 hidden_in: np.ndarray, *, n_q_heads: int, n_kv_heads: int, head_dim: int,
                 pos0: int, rms_eps: float = 1e-5, rope_base: float = 10000.0,
                 return_kv: bool = False, suffix_k: Optional[np.ndarray] = None,
                 suffix_v: Optional[np.ndarray] = None):
    """hidden_in [G,B,d] -> hidden_out [G,B,d].

    Each g is processed on its own (that independence is the attention mask of Fig. 4):
    block rows attend to the P cached prefix keys followed by the B keys of their own
    block, bidirectionally.  prefix_k / prefix_v are [Hkv, P, hd]; prefix_k is already
    rotated at positions 0..P-1.  The block sits at positions pos0..pos0+B-1 for every g
    (Sec. 4.3, "appropriate positional embeddings").

    suffix_k / suffix_v [Hkv, S, hd] (dual cache, Sec. 4.3 / App. A.2): fixed keys / values of
    the S true-sequence tokens after the block, suffix_k already rotated at positions
    pos0+B .. pos0+B+S-1.  Every block, true or draft, attends to them as it attends to the
    prefix (Fig. 4 caption: all blocks of the true sequence except the one drafted for).
    """
    x_all = np.asarray(hidden_in, F64)
    G, B, d = x_all.shape
    Hq, Hkv, hd = n_q_heads, n_kv_heads, head_dim
    rep = Hq // Hkv
    pk, pv = np.asarray(prefix_k, F64), np.asarray(prefix_v, F64)
    wq, wk, wv, wo = _w(w, "wq"), _w(w, "wk"), _w(w, "wv"), _w(w, "wo")
    wg, wu, wd = _w(w, "w_gate"), _w(w, "w_up"), _w(w, "w_down")
    bq, bk, bv = _w(w, "bq"), _w(w, "bk"), _w(w, "bv")
    pos = pos0 + np.arange(B)
    out = np.empty_like(x_all)
    ks, vs = [], []
    if suffix_k is None:
        sk, sv = np.zeros((Hkv, 0, hd), F64), np.zeros((Hkv, 0, hd), F64)
    else:
        sk, sv = np.asarray(suffix_k, F64), np.asarray(suffix_v, F64)
    for g in range(G):
        x = x_all[g]                                            # [B, d]
        n = rms_norm(x, w["norm1"], rms_eps)
        q = n @ wq.T
        k = n @ wk.T
        v = n @ wv.T
        if bq is not None:
            q = q + bq
        if bk is not None:
            k = k + bk
        if bv is not None:
            v = v + bv
        q = rope(q.reshape(B, Hq, hd).transpose(1, 0, 2), pos, rope_base)    # [Hq,B,hd]
        k = rope(k.reshape(B, Hkv, hd).transpose(1, 0, 2), pos, rope_base)   # [Hkv,B,hd]
        v = v.reshape(B, Hkv, hd).transpose(1, 0, 2)
        o = np.empty((B, Hq, hd), F64)
        for h in range(Hq):
            kvh = h // rep
            keys = np.concatenate([pk[kvh], k[kvh], sk[kvh]], axis=0)    # [P+B+S, hd]
            vals = np.concatenate([pv[kvh], v[kvh], sv[kvh]], axis=0)
            s = (q[h] @ keys.T) / np.sqrt(float(hd))            # [B, P+B+S]
            p = softmax_rows(s)
            o[:, h, :] = p @ vals
        h1 = x + o.reshape(B, Hq * hd) @ wo.T
        n2 = rms_norm(h1, w["norm2"], rms_eps)
        y = h1 + (silu(n2 @ wg.T) * (n2 @ wu.T)) @ wd.T
        out[g] = y
        ks.append(k)
        vs.append(v)
    if return_kv:
        return out, np.stack(ks), np.stack(vs)
    return out


def embed(w_embed: np.ndarray, block_tokens: np.ndarray) -> np.ndarray:
    """hidden[g,b,:] = W_emb[block_tokens[g,b], :]; masked positions carry the MASK id's row."""
    return np.asarray(w_embed, F64)[np.asarray(block_tokens)]


# ----------------------------------------------------------------------------------------
# O2: LM head -> top-1 token, confidence, threshold-unmask decision, next state
# ----------------------------------------------------------------------------------------

def decode_head(hidden: np.ndarray, final_norm: np.ndarray, w_vocab: np.ndarray,
                block_tokens: np.ndarray, mask_id: int, threshold: float, *,
                rms_eps: float = 1e-5, logit_scale: float = 1.0, force_one: bool = True,
                operand_dtype: Optional[str] = None):
    """Alg. 1 steps 1-4 with the threshold rule of Sec. 3.1, for every one of the G states.

    operand_dtype="bf16" rounds the normalised hidden row to bfloat16 before the vocabulary
    product.  The argmax / threshold decisions are integers decided by floats, so when the
    GPU path is compared in its bf16 configuration both sides take that decision from
    operands of the same precision (the kernel's matrix-core operands are bf16); with None the
    row stays float64 (the fp32 configuration and every pin).

    Returns (argmax [G,B] int32, conf [G,B] float32, unmask [G,B] uint8,
             margin [G,B] float64, target_states [G,B] int32).
    At positions that are not masked: argmax = the token already there, conf = 0,
    unmask = 0, margin = +inf (they never compete, they keep their token).
    """
    hid = np.asarray(hidden, F64)
    G, B, d = hid.shape
    tok = np.asarray(block_tokens)
    wv = np.asarray(w_vocab, F64)
    amax = tok.astype(np.int32).copy()
    conf = np.zeros((G, B), np.float32)
    unmask = np.zeros((G, B), np.uint8)
    margin = np.full((G, B), np.inf, F64)
    tau32 = np.float32(threshold)
    for g in range(G):
        masked_pos = np.nonzero(tok[g] == mask_id)[0]
        if masked_pos.size:
            n = rms_norm(hid[g, masked_pos], final_norm, rms_eps)   # [n_masked, d]
            if operand_dtype == "bf16":
                n = round_to_bf16(n)
            logits_all = logit_scale * (n @ wv.T)                   # [n_masked, V], Alg. 1 step 1
        for r, b in enumerate(masked_pos):
            logits = logits_all[r]
            j = int(np.argmax(logits))                          # lowest index on ties
            p_top = 1.0 / np.sum(np.exp(logits - logits[j]))    # = max_v softmax(logits)_v
            rest = np.delete(logits, j)
            amax[g, b] = j
            conf[g, b] = np.float32(p_top)
            margin[g, b] = logits[j] - (np.max(rest) if rest.size else -np.inf)
            unmask[g, b] = 1 if conf[g, b] > tau32 else 0
        masked = np.nonzero(tok[g] == mask_id)[0]
        if force_one and masked.size and not unmask[g, masked].any():
            best = masked[int(np.argmax(conf[g, masked]))]      # lowest index on ties
            unmask[g, best] = 1
    target = np.where(unmask == 1, amax, tok).astype(np.int32)
    return amax, conf, unmask, margin, target


# ----------------------------------------------------------------------------------------
# O3: acceptance walk over the draft graph
# ----------------------------------------------------------------------------------------

def graph_accept(edges: np.ndarray, draft_states: np.ndarray, target_states: np.ndarray,
                 root: int = 0):
    """Alg. 1 step 5.  Node ``root`` is the current true state; target_states[n] is
    Next(state n, distribution computed for state n).  Starting at the root, move to a
    child (by the given edge list only) whose draft state equals the current node's
    target state in all B positions; repeat from there; stop when no child matches.
    Several matching children are necessarily copies of one state: the lowest id is taken.

    Returns (node, depth, n_steps, accepted_state[B]) with n_steps = depth + 1 decode
    steps covered by this one forward pass.
    """
    e = np.asarray(edges).reshape(-1, 2)
    ds, ts = np.asarray(draft_states), np.asarray(target_states)
    G = ds.shape[0]
    cur, depth = int(root), 0
    seen = {cur}
    while depth < G:
        cand = sorted(int(c) for p, c in e
                      if int(p) == cur and np.array_equal(ds[int(c)], ts[cur]))
        cand = [c for c in cand if c not in seen]
        if not cand:
            break
        cur = cand[0]
        seen.add(cur)
        depth += 1
    return cur, depth, depth + 1, ts[cur].astype(np.int32).copy()


# ----------------------------------------------------------------------------------------
# whole step (all layers, head, walk)
# ----------------------------------------------------------------------------------------

def verify_step(layers: Sequence[Dict], prefix: Sequence[Tuple[np.ndarray, np.ndarray]],
                w_embed, final_norm, w_vocab, block_tokens, edges, *, n_q_heads, n_kv_heads,
                head_dim, pos0, mask_id, threshold, rms_eps=1e-5, rope_base=10000.0,
                logit_scale=1.0, force_one=True, root=0, suffix=None):
    """suffix: None, or per layer (suffix_k, suffix_v) of the dual cache."""
    h = embed(w_embed, block_tokens)
    for l, (w, (pk, pv)) in enumerate(zip(layers, prefix)):
        sk, sv = suffix[l] if suffix is not None else (None, None)
        h = verify_layer(w, pk, pv, h, n_q_heads=n_q_heads, n_kv_heads=n_kv_heads,
                         head_dim=head_dim, pos0=pos0, rms_eps=rms_eps, rope_base=rope_base,
                         suffix_k=sk, suffix_v=sv)
    amax, conf, unmask, margin, target = decode_head(
        h, final_norm, w_vocab, block_tokens, mask_id, threshold, rms_eps=rms_eps,
        logit_scale=logit_scale, force_one=force_one)
    node, depth, n_steps, state = graph_accept(edges, block_tokens, target, root)
    return dict(hidden=h, argmax=amax, conf=conf, unmask=unmask, margin=margin,
                target_states=target, node=node, depth=depth, n_steps=n_steps,
                accepted_state=state)


# ----------------------------------------------------------------------------------------
# O4: second, independent formulation used only to pin O1: ONE token sequence, explicit
# position ids, explicit dense boolean attention mask (the paper's own construction)
# ----------------------------------------------------------------------------------------

def masked_forward(layers: Sequence[Dict], x: np.ndarray, positions: np.ndarray,
                   allow: np.ndarray, *, n_q_heads: int, n_kv_heads: int, head_dim: int,
                   rms_eps: float = 1e-5, rope_base: float = 10000.0):
    """Plain transformer over one sequence x[T,d] with position ids and a dense boolean
    mask allow[T,T] (True = row may attend to column).  Returns (hidden per layer boundary
    [L+1][T,d], rotated K per layer [L][Hkv,T,hd], V per layer)."""
    x = np.asarray(x, F64)
    T = x.shape[0]
    Hq, Hkv, hd = n_q_heads, n_kv_heads, head_dim
    rep = Hq // Hkv
    hs, Ks, Vs = [x], [], []
    for w in layers:
        n = rms_norm(x, w["norm1"], rms_eps)
        q = n @ _w(w, "wq").T
        k = n @ _w(w, "wk").T
        v = n @ _w(w, "wv").T
        if w.get("bq") is not None:
            q = q + _w(w, "bq")
        if w.get("bk") is not None:
            k = k + _w(w, "bk")
        if w.get("bv") is not None:
            v = v + _w(w, "bv")
        q = rope(q.reshape(T, Hq, hd).transpose(1, 0, 2), positions, rope_base)
        k = rope(k.reshape(T, Hkv, hd).transpose(1, 0, 2), positions, rope_base)
        v = v.reshape(T, Hkv, hd).transpose(1, 0, 2)
        o = np.empty((T, Hq, hd), F64)
        for h in range(Hq):
            s = (q[h] @ k[h // rep].T) / np.sqrt(float(hd))
            s = np.where(allow, s, -np.inf)
            o[:, h, :] = softmax_rows(s) @ v[h // rep]
        h1 = x + o.reshape(T, Hq * hd) @ _w(w, "wo").T
        n2 = rms_norm(h1, w["norm2"], rms_eps)
        x = h1 + (silu(n2 @ _w(w, "w_gate").T) * (n2 @ _w(w, "w_up").T)) @ _w(w, "w_down").T
        hs.append(x)
        Ks.append(k)
        Vs.append(v)
    return hs, Ks, Vs


def verification_mask(P: int, B: int, G: int, S: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """Dense mask and position ids of the single-sequence formulation
    [prefix ; block_0 ; ... ; block_{G-1} ; suffix] (Fig. 4 caption, with fixed context KV):
    context rows (prefix and the S suffix tokens after the block) see the context only; the
    rows of block g see the context and block g.  Every block reuses positions P..P+B-1;
    the suffix sits at P+B..P+B+S-1."""
    T = P + G * B + S
    ctx = np.zeros(T, bool)
    ctx[:P] = True
    ctx[P + G * B:] = True
    allow = np.zeros((T, T), bool)
    allow[np.ix_(ctx, ctx)] = True
    for g in range(G):
        r = slice(P + g * B, P + (g + 1) * B)
        allow[r, ctx] = True
        allow[r, r] = True
    pos = np.concatenate([np.arange(P)] + [P + np.arange(B)] * G + [P + B + np.arange(S)])
    return allow, pos


# ----------------------------------------------------------------------------------------
# block decode loops, used only for the losslessness pin (Theorem, App. A)
# ----------------------------------------------------------------------------------------

Drafter = Callable[[np.ndarray, Dict], Tuple[np.ndarray, np.ndarray]]


def decode_block(model: Dict, block0: np.ndarray, *, drafter: Optional[Drafter] = None,
                 max_steps: int = 1000):
    """Decode one block to completion.  ``model`` holds layers, prefix, w_embed,
    final_norm, w_vocab and the keyword settings of ``verify_step``.

    With a "suffix_tokens" entry the forward is that of a full-sequence model (the tokens after the
    block are recomputed in every pass).
    drafter=None: vanilla loop, one forward per state (G=1, no edges).
    drafter(state, info): returns (draft_states [D,B], edges [E,2] over nodes 0..D with
    node 0 = the true state) to be verified together with the true state.

    Returns (final_state, trajectory = list of states after every forward, NFE,
             list of accepted depths, list of forwards saved per call).
    An accepted draft that has no MASK left saves nothing (its next state is itself and
    the vanilla loop would have stopped there too), so "saved" is the depth minus one in
    that case; otherwise saved == depth.
    """
    kw = model["kw"]
    state = np.asarray(block0, np.int32).copy()
    traj, depths, saved, nfe = [state.copy()], [], [], 0
    info: Dict = {}
    while (state == kw["mask_id"]).any() and nfe < max_steps:
        if drafter is None:
            states, edges = state[None, :], np.zeros((0, 2), np.int32)
        else:
            dr, edges = drafter(state, info)
            states = np.concatenate([state[None, :], np.asarray(dr, np.int32).reshape(-1, state.size)])
        if "suffix_tokens" in model:      # full-sequence model with a prefix cache only (Sec. 4.3)
            r = verify_step_fullseq(model["layers"], model["prefix"], model["w_embed"], model["final_norm"],
                                    model["w_vocab"], states, model["suffix_tokens"], edges, **kw)
        else:
            r = verify_step(model["layers"], model["prefix"], model["w_embed"], model["final_norm"],
                            model["w_vocab"], states, edges, **kw)
        nfe += 1
        depths.append(r["depth"])
        vacuous = r["depth"] > 0 and not (states[r["node"]] == kw["mask_id"]).any()
        saved.append(r["depth"] - (1 if vacuous else 0))
        state = r["accepted_state"]
        info = r
        traj.append(state.copy())
    return state, traj, nfe, depths, saved


# ----------------------------------------------------------------------------------------
# drafting from the current distribution and pruning of the draft graph (Sec. 4.4)
# ----------------------------------------------------------------------------------------

def head_topk(hidden: np.ndarray, final_norm: np.ndarray, w_vocab: np.ndarray, k: int, *,
              rms_eps: float, logit_scale: float = 1.0, operand_dtype: str = "f64"
              ) -> Tuple[np.ndarray, np.ndarray]:
    """Drafting source (Sec. 4.4.2): for every position of one block, the k most likely
    tokens of the current distribution and their probabilities, most likely first
    (the vocabulary sort that defines the vocabulary rank j; ties go to the lowest token id).

    hidden [B,d] -> (tokens [B,k] int32, probs [B,k] float64).
    """
    h = rms_norm(np.asarray(hidden, F64), final_norm, rms_eps)
    if operand_dtype == "bf16":
        h = round_to_bf16(h)
    logits = logit_scale * (h @ np.asarray(w_vocab, F64).T)
    p = softmax_rows(logits)
    B, V = p.shape
    tok = np.zeros((B, k), np.int32)
    pr = np.zeros((B, k), F64)
    for b in range(B):
        order = sorted(range(V), key=lambda v: (-logits[b, v], v))[:k]
        tok[b] = order
        pr[b] = p[b, order]
    return tok, pr


def position_order(state: np.ndarray, mask_id: int, conf: np.ndarray) -> List[int]:
    """Token position sort (Sec. 4.4.2, first relation): the still-masked positions of the
    block, most confident first.  position_order(...)[i-1] is the position whose token
    position rank is i.  Reading: only masked positions are candidates for unmasking; equal
    confidences go to the lower position."""
    masked = [b for b in range(len(state)) if int(state[b]) == mask_id]
    return sorted(masked, key=lambda b: (-float(conf[b]), b))


def geometric_mean(values: Sequence[float]) -> float:
    """GM(v_1..v_k) = (prod v)^(1/k) (Sec. 4.4.4)."""
    v = [float(x) for x in values]
    assert len(v) > 0
    if min(v) <= 0.0:
        return 0.0
    return float(np.exp(np.mean(np.log(np.asarray(v, F64)))))


def draft_and_prune(state: np.ndarray, mask_id: int, topk_tokens: np.ndarray, topk_probs: np.ndarray,
                    formulas: Sequence[Sequence[Tuple[int, int]]], edges: np.ndarray, d_star: int) -> Dict:
    """Build the draft blocks of a draft graph from the current distribution and prune the
    graph to a budget (Sec. 4.4.2 and 4.4.4).

    state        [B]    the current block X_k(t) (mask_id where masked)
    topk_tokens  [B,K]  c_{.j}: the K most likely tokens per position, most likely first
    topk_probs   [B,K]  their probabilities (column 0 = the confidence max(p_b))
    formulas     D draft formulas, formula m = set of (i, j), 1-based: i = token position rank,
                 j = vocabulary rank.  Node m (1..D) of the graph is the block obtained by
                 unmasking c_ij at the position of rank i for every (i, j) of formula m;
                 node 0 is the current block (empty formula).
    edges        [E,2]  (parent, child) over nodes 0..D
    d_star       number of draft nodes to keep

    Readings (the paper does not say): a formula that names a position rank beyond the number
    of masked positions, a vocabulary rank beyond K, or the same position twice cannot be
    built and is dropped; children(q) for the child score are the buildable children of q in
    `edges`; a node without buildable children scores its local score alone; the D* best
    scores are kept, equal scores in favour of the lower node index; the root is always kept;
    edges whose two ends are kept survive.

    Returns dict: drafts [D+1,B] (row 0 = state, unbuildable rows = state), buildable [D+1] bool,
    local [D+1], child [D+1] (nan where there is none), score [D+1], kept (ascending node
    indices, root first), states [len(kept),B], edges [E',2] renumbered to positions in kept.
    """
    state = np.asarray(state, np.int32)
    B = state.size
    K = int(np.asarray(topk_tokens).shape[1])
    D = len(formulas)
    order = position_order(state, mask_id, np.asarray(topk_probs, F64)[:, 0])
    drafts = np.tile(state, (D + 1, 1))
    buildable = np.zeros(D + 1, bool)
    buildable[0] = True
    local = np.full(D + 1, np.nan, F64)
    for m, formula in enumerate(formulas, start=1):
        pairs = list(formula)
        ranks = [i for i, _ in pairs]
        ok = len(pairs) > 0 and len(set(ranks)) == len(ranks) and all(
            1 <= i <= len(order) and 1 <= j <= K for i, j in pairs)
        if not ok:
            continue
        probs = []
        for i, j in pairs:
            b = order[i - 1]
            drafts[m, b] = int(topk_tokens[b, j - 1])
            probs.append(float(topk_probs[b, j - 1]))
        buildable[m] = True
        local[m] = geometric_mean(probs)                                   # localScore
    edges = np.asarray(edges, np.int64).reshape(-1, 2)
    child = np.full(D + 1, np.nan, F64)
    score = np.full(D + 1, np.nan, F64)
    for m in range(1, D + 1):
        if not buildable[m]:
            continue
        kids = sorted({int(c) for a, c in edges if int(a) == m and 1 <= int(c) <= D and buildable[int(c)]})
        if kids:
            child[m] = geometric_mean([local[c] for c in kids])           # childScore
            score[m] = geometric_mean([local[m], child[m]])               # score
        else:
            score[m] = local[m]
    cand = [m for m in range(1, D + 1) if buildable[m]]
    best = sorted(cand, key=lambda m: (-score[m], m))[:max(0, int(d_star))]
    kept = [0] + sorted(best)
    pos = {m: r for r, m in enumerate(kept)}
    new_edges = [(pos[int(a)], pos[int(c)]) for a, c in edges if int(a) in pos and int(c) in pos]
    return {"order": order, "drafts": drafts, "buildable": buildable, "local": local, "child": child,
            "score": score, "kept": np.asarray(kept, np.int32), "states": drafts[kept],
            "edges": np.asarray(new_edges, np.int32).reshape(-1, 2)}


# ----------------------------------------------------------------------------------------
# offline calibration, part 3: optimal connected subgraph (Alg. 2; App. D.1)
# ----------------------------------------------------------------------------------------

def subgraph_is_connected(nodes: Sequence[int], level: Sequence[int], parents: Sequence[set]) -> bool:
    """App. D.1: a node is connected to the set g if its level is 1 or 2 or one of its parents
    is in g; g is connected if every one of its nodes is."""
    g = set(nodes)
    return all(level[q] in (1, 2) or (parents[q] & g) for q in g)


def subgraph_search(count: Sequence[int], level: Sequence[int], edges: np.ndarray, D: int) -> Dict:
    """G* = argmax over connected node sets Q of size D of sum_{q in Q} count(q) (App. D.1).

    count[q], level[q] (1-based level k of node q_kv) for the N nodes of the candidate graph;
    edges [E,2] rows (p, q): p is a parent of q (rows with an end outside 0..N-1 are ignored).
    Every size-D subset is tried.  Equal sums go to the subset whose bit mask
    sum_q 2^q is smallest.  Returns best_nodes (ascending; empty if no connected set of size D
    exists), best_mask, best_sum (0 if none), n_connected (the size of G')."""
    import itertools
    N = len(count)
    parents = [set() for _ in range(N)]
    for p, q in np.asarray(edges, np.int64).reshape(-1, 2):
        if 0 <= p < N and 0 <= q < N:
            parents[q].add(int(p))
    best, best_mask, best_sum, n_conn = (), 0, 0, 0
    for nodes in itertools.combinations(range(N), D):
        if not subgraph_is_connected(nodes, level, parents):
            continue
        n_conn += 1
        total = sum(int(count[q]) for q in nodes)
        mask = sum(1 << q for q in nodes)
        if n_conn == 1 or total > best_sum or (total == best_sum and mask < best_mask):
            best, best_mask, best_sum = nodes, mask, total
    return dict(best_nodes=list(best), best_mask=best_mask, best_sum=best_sum, n_connected=n_conn)


# ----------------------------------------------------------------------------------------
# full-sequence models with a prefix cache only (Sec. 4.3, Fig. 4, App. A.2)
# ----------------------------------------------------------------------------------------

def _attend(q, keys, vals, head_dim):
    s = (q @ keys.T) / np.sqrt(float(head_dim))
    return softmax_rows(s) @ vals


def verify_layer_fullseq(w: Dict[str, np.ndarray], prefix_k: np.ndarray, prefix_v: np.ndarray,
                         hidden_blocks: np.ndarray, hidden_suffix: np.ndarray, *, n_q_heads: int,
                         n_kv_heads: int, head_dim: int, pos0: int, rms_eps: float = 1e-5,
                         rope_base: float = 10000.0, return_kv: bool = False):
    """One layer of the verification call of a full-sequence bidirectional model that caches only
    the prefix: hidden_blocks [G,B,d] (block 0 = the true block, the others drafts) and
    hidden_suffix [S,d] (the true tokens after the block) -> (out_blocks, out_suffix).

    Fig. 4: the true sequence keeps attending to itself, so the rows of block 0 and of the suffix
    see the cached prefix, block 0 and the suffix; the rows of a draft block see the prefix, their
    own block and the true suffix (all true blocks except the one drafted for).  Block rows sit at
    positions pos0..pos0+B-1 for every g, suffix rows at pos0+B..pos0+B+S-1."""
    xb = np.asarray(hidden_blocks, F64)
    xs = np.asarray(hidden_suffix, F64)
    G, B, d = xb.shape
    S = xs.shape[0]
    Hq, Hkv, hd = n_q_heads, n_kv_heads, head_dim
    rep = Hq // Hkv
    pk, pv = np.asarray(prefix_k, F64), np.asarray(prefix_v, F64)

    def qkv(x, pos):
        n = rms_norm(x, w["norm1"], rms_eps)
        q, k, v = n @ _w(w, "wq").T, n @ _w(w, "wk").T, n @ _w(w, "wv").T
        if _w(w, "bq") is not None:
            q = q + _w(w, "bq")
        if _w(w, "bk") is not None:
            k = k + _w(w, "bk")
        if _w(w, "bv") is not None:
            v = v + _w(w, "bv")
        T = x.shape[0]
        q = rope(q.reshape(T, Hq, hd).transpose(1, 0, 2), pos, rope_base)
        k = rope(k.reshape(T, Hkv, hd).transpose(1, 0, 2), pos, rope_base)
        return q, k, v.reshape(T, Hkv, hd).transpose(1, 0, 2)

    def rest(x, o):
        h1 = x + o @ _w(w, "wo").T
        n2 = rms_norm(h1, w["norm2"], rms_eps)
        return h1 + (silu(n2 @ _w(w, "w_gate").T) * (n2 @ _w(w, "w_up").T)) @ _w(w, "w_down").T

    pos_b = pos0 + np.arange(B)
    pos_s = pos0 + B + np.arange(S)
    qs, ks, vs = qkv(xs, pos_s)                                  # the true suffix
    blocks = [qkv(xb[g], pos_b) for g in range(G)]
    out_b = np.empty_like(xb)
    for g in range(G):
        qg, kg, vg = blocks[g]
        o = np.empty((B, Hq, hd), F64)
        for h in range(Hq):
            c = h // rep
            keys = np.concatenate([pk[c], kg[c], ks[c]], axis=0)
            vals = np.concatenate([pv[c], vg[c], vs[c]], axis=0)
            o[:, h, :] = _attend(qg[h], keys, vals, hd)
        out_b[g] = rest(xb[g], o.reshape(B, Hq * hd))
    _, k0, v0 = blocks[0]                                        # the true block
    o = np.empty((S, Hq, hd), F64)
    for h in range(Hq):
        c = h // rep
        keys = np.concatenate([pk[c], k0[c], ks[c]], axis=0)
        vals = np.concatenate([pv[c], v0[c], vs[c]], axis=0)
        o[:, h, :] = _attend(qs[h], keys, vals, hd)
    out_s = rest(xs, o.reshape(S, Hq * hd)) if S else xs.copy()
    if return_kv:                                                # rotated keys and values of the true block
        return out_b, out_s, k0, v0
    return out_b, out_s


def verify_step_fullseq(layers: Sequence[Dict], prefix: Sequence[Tuple[np.ndarray, np.ndarray]],
                        w_embed, final_norm, w_vocab, block_tokens, suffix_tokens, edges, *,
                        n_q_heads, n_kv_heads, head_dim, pos0, mask_id, threshold, rms_eps=1e-5,
                        rope_base=10000.0, logit_scale=1.0, force_one=True, root=0):
    """The whole step for a full-sequence model: embed, the layers above, the head on the G blocks
    (the suffix is only context), the walk."""
    hb = embed(w_embed, block_tokens)
    hs = embed(w_embed, np.asarray(suffix_tokens).reshape(-1))
    for w, (pk, pv) in zip(layers, prefix):
        hb, hs = verify_layer_fullseq(w, pk, pv, hb, hs, n_q_heads=n_q_heads, n_kv_heads=n_kv_heads,
                                      head_dim=head_dim, pos0=pos0, rms_eps=rms_eps, rope_base=rope_base)
    amax, conf, unmask, margin, target = decode_head(
        hb, final_norm, w_vocab, block_tokens, mask_id, threshold, rms_eps=rms_eps,
        logit_scale=logit_scale, force_one=force_one)
    node, depth, n_steps, state = graph_accept(edges, block_tokens, target, root)
    return dict(hidden=hb, hidden_suffix=hs, argmax=amax, conf=conf, unmask=unmask, margin=margin,
                target_states=target, node=node, depth=depth, n_steps=n_steps, accepted_state=state)

"""Seeded synthetic inputs for the draft-graph verification step.

This module only *makes inputs* (weights, cached prefix KV, hidden states, draft
states, draft graphs, planted target states).  It holds none of the method's
arithmetic: no attention, no projection, no softmax, no acceptance walk.  Both the
CPU oracle's tests and the GPU binding's tests draw their inputs from here, so the
two sides see identical bits without sharing any computation.

Shapes follow the five workload configurations (tiny fp32 case, one LLaDA-8B-shaped
layer, the 32-layer LLaDA-8B-shaped stack, the Dream-7B-shaped GQA stack, and the
SDAR-style small-block long-prefix case).  Trained weights and the paper's datasets
(Sec. 5) are not available; random-init weights N(0, 0.02) and N(0, 1) KV of the
same shapes stand in for them.

A draft state is a block of B token ids where still-masked positions hold
``mask_id`` (Sec. 4.2).  A draft graph is an edge list (parent, child) following
the parent/child relation of Eqs. (4)-(6): the child's unmasked set strictly
contains the parent's.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List, Optional, Tuple

import numpy as np
import torch

DEFAULT_SEED = 20250918


@dataclass(frozen=True)
class Config:
    name: str
    L: int          # layers
    d: int          # model width
    Hq: int         # query heads
    Hkv: int        # key/value heads
    hd: int         # head dim
    F: int          # SwiGLU FFN width
    V: int          # vocabulary
    P: int          # cached prefix length
    B: int          # block size (the paper's L)
    G: int          # states verified per step (node 0 = current true state)
    dtype: str      # "f32" | "bf16"
    threshold: float
    rms_eps: float = 1e-5
    rope_base: float = 10000.0

    @property
    def mask_id(self) -> int:
        return self.V - 1

    @property
    def M(self) -> int:
        return self.G * self.B

    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    def scaled(self, **kw) -> "Config":
        return replace(self, **kw)


CONFIGS: Dict[str, Config] = {
    "c1": Config("c1_tiny_fp32", 2, 256, 4, 4, 64, 688, 1024, 64, 8, 4, "f32", 0.9),
    "c2": Config("c2_llada8b_layer", 1, 4096, 32, 32, 128, 12288, 126464, 512, 32, 16, "bf16", 0.9),
    "c3": Config("c3_llada8b_stack", 32, 4096, 32, 32, 128, 12288, 126464, 1024, 32, 32, "bf16", 0.9),
    "c4": Config("c4_dream7b_gqa", 28, 3584, 28, 4, 128, 18944, 152064, 2048, 32, 24, "bf16", 0.9),
    "c5": Config("c5_sdar_smallblock", 32, 4096, 32, 32, 128, 12288, 126464, 8192, 4, 64, "bf16", 0.8),
}

# tensor ids used to derive independent streams from one seed
_TID = dict(wq=1, wk=2, wv=3, wo=4, w_gate=5, w_up=6, w_down=7, norm1=8, norm2=9,
            prefix_k=10, prefix_v=11, w_embed=12, w_vocab=13, final_norm=14, hidden=15,
            bq=16, bk=17, bv=18, suffix_k=19, suffix_v=20)


def _gen(seed: int, tid: int, layer: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((seed * 1000003 + tid * 7919 + layer * 104729) & 0x7FFFFFFFFFFF)
    return g


def _normal(shape, std, mean, seed, tid, layer, device, dtype) -> torch.Tensor:
    g = _gen(seed, tid, layer, device)
    x = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    if std != 1.0:
        x.mul_(std)
    if mean != 0.0:
        x.add_(mean)
    return x.to(dtype)


def layer_weights(cfg: Config, layer: int, seed: int = DEFAULT_SEED, device="cpu",
                  bias: bool = False) -> Dict[str, torch.Tensor]:
    """Random-init weights of one transformer layer, [out, in] row-major."""
    dt = cfg.torch_dtype()
    qd, kvd = cfg.Hq * cfg.hd, cfg.Hkv * cfg.hd
    shapes = dict(wq=(qd, cfg.d), wk=(kvd, cfg.d), wv=(kvd, cfg.d), wo=(cfg.d, qd),
                  w_gate=(cfg.F, cfg.d), w_up=(cfg.F, cfg.d), w_down=(cfg.d, cfg.F))
    w = {k: _normal(s, 0.02, 0.0, seed, _TID[k], layer, device, dt) for k, s in shapes.items()}
    w["norm1"] = _normal((cfg.d,), 0.02, 1.0, seed, _TID["norm1"], layer, device, dt)
    w["norm2"] = _normal((cfg.d,), 0.02, 1.0, seed, _TID["norm2"], layer, device, dt)
    if bias:
        w["bq"] = _normal((qd,), 0.02, 0.0, seed, _TID["bq"], layer, device, dt)
        w["bk"] = _normal((kvd,), 0.02, 0.0, seed, _TID["bk"], layer, device, dt)
        w["bv"] = _normal((kvd,), 0.02, 0.0, seed, _TID["bv"], layer, device, dt)
    return w


def prefix_kv(cfg: Config, layer: int, seed: int = DEFAULT_SEED, device="cpu",
              P: Optional[int] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Cached prefix K and V, each [Hkv, P, hd], N(0,1); K counts as already rotated."""
    P = cfg.P if P is None else P
    dt = cfg.torch_dtype()
    k = _normal((cfg.Hkv, P, cfg.hd), 1.0, 0.0, seed, _TID["prefix_k"], layer, device, dt)
    v = _normal((cfg.Hkv, P, cfg.hd), 1.0, 0.0, seed, _TID["prefix_v"], layer, device, dt)
    return k, v


def suffix_kv(cfg: Config, layer: int, S: int, seed: int = DEFAULT_SEED, device="cpu"
              ) -> Tuple[torch.Tensor, torch.Tensor]:
    """Cached K and V of the S tokens after the block (dual cache), each [Hkv, S, hd], N(0,1); K counts as
    already rotated."""
    dt = cfg.torch_dtype()
    k = _normal((cfg.Hkv, S, cfg.hd), 1.0, 0.0, seed, _TID["suffix_k"], layer, device, dt)
    v = _normal((cfg.Hkv, S, cfg.hd), 1.0, 0.0, seed, _TID["suffix_v"], layer, device, dt)
    return k, v


def head_weights(cfg: Config, seed: int = DEFAULT_SEED, device="cpu") -> Dict[str, torch.Tensor]:
    dt = cfg.torch_dtype()
    return dict(
        w_vocab=_normal((cfg.V, cfg.d), 0.02, 0.0, seed, _TID["w_vocab"], 0, device, dt),
        final_norm=_normal((cfg.d,), 0.02, 1.0, seed, _TID["final_norm"], 0, device, dt),
    )


def embed_weights(cfg: Config, seed: int = DEFAULT_SEED, device="cpu") -> torch.Tensor:
    return _normal((cfg.V, cfg.d), 0.02, 0.0, seed, _TID["w_embed"], 0, device, cfg.torch_dtype())


def hidden_states(cfg: Config, seed: int = DEFAULT_SEED, device="cpu", std: float = 1.0,
                  G: Optional[int] = None) -> torch.Tensor:
    """Stand-alone layer input [G, B, d], N(0, std)."""
    G = cfg.G if G is None else G
    return _normal((G, cfg.B, cfg.d), std, 0.0, seed, _TID["hidden"], 0, device, cfg.torch_dtype())


# ----------------------------------------------------------------------------------------
# draft states and graphs (integer work, numpy)
# ----------------------------------------------------------------------------------------

def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed & 0xFFFFFFFFFFFFFFFF, stream]))


def unmasked_positions(state: np.ndarray, mask_id: int) -> frozenset:
    return frozenset(int(i) for i in np.nonzero(state != mask_id)[0])


def edges_by_superset(states: np.ndarray, mask_id: int, require_token_match: bool = True
                      ) -> np.ndarray:
    """Edge a->c wherever c's unmasked position set strictly contains a's (Eq. 6 plus the
    "additional edges" rule of Alg. 2 part 2).  With ``require_token_match`` the child must
    also keep the parent's tokens at the parent's unmasked positions, i.e. it is a state
    reachable from the parent by further unmasking."""
    G = states.shape[0]
    um = [unmasked_positions(states[g], mask_id) for g in range(G)]
    out = []
    for a in range(G):
        for c in range(G):
            if a == c or not (um[a] < um[c]):
                continue
            if require_token_match and any(states[a, p] != states[c, p] for p in um[a]):
                continue
            out.append((a, c))
    return np.asarray(out, dtype=np.int32).reshape(-1, 2)


def random_states(G: int, B: int, V: int, frac_lo: float, frac_hi: float, seed: int,
                  stream: int = 100) -> np.ndarray:
    """G independent states; each draft's masked fraction is uniform in [lo, hi]."""
    r = _rng(seed, stream)
    mask_id = V - 1
    st = r.integers(0, V - 1, size=(G, B), dtype=np.int64).astype(np.int32)
    for g in range(G):
        frac = r.uniform(frac_lo, frac_hi)
        n_mask = int(round(frac * B))
        pos = r.permutation(B)[:n_mask]
        st[g, pos] = mask_id
    return st


def grown_dag(level_sizes: List[int], B: int, V: int, root_masked_frac: float,
              extra_lo: int, extra_hi: int, seed: int, stream: int = 200
              ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Root (node 0) plus levels of nodes, each a state of the previous level with
    ``extra_lo..extra_hi`` more positions unmasked with uniform tokens.  Returns
    (states [G,B], edges [E,2] by the superset rule, level [G])."""
    r = _rng(seed, stream)
    mask_id = V - 1
    root = r.integers(0, V - 1, size=B, dtype=np.int64).astype(np.int32)
    n_mask = max(1, int(round(root_masked_frac * B)))
    root[r.permutation(B)[:n_mask]] = mask_id
    states, level = [root], [0]
    prev = [0]
    for lv, n in enumerate(level_sizes, start=1):
        cur = []
        for _ in range(n):
            par = states[int(r.choice(prev))]
            child = par.copy()
            masked = np.nonzero(child == mask_id)[0]
            if masked.size:
                k = int(min(masked.size, r.integers(extra_lo, extra_hi + 1)))
                pos = r.choice(masked, size=k, replace=False)
                child[pos] = r.integers(0, V - 1, size=k)
            cur.append(len(states))
            states.append(child)
            level.append(lv)
        prev = cur
    st = np.stack(states).astype(np.int32)
    return st, edges_by_superset(st, mask_id), np.asarray(level, dtype=np.int32)


def pruned_dag(n_keep: int, level_sizes: List[int], B: int, V: int, frac_lo: float,
               frac_hi: float, seed: int, stream: int = 300):
    """A larger grown DAG reduced to root + (n_keep-1) nodes chosen by a seeded score, the
    synthetic stand-in for dynamic pruning to a budget D* (Sec. 4.4.4)."""
    r = _rng(seed, stream)
    frac = float(r.uniform(frac_lo, frac_hi))
    st, _, level = grown_dag(level_sizes, B, V, frac, 1, 4, seed, stream + 1)
    score = r.random(st.shape[0])
    keep = [0] + sorted(sorted(range(1, st.shape[0]), key=lambda i: -score[i])[: n_keep - 1])
    st = st[keep]
    return st, edges_by_superset(st, V - 1), level[keep]


def subset_lattice(B: int, V: int, copies: int, seed: int, stream: int = 400):
    """All 2^B unmask-subsets of a block (node 0 = all masked) with tokens fixed per
    position, repeated ``copies`` times; edges = every strict-subset pair from the first
    copy to every copy."""
    r = _rng(seed, stream)
    mask_id = V - 1
    tok = r.integers(0, V - 1, size=B, dtype=np.int64).astype(np.int32)
    n = 1 << B
    base = np.full((n, B), mask_id, dtype=np.int32)
    for s in range(n):
        for b in range(B):
            if (s >> b) & 1:
                base[s, b] = tok[b]
    st = np.concatenate([base] * copies, axis=0)
    edges = []
    for a in range(n):
        for c in range(n):
            if a != c and (a & c) == a:
                for k in range(copies):
                    edges.append((a, c + k * n))
    return st, np.asarray(edges, dtype=np.int32).reshape(-1, 2), None


def planted_targets(states: np.ndarray, edges: np.ndarray, V: int, depth: int, seed: int,
                    stream: int = 500) -> Tuple[np.ndarray, List[int]]:
    """Target states "sampled from seed": a path root -> n1 -> ... of (up to) ``depth``
    edges is planted by setting target[n_i] = state[n_{i+1}]; every other node's target
    is its own state with one masked position filled by a token that matches no child.
    Returns (targets [G,B], planted path)."""
    r = _rng(seed, stream)
    G, B = states.shape
    mask_id = V - 1
    children: Dict[int, List[int]] = {g: [] for g in range(G)}
    for p, c in edges:
        children[int(p)].append(int(c))
    tgt = states.copy()
    for g in range(G):
        masked = np.nonzero(states[g] == mask_id)[0]
        if masked.size == 0:
            continue
        pos = int(r.choice(masked))
        used = {int(states[c, pos]) for c in children[g]}
        t = int(r.integers(0, V - 1))
        while t in used:
            t = (t + 1) % (V - 1)
        tgt[g, pos] = t
    path = [0]
    cur = 0
    for _ in range(depth):
        if not children[cur]:
            break
        nxt = int(r.choice(children[cur]))
        tgt[cur] = states[nxt]
        path.append(nxt)
        cur = nxt
    return tgt, path


def draft_graph(cfg_key: str, cfg: Config, seed: int = DEFAULT_SEED):
    """States and edges for one of the five workload configurations."""
    if cfg_key == "c1":
        st, e, _ = grown_dag([2, 1], cfg.B, cfg.V, 0.75, 1, 2, seed)
        return st[: cfg.G], edges_by_superset(st[: cfg.G], cfg.mask_id)
    if cfg_key == "c1_literal":
        st = random_states(cfg.G, cfg.B, cfg.V, 0.5, 0.5, seed)
        return st, edges_by_superset(st, cfg.mask_id, require_token_match=False)
    if cfg_key == "c2":
        st = random_states(cfg.G, cfg.B, cfg.V, 0.25, 0.75, seed)
        return st, np.zeros((0, 2), np.int32)
    if cfg_key == "c3":
        st, e, _ = grown_dag([6, 8, 9, 8], cfg.B, cfg.V, 0.75, 1, 4, seed)
        return st, e
    if cfg_key == "c4":
        st, e, _ = pruned_dag(cfg.G, [6, 8, 9, 9, 7], cfg.B, cfg.V, 0.1, 0.9, seed)
        return st, e
    if cfg_key == "c5":
        copies = cfg.G // (1 << cfg.B)
        st, e, _ = subset_lattice(cfg.B, cfg.V, copies, seed)
        return st, e
    raise KeyError(cfg_key)


def candidate_graph(n_levels: int, width: int = 3, seed: int = DEFAULT_SEED, extend_prob: float = 0.75,
                    top_count: int = 4000, stream: int = 500):
    """Synthetic candidate graph of the shape Alg. 2 part 2 produces: n_levels levels of `width` nodes, every
    node a set of (token position rank, vocabulary rank) pairs.  A node of level k > 1 extends a random node of
    level k-1 by one to three pairs with probability extend_prob (so chains of subsets exist, as frequent
    unmasking sequences give), else it is a fresh set of k..k+2 pairs; edges are all (p, q) with p a strict
    subset of q; counts fall off with the level (frequent short sequences, rare long ones) with noise.
    Returns (count [N] int64, level [N] int32 1-based, edges [E,2] int32 (parent, child), formulas)."""
    r = _rng(seed, stream)
    formulas: List[frozenset] = []
    level: List[int] = []

    def fresh_pair(have):
        while True:
            p = (int(r.integers(1, 9)), int(1 + (r.random() < 0.2) + (r.random() < 0.05)))
            if all(p[0] != q[0] for q in have):
                return p

    for k in range(1, n_levels + 1):
        made = []
        while len(made) < width:
            prev = [f for f, l in zip(formulas, level) if l == k - 1]
            if prev and r.random() < extend_prob:
                f = set(prev[int(r.integers(0, len(prev)))])
                n_add = int(r.integers(1, 4))
            else:
                f, n_add = set(), int(r.integers(k, k + 3))
            for _ in range(n_add):
                if len({q[0] for q in f}) >= 8:
                    break
                f.add(fresh_pair(f))
            f = frozenset(f)
            if f and f not in formulas and f not in made:
                made.append(f)
        formulas += made
        level += [k] * width
    N = len(formulas)
    edges = np.array([(p, q) for p in range(N) for q in range(N) if formulas[p] < formulas[q]], np.int32).reshape(-1, 2)
    count = np.array([max(1, int(top_count / l ** 1.3 * r.uniform(0.3, 1.0))) for l in level], np.int64)
    return count, np.array(level, np.int32), edges, [sorted(f) for f in formulas]

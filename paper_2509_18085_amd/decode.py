"""Host loop of speculative block decoding (Alg. 1) on top of the C-ABI entry points.

One iteration = one forward pass: spiffy_verify_step over the current block and its drafts, then, while
MASK tokens remain, the next step's draft graph on the device (spiffy_head_topk + spiffy_draft_prune).
When a block is complete its keys / values are appended to the prefix cache (prefix caching of Sec. 3.1:
spiffy_commit_block, or, when another block follows, inside that block's first pass with
spiffy_verify_step_commit) and the next block starts.  Per forward pass the host reads back 4 + B + 2
integers in one transfer (accept result, accepted block, sizes of the pruned graph); everything else stays
on the device.
Only argument marshalling and the loop live here: every step of the path runs in the library's kernels.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
import torch

from . import spiffy as sp


class DraftGraph:
    """D draft formulas {(i, j)} (1-based: token position rank, vocabulary rank; Sec. 4.4.3) and the edges
    (parent, child) over nodes 0..D, node 0 = the current block.  Edges default to formula inclusion."""

    def __init__(self, formulas: Sequence[Sequence[Tuple[int, int]]], edges: Optional[np.ndarray] = None,
                 device="cuda"):
        self.formulas = [list(map(tuple, f)) for f in formulas]
        self.D = len(self.formulas)
        self.K = max([j for f in self.formulas for _, j in f], default=1)
        if edges is None:
            sets = [set()] + [set(f) for f in self.formulas]
            edges = np.array([(a, c) for a in range(self.D + 1) for c in range(1, self.D + 1)
                              if a != c and sets[a] < sets[c]], np.int32).reshape(-1, 2)
        self.edges_np = np.asarray(edges, np.int32).reshape(-1, 2)
        off = np.cumsum([0] + [len(f) for f in self.formulas]).astype(np.int32)
        pairs = np.array([p for f in self.formulas for p in f], np.int32).reshape(-1, 2)
        self.offsets = torch.from_numpy(off).to(device)
        self.pairs = torch.from_numpy(pairs).to(device) if len(pairs) else None
        self.edges = torch.from_numpy(self.edges_np).to(device) if len(self.edges_np) else None


class BlockDecoder:
    """Decodes blocks of B tokens one after the other against a growing prefix cache.

    layers: per layer dict of device weight tensors; cache_k / cache_v: per layer device tensors
    [Hkv, capacity, hd] whose first P0 rows hold the context; graph: DraftGraph or None (vanilla decoding,
    one state per forward pass); d_star: draft nodes kept per step.  S0 > 0: dual cache, rows P0+B .. P0+B+S0-1
    hold fixed keys / values of the tokens after the first block; every committed block takes B rows off it.
    seq_S0 > 0 (instead of S0): full-sequence model with a prefix cache only: seq_S0 MASK tokens after the first
    block are recomputed in every pass (spiffy_verify_step_seq); a finished block is committed by one more such
    pass on its final tokens, which leaves its keys / values in its slot of the cache.  That pass also ran the
    next block's positions, as all-MASK suffix rows over the very sequence that block's first pass would see: with
    reuse_commit_pass the next block's first step takes its hidden states from there and only runs the head
    (one forward pass less per block; saved_passes counts them).  The two ways compute the same function with
    different rounding (suffix rows read the block's keys from the cache and split their keys differently), so
    in bf16 a near-tie can fall the other way: off by default.
    graph_replay (cached-prefix models): every pass after a block's first is one HIP-graph launch: verify, top-K,
    drafting, pruning and the next pass's inputs are recorded once per block (the prefix length is a kernel
    argument) at the fixed shape of 1 + d_star states and replayed; the host only reads 4 + B + 2 integers per
    pass.  Same tokens, forward passes and accepted depths as the eager loop.
    """

    def __init__(self, cfg: sp.ModelCfg, layers: Sequence[Dict[str, torch.Tensor]], cache_k: Sequence[torch.Tensor],
                 cache_v: Sequence[torch.Tensor], P0: int, w_embed: torch.Tensor, final_norm: torch.Tensor,
                 w_vocab: torch.Tensor, B: int, threshold: float, logit_scale: float = 1.0, force_one: bool = True,
                 graph: Optional[DraftGraph] = None, d_star: int = 0, device="cuda", S0: int = 0, seq_S0: int = 0,
                 reuse_commit_pass: bool = False, graph_replay: bool = False):
        self.cfg, self.B, self.graph, self.device = cfg, B, graph, device
        self.graph_replay = bool(graph_replay) and not seq_S0
        self._pass_graph = None       # (prefix length it was recorded for, HIP graph) of the fixed-shape pass
        self._g_dirty = True          # the static inputs of the fixed-shape pass do not hold the current states yet
        self.graph_launches = 0
        self.d_star = d_star if graph is not None else 0
        self.logit_scale = logit_scale
        self.P, self.S = P0, S0
        self.capacity = int(cache_k[0].shape[1])
        prefix = [sp.prefix_kv(k, v, P0, S0) for k, v in zip(cache_k, cache_v)]
        self.seq_S = seq_S0
        self.reuse_commit_pass = reuse_commit_pass
        self._pending = None
        self._next_hidden = None      # full-sequence model: hidden states of the next block's positions from the commit pass
        self.saved_passes = 0
        self._zero_result = torch.zeros(4, dtype=torch.int32, device=device)   # accept result of a pass with one state
        if seq_S0:
            if S0:
                raise sp.SpiffyError(sp.SPIFFY_EINVAL, "BlockDecoder: a cached suffix and a recomputed one exclude each other")
            self.plan = sp.SeqStepPlan(cfg, [sp.layer_weights(w) for w in layers], prefix, w_embed, final_norm, w_vocab,
                                       1 + self.d_star, B, seq_S0, P0, threshold, logit_scale=logit_scale,
                                       force_one=force_one, device=device)
            self.suffix = torch.full((seq_S0,), cfg.mask_id, dtype=torch.int32, device=device)
        else:
            self.plan = sp.StepPlan(cfg, [sp.layer_weights(w) for w in layers], prefix, w_embed, final_norm, w_vocab,
                                    1 + self.d_star, B, P0, threshold, logit_scale=logit_scale, force_one=force_one,
                                    device=device, keep_hidden=False)     # the loop reads decisions only: the last layer runs on masked rows
            # the workspace must also fit the longest prefix the cache can hold
            self.plan.workspace = sp.alloc_workspace(cfg, 1 + self.d_star, B, self.capacity, device)
            if self.graph_replay:
                self._init_fixed_pass()

    # ---- a forward pass of fixed shape, recorded once per block into a HIP graph and replayed for every further pass ----
    def _init_fixed_pass(self) -> None:
        """Static buffers of the fixed-shape pass: always 1 + d_star states and the whole edge list.  States that the
        pruning did not keep are copies of the current block and edges that did not survive are (0, 0): neither can be
        reached by the walk, and a state's rows do not depend on the states verified with it, so every result equals
        that of the variable-shape pass."""
        dev, G, B = self.device, 1 + self.d_star, self.B
        E = int(self.graph.edges.shape[0]) if (self.graph is not None and self.graph.edges is not None) else 0
        self._g_states = torch.full((G, B), self.cfg.mask_id, dtype=torch.int32, device=dev)
        self._g_edges = torch.zeros((max(E, 1), 2), dtype=torch.int32, device=dev)
        self._g_pack = torch.zeros(4 + B + 2, dtype=torch.int32, device=dev)      # accept result, accepted block, pruned sizes
        self._g_rows = torch.arange(G, device=dev).reshape(G, 1)
        self._g_erows = torch.arange(max(E, 1), device=dev).reshape(-1, 1)
        self._fixed_pass()            # once outside any capture: one-time kernel attributes of every tile shape it uses
        torch.cuda.synchronize()
        self._g_states.fill_(self.cfg.mask_id)
        self._g_edges.zero_()

    def _fixed_pass(self) -> None:
        """verify -> top-K of the accepted node -> drafting and pruning -> the next pass's inputs, all on the device."""
        drafting = self.graph is not None and self.d_star > 0
        E = int(self.graph.edges.shape[0]) if (drafting and self.graph.edges is not None) else 0
        out = self.plan.run(self._g_states, self._g_edges if E else None)
        new_state = out["accepted_state"]
        if drafting:
            tok, prob = sp.head_topk(self.cfg, self.plan.w_vocab, self._g_states, self.graph.K, self.logit_scale,
                                     self.plan.workspace, result=out["result"], after_step=True)
            dp = sp.draft_prune(new_state, self.cfg.mask_id, tok, prob, self.graph.offsets, self.graph.pairs,
                                self.graph.edges, self.d_star)
            counts = dp["counts"]
            self._g_states.copy_(torch.where(self._g_rows < counts[0], dp["states"], new_state.reshape(1, self.B)))
            if E:
                self._g_edges.copy_(torch.where(self._g_erows < counts[1], dp["edges"], torch.zeros_like(dp["edges"])))
            self._g_pack.copy_(torch.cat([out["result"], new_state, counts]))
        else:
            self._g_states.copy_(new_state.reshape(1, self.B))
            self._g_pack[:4 + self.B].copy_(torch.cat([out["result"], new_state]))

    def _replay_pass(self) -> None:
        if self._pass_graph is None or self._pass_graph[0] != (self.P, self.S):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                self._fixed_pass()
            self._pass_graph = ((self.P, self.S), g)
        self._pass_graph[1].replay()
        self.graph_launches += 1

    def _step(self, states, edges):
        if isinstance(self.plan, sp.SeqStepPlan):
            return self.plan.run(states, self.suffix[:self.seq_S], edges)
        if self._pending is not None:
            # the block finished last is committed by the first pass of this one (one pass over the weights for both)
            out = self.plan.run_commit(self._pending, states, edges)
            self._pending = None
            self._advance()
            return out
        return self.plan.run(states, edges)

    def _advance(self):
        self.P += self.B
        self.S = max(0, self.S - self.B)
        self.plan.set_prefix_len(self.P, S=self.S)

    def flush(self) -> None:
        """Commit a block whose commit was deferred (no further block followed it)."""
        if self._pending is not None:
            self.plan.commit_block(self._pending)
            self._pending = None
            self._advance()

    def decode_block(self, block0: torch.Tensor, max_steps: int = 4096) -> Dict:
        """block0 [B] int32 on the device.  Returns the final block (device), the number of forward passes,
        the accepted depth and the number of states verified in every pass, and the block after every pass
        (host copies)."""
        mask_id = self.cfg.mask_id
        state = block0.to(torch.int32).reshape(1, self.B).contiguous()
        states, edges = state, None
        cur = state[0].cpu().numpy()
        nfe, depths, n_states, traj = 0, [], [], [cur.copy()]
        drafting = self.graph is not None and self.d_star > 0

        def finish_pass(result, new_state, after_step):
            """Enqueue the next pass's drafts (top-K of the accepted node, read on the device, then drafting and
            pruning) before the host looks at anything; ONE host read then brings back the accept result (4), the
            accepted block (B) and the pruned sizes (2)."""
            nonlocal cur, states, edges
            parts = [result, new_state]
            if drafting:
                tok, prob = sp.head_topk(self.cfg, self.plan.w_vocab, states.contiguous(), self.graph.K,
                                         self.logit_scale, self.plan.workspace, result=result, after_step=after_step)
                dp = sp.draft_prune(new_state, mask_id, tok, prob, self.graph.offsets, self.graph.pairs,
                                    self.graph.edges, self.d_star)
                parts.append(dp["counts"])
            host = torch.cat(parts).cpu().numpy()
            depths.append(int(host[1]))
            cur = host[4:4 + self.B].copy()
            traj.append(cur.copy())
            if drafting and (cur == mask_id).any():
                n_kept, n_edges = int(host[4 + self.B]), int(host[5 + self.B])
                states = dp["states"][:n_kept]
                edges = dp["edges"][:n_edges].contiguous() if n_edges else None
            else:
                states, edges = new_state.reshape(1, self.B), None

        if self._next_hidden is not None:
            # Full-sequence model: the pass that committed the previous block ran this block's positions as all-MASK
            # suffix rows over exactly the sequence this block's first pass would see, so that pass only needs the
            # head: no forward pass is spent on it.
            hidden, self._next_hidden = self._next_hidden, None
            if bool((cur == mask_id).all()):
                dh = sp.decode_head(self.cfg, hidden, self.plan.final_norm, self.plan.w_vocab, states.contiguous(),
                                    self.plan.threshold, self.plan.workspace, logit_scale=self.logit_scale,
                                    force_one=bool(self.plan.force_one))
                n_states.append(1)
                self.saved_passes += 1
                finish_pass(self._zero_result, dh["target_states"][0].clone(), False)
        while nfe < max_steps and (cur == mask_id).any():
            if self.graph_replay and nfe > 0 and self._pending is None:
                # every pass after the block's first: the fixed-shape pass, replayed from the graph recorded for this
                # block's prefix length; the host reads the same 4 + B + 2 integers
                if nfe == 1 or self._g_dirty:
                    G_cap = self._g_states.shape[0]
                    self._g_states.copy_(cur_dev.reshape(1, self.B).expand(G_cap, self.B))
                    self._g_states[:states.shape[0]].copy_(states)
                    self._g_edges.zero_()
                    if edges is not None:
                        self._g_edges[:edges.shape[0]].copy_(edges)
                    self._g_dirty = False
                n_states.append(int(states.shape[0]))
                self._replay_pass()
                nfe += 1
                host = self._g_pack.cpu().numpy()
                depths.append(int(host[1]))
                cur = host[4:4 + self.B].copy()
                traj.append(cur.copy())
                n_kept = int(host[4 + self.B]) if drafting else 1
                states = self._g_states[:max(1, n_kept)]            # what the next pass verifies (the rest is padding)
                continue
            out = self._step(states.contiguous(), edges)
            nfe += 1
            n_states.append(int(states.shape[0]))
            cur_dev = out["accepted_state"].clone()
            finish_pass(out["result"], cur_dev, True)
            self._g_dirty = True
        return dict(final=states[0].clone(), nfe=nfe, depths=depths, n_states=n_states, trajectory=traj)

    def commit(self, block: torch.Tensor, defer: bool = False) -> None:
        """Append the finished block to the cache; the next block sits right after it.  defer=True (cached-prefix
        models): the block's forward pass is folded into the first pass of the next block (spiffy_verify_step_commit,
        same results); flush() commits it if no block follows."""
        self.flush()
        if self.P + self.B > self.capacity:
            raise sp.SpiffyError(sp.SPIFFY_ESHAPE, "BlockDecoder.commit: cache is full")
        if isinstance(self.plan, sp.SeqStepPlan):
            if self.seq_S:
                # one pass on the finished block: every pass with a suffix writes the true block's keys / values
                # (which depend on the suffix) into its slot
                out = self._step(block.to(torch.int32).reshape(1, self.B).contiguous(), None)
                if self.seq_S >= self.B and self.reuse_commit_pass:
                    self._next_hidden = out["hidden"][self.B:2 * self.B].clone().reshape(1, self.B, self.cfg.d)
            else:
                self.plan.commit_block(block.to(torch.int32).contiguous())
            self.P += self.B
            self.seq_S = max(0, self.seq_S - self.B)
            self.plan.set_prefix_len(self.P)
            return
        if defer and self.P + 2 * self.B <= self.capacity:
            self._pending = block.to(torch.int32).contiguous()
            return
        self.plan.commit_block(block.to(torch.int32).contiguous())
        self._advance()

    def generate(self, n_blocks: int) -> Dict:
        """Decode n_blocks all-MASK blocks in sequence.  Returns tokens [n_blocks*B] (host), forward passes,
        accepted depths and states verified per pass, per block."""
        out_tokens: List[np.ndarray] = []
        nfe, depths, n_states = [], [], []
        for i in range(n_blocks):
            block0 = torch.full((self.B,), self.cfg.mask_id, dtype=torch.int32, device=self.device)
            r = self.decode_block(block0)
            out_tokens.append(r["final"].cpu().numpy())
            nfe.append(r["nfe"])
            depths.append(r["depths"])
            n_states.append(r["n_states"])
            self.commit(r["final"], defer=i + 1 < n_blocks)
        return dict(tokens=np.concatenate(out_tokens), nfe=nfe, depths=depths, n_states=n_states)

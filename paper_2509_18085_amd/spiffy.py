"""Thin ctypes binding over libspiffy.so (the C ABI declared in include/spiffy.h).

Argument marshalling only: every step of the verification path runs in the HIP kernels behind
the C ABI.  PyTorch is used for device memory and the stream handle.  Importing this module loads
the library and raises if it has not been built (python -m paper_2509_18085_amd.build); there is
no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# SPIFFY_LIB names another build of the same library (the host-sanitizer build of the tests); default: the in-tree one
LIB_PATH = os.environ.get("SPIFFY_LIB") or os.path.join(_HERE, "libspiffy.so")

SPIFFY_OK, SPIFFY_EINVAL, SPIFFY_ESHAPE, SPIFFY_EALIGN, SPIFFY_EWORKSPACE, SPIFFY_EDEVICE = 0, -1, -2, -3, -4, -5
SPIFFY_ELIMIT = -6
STATIC_SCRATCH_BYTES, STATIC_MAX_ROWS = 8 << 20, 128
SPIFFY_BF16, SPIFFY_F32 = 0, 1
MAX_G = 64

EXPORTS = ["spiffy_status_str", "spiffy_uses_mfma", "spiffy_workspace_bytes", "spiffy_embed",
           "spiffy_verify_layer", "spiffy_verify_layer_last", "spiffy_decode_head", "spiffy_gemm", "spiffy_graph_accept", "spiffy_draft_prune", "spiffy_head_topk", "spiffy_commit_block",
           "spiffy_subgraph_search_workspace_bytes", "spiffy_subgraph_search", "spiffy_verify_step",
           "spiffy_workspace_bytes_seq", "spiffy_verify_step_seq", "spiffy_workspace_bytes_commit",
           "spiffy_verify_step_commit", "spiffy_decode_head_static", "spiffy_gemm_plan"]
GEMM_STORE, GEMM_RESID, GEMM_SWIGLU = 0, 1, 2


class ModelCfg(C.Structure):
    _fields_ = [("d", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("ffn", C.c_int32), ("vocab", C.c_int32),
                ("mask_id", C.c_int32), ("dtype", C.c_int32), ("rms_eps", C.c_float),
                ("rope_base", C.c_float)]


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down",
                                          "norm1", "norm2", "bq", "bk", "bv")]


class PrefixKV(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("P", C.c_int32), ("capacity", C.c_int32), ("S", C.c_int32)]


class AcceptResult(C.Structure):
    _fields_ = [("node", C.c_int32), ("depth", C.c_int32), ("n_steps", C.c_int32), ("flags", C.c_int32)]


class GemmLaunch(C.Structure):
    _fields_ = [("tile_rows", C.c_int32), ("tile_cols", C.c_int32), ("col0", C.c_int32), ("n_cols", C.c_int32),
                ("workgroups", C.c_int32)]


class GemmPlan(C.Structure):
    _fields_ = [("n_launches", C.c_int32), ("k_slices", C.c_int32), ("launch", GemmLaunch * 2)]


class SpiffyError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (status %d)" % (where, status_str(status), status))


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError("libspiffy.so is not built (%s missing): run `python -m paper_2509_18085_amd.build`; "
                          "there is no fallback path" % LIB_PATH)
    lib = C.CDLL(LIB_PATH)
    vp, i32, f32, sz = C.c_void_p, C.c_int32, C.c_float, C.c_size_t
    cfgp = C.POINTER(ModelCfg)
    lib.spiffy_status_str.restype = C.c_char_p
    lib.spiffy_status_str.argtypes = [C.c_int]
    lib.spiffy_uses_mfma.restype = C.c_int
    lib.spiffy_uses_mfma.argtypes = [cfgp, i32]
    lib.spiffy_workspace_bytes.restype = sz
    lib.spiffy_workspace_bytes.argtypes = [cfgp, i32, i32, i32]
    lib.spiffy_embed.restype = C.c_int
    lib.spiffy_embed.argtypes = [cfgp, vp, vp, i32, i32, vp, vp]
    lib.spiffy_verify_layer.restype = C.c_int
    lib.spiffy_verify_layer.argtypes = [cfgp, C.POINTER(LayerWeights), C.POINTER(PrefixKV), vp, i32, i32, i32,
                                        vp, vp, sz, vp]
    lib.spiffy_verify_layer_last.restype = C.c_int
    lib.spiffy_verify_layer_last.argtypes = [cfgp, C.POINTER(LayerWeights), C.POINTER(PrefixKV), vp, vp, vp, i32, i32,
                                             i32, vp, vp, sz, vp]
    lib.spiffy_decode_head.restype = C.c_int
    lib.spiffy_decode_head.argtypes = [cfgp, vp, vp, vp, vp, vp, i32, i32, f32, f32, i32, vp, vp, vp, vp, vp,
                                       vp, sz, vp]
    lib.spiffy_decode_head_static.restype = C.c_int
    lib.spiffy_decode_head_static.argtypes = [cfgp, vp, vp, vp, vp, vp, i32, i32, f32, f32, i32, vp, vp, vp, vp, vp, vp]
    lib.spiffy_gemm_plan.restype = C.c_int
    lib.spiffy_gemm_plan.argtypes = [i32, i32, i32, i32, i32, C.POINTER(GemmPlan)]
    lib.spiffy_gemm.restype = C.c_int
    lib.spiffy_gemm.argtypes = [i32, i32, vp, vp, vp, vp, vp, i32, i32, i32, vp, sz, vp]
    lib.spiffy_graph_accept.restype = C.c_int
    lib.spiffy_graph_accept.argtypes = [vp, i32, vp, vp, i32, i32, i32, vp, vp, vp]
    lib.spiffy_commit_block.restype = C.c_int
    lib.spiffy_commit_block.argtypes = [cfgp, i32, C.POINTER(LayerWeights), C.POINTER(PrefixKV), vp, vp, i32, i32,
                                        vp, sz, vp]
    lib.spiffy_head_topk.restype = C.c_int
    lib.spiffy_head_topk.argtypes = [cfgp, vp, vp, i32, i32, vp, i32, i32, f32, i32, vp, vp, vp, sz, vp]
    lib.spiffy_draft_prune.restype = C.c_int
    lib.spiffy_draft_prune.argtypes = [vp, i32, i32, vp, vp, i32, vp, vp, i32, i32, vp, i32, i32, vp, vp, vp, vp,
                                       vp, vp, vp, vp, vp]
    lib.spiffy_subgraph_search_workspace_bytes.restype = C.c_size_t
    lib.spiffy_subgraph_search_workspace_bytes.argtypes = []
    lib.spiffy_subgraph_search.restype = C.c_int
    lib.spiffy_subgraph_search.argtypes = [vp, vp, i32, vp, i32, i32, vp, vp, vp, vp, vp, sz, vp]
    lib.spiffy_workspace_bytes_seq.restype = sz
    lib.spiffy_workspace_bytes_seq.argtypes = [cfgp, i32, i32, i32, i32]
    lib.spiffy_verify_step_seq.restype = C.c_int
    lib.spiffy_verify_step_seq.argtypes = [cfgp, i32, C.POINTER(LayerWeights), C.POINTER(PrefixKV), vp, vp, vp, vp, vp,
                                           i32, i32, i32, i32, vp, i32, i32, f32, f32, i32, vp, vp, vp, vp, vp, vp, vp,
                                           vp, vp, sz, vp]
    lib.spiffy_workspace_bytes_commit.restype = sz
    lib.spiffy_workspace_bytes_commit.argtypes = [cfgp, i32, i32, i32]
    lib.spiffy_verify_step_commit.restype = C.c_int
    lib.spiffy_verify_step_commit.argtypes = [cfgp, i32, C.POINTER(LayerWeights), C.POINTER(PrefixKV), vp, vp, vp, vp, vp,
                                              i32, i32, i32, vp, i32, i32, f32, f32, i32, vp, vp, vp, vp, vp, vp, vp,
                                              vp, vp, sz, vp]
    lib.spiffy_verify_step.restype = C.c_int
    lib.spiffy_verify_step.argtypes = [cfgp, i32, C.POINTER(LayerWeights), C.POINTER(PrefixKV), vp, vp, vp, vp,
                                       i32, i32, i32, vp, i32, i32, f32, f32, i32, vp, vp, vp, vp, vp, vp, vp,
                                       vp, vp, sz, vp]
    return lib


lib = _load()


def status_str(status: int) -> str:
    return lib.spiffy_status_str(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != SPIFFY_OK:
        raise SpiffyError(status, where)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return t.data_ptr()


def _stream(stream=None) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    s = stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)
    return s or None


def make_cfg(*, d, n_q_heads, n_kv_heads, head_dim, ffn, vocab, mask_id, dtype, rms_eps=1e-5,
             rope_base=10000.0) -> ModelCfg:
    code = {torch.bfloat16: SPIFFY_BF16, torch.float32: SPIFFY_F32, "bf16": SPIFFY_BF16, "f32": SPIFFY_F32}[dtype]
    return ModelCfg(d, n_q_heads, n_kv_heads, head_dim, ffn, vocab, mask_id, code, rms_eps, rope_base)


def cfg_from_synth(c) -> ModelCfg:
    return make_cfg(d=c.d, n_q_heads=c.Hq, n_kv_heads=c.Hkv, head_dim=c.hd, ffn=c.F, vocab=c.V,
                    mask_id=c.mask_id, dtype=c.dtype, rms_eps=c.rms_eps, rope_base=c.rope_base)


def layer_weights(w: Dict[str, torch.Tensor]) -> LayerWeights:
    lw = LayerWeights()
    for name, _ in LayerWeights._fields_:
        setattr(lw, name, _ptr(w.get(name)))
    lw._keep = w          # keep the tensors alive as long as the struct
    return lw


def prefix_kv(k: Optional[torch.Tensor], v: Optional[torch.Tensor], P: Optional[int] = None, S: int = 0) -> PrefixKV:
    """k, v [Hkv, rows, hd], row j = sequence position j.  P = prefix rows in use (default: all of them); rows
    beyond P are room for commit_block to extend the cache; S = rows of the tokens after the block (dual
    cache), which sit at rows P+B .. P+B+S-1."""
    rows = 0 if k is None else int(k.shape[1])
    P = rows if P is None else int(P)
    p = PrefixKV(_ptr(k) if rows else None, _ptr(v) if rows else None, P, rows if rows != P else 0, int(S))
    p._keep = (k, v)
    return p


def uses_mfma(cfg: ModelCfg, B: int) -> int:
    return lib.spiffy_uses_mfma(C.byref(cfg), B)


def workspace_bytes(cfg: ModelCfg, G: int, B: int, P_max: int) -> int:
    return int(lib.spiffy_workspace_bytes(C.byref(cfg), G, B, P_max))


def alloc_workspace(cfg: ModelCfg, G: int, B: int, P_max: int, device="cuda") -> torch.Tensor:
    n = workspace_bytes(cfg, G, B, P_max)
    if n == 0:
        raise SpiffyError(SPIFFY_EINVAL, "spiffy_workspace_bytes")
    return torch.empty(n + 256, dtype=torch.uint8, device=device)


def _ws(ws: torch.Tensor) -> Tuple[int, int]:
    p = ws.data_ptr()
    off = (-p) % 256
    return p + off, ws.numel() - off


def _tdtype(cfg: ModelCfg):
    return torch.float32 if cfg.dtype == SPIFFY_F32 else torch.bfloat16


def embed(cfg: ModelCfg, w_embed: torch.Tensor, block_tokens: torch.Tensor, out: Optional[torch.Tensor] = None,
          stream=None) -> torch.Tensor:
    G, B = block_tokens.shape
    if out is None:
        out = torch.empty((G, B, cfg.d), dtype=_tdtype(cfg), device=w_embed.device)
    _check(lib.spiffy_embed(C.byref(cfg), _ptr(w_embed), _ptr(block_tokens), G, B, _ptr(out), _stream(stream)),
           "spiffy_embed")
    return out


def verify_layer(cfg: ModelCfg, w: LayerWeights, prefix: PrefixKV, hidden_in: torch.Tensor, pos0: int,
                 workspace: torch.Tensor, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    G, B, _ = hidden_in.shape
    if out is None:
        out = torch.empty_like(hidden_in)
    wp, wn = _ws(workspace)
    _check(lib.spiffy_verify_layer(C.byref(cfg), C.byref(w), C.byref(prefix), _ptr(hidden_in), G, B, pos0,
                                   _ptr(out), wp, wn, _stream(stream)), "spiffy_verify_layer")
    return out


def verify_layer_last(cfg: ModelCfg, w: LayerWeights, prefix: PrefixKV, hidden_in: torch.Tensor,
                      block_tokens: torch.Tensor, pos0: int, workspace: torch.Tensor, out: torch.Tensor,
                      mask: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """The last layer of a step: rows of masked positions of `out` are written, the others are left as they are."""
    G, B, _ = hidden_in.shape
    wp, wn = _ws(workspace)
    _check(lib.spiffy_verify_layer_last(C.byref(cfg), C.byref(w), C.byref(prefix), _ptr(hidden_in), _ptr(block_tokens),
                                        _ptr(mask), G, B, pos0, _ptr(out), wp, wn, _stream(stream)),
           "spiffy_verify_layer_last")
    return out


def decode_head(cfg: ModelCfg, hidden: torch.Tensor, final_norm: torch.Tensor, w_vocab: torch.Tensor,
                block_tokens: torch.Tensor, threshold: float, workspace: torch.Tensor, *,
                mask: Optional[torch.Tensor] = None, logit_scale: float = 1.0, force_one: bool = True,
                stream=None) -> Dict[str, torch.Tensor]:
    G, B = block_tokens.shape
    dev = hidden.device
    out = dict(argmax=torch.empty((G, B), dtype=torch.int32, device=dev),
               conf=torch.empty((G, B), dtype=torch.float32, device=dev),
               unmask=torch.empty((G, B), dtype=torch.uint8, device=dev),
               margin=torch.empty((G, B), dtype=torch.float32, device=dev),
               target_states=torch.empty((G, B), dtype=torch.int32, device=dev))
    wp, wn = _ws(workspace)
    _check(lib.spiffy_decode_head(C.byref(cfg), _ptr(hidden), _ptr(final_norm), _ptr(w_vocab), _ptr(block_tokens),
                                  _ptr(mask), G, B, threshold, logit_scale, int(force_one), _ptr(out["argmax"]),
                                  _ptr(out["conf"]), _ptr(out["unmask"]), _ptr(out["margin"]),
                                  _ptr(out["target_states"]), wp, wn, _stream(stream)), "spiffy_decode_head")
    return out


def decode_head_static(cfg: ModelCfg, hidden: torch.Tensor, final_norm: torch.Tensor, w_vocab: torch.Tensor,
                       block_tokens: torch.Tensor, threshold: float, out: Dict[str, torch.Tensor], *,
                       mask: Optional[torch.Tensor] = None, logit_scale: float = 1.0, force_one: bool = True,
                       stream=None) -> Dict[str, torch.Tensor]:
    """spiffy_decode_head_static: decode_head on the library's own device scratch.  Nothing is allocated, here or
    in the library: `out` holds the caller's output tensors (argmax, conf, unmask, margin, target_states: the
    dictionary decode_head returns has the right shapes)."""
    G, B = block_tokens.shape
    _check(lib.spiffy_decode_head_static(C.byref(cfg), _ptr(hidden), _ptr(final_norm), _ptr(w_vocab), _ptr(block_tokens),
                                         _ptr(mask), G, B, threshold, logit_scale, int(force_one), _ptr(out["argmax"]),
                                         _ptr(out["conf"]), _ptr(out["unmask"]), _ptr(out.get("margin")),
                                         _ptr(out.get("target_states")), _stream(stream)), "spiffy_decode_head_static")
    return out


def gemm(epilogue: int, A: torch.Tensor, W0: torch.Tensor, W1: Optional[torch.Tensor] = None,
         R: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None,
         workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    M, K = A.shape
    N = W0.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=A.dtype, device=A.device)
    dt = SPIFFY_F32 if A.dtype == torch.float32 else SPIFFY_BF16
    wp, wn = _ws(workspace) if workspace is not None else (None, 0)
    _check(lib.spiffy_gemm(dt, epilogue, _ptr(A), _ptr(W0), _ptr(W1), _ptr(R), _ptr(out), M, N, K, wp, wn,
                           _stream(stream)), "spiffy_gemm")
    return out


def gemm_plan(epilogue: int, M: int, N: int, K: int, with_workspace: bool = True) -> dict:
    """The launches spiffy_gemm / verify_layer use for a bf16 projection of that shape (host arithmetic, no device)."""
    p = GemmPlan()
    _check(lib.spiffy_gemm_plan(epilogue, M, N, K, int(with_workspace), C.byref(p)), "spiffy_gemm_plan")
    return {"k_slices": p.k_slices,
            "launches": [{"tile": (l.tile_rows, l.tile_cols), "col0": l.col0, "n_cols": l.n_cols,
                          "workgroups": l.workgroups} for l in p.launch[:p.n_launches]]}


def graph_accept(graph_edges: torch.Tensor, draft_states: torch.Tensor, target_states: torch.Tensor,
                 root: int = 0, stream=None, res: Optional[torch.Tensor] = None,
                 state: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Returns (result int32[4] = node, depth, n_steps, flags ; accepted_state int32[B]), on device (written into
    `res` / `state` when the caller passes them)."""
    G, B = draft_states.shape
    E = int(graph_edges.shape[0]) if graph_edges is not None else 0
    if res is None:
        res = torch.empty(4, dtype=torch.int32, device=draft_states.device)
    if state is None:
        state = torch.empty(B, dtype=torch.int32, device=draft_states.device)
    _check(lib.spiffy_graph_accept(_ptr(graph_edges) if E else None, E, _ptr(draft_states), _ptr(target_states),
                                   G, B, root, _ptr(res), _ptr(state), _stream(stream)), "spiffy_graph_accept")
    return res, state


def head_topk(cfg: ModelCfg, w_vocab: torch.Tensor, block_tokens: torch.Tensor, K: int, logit_scale: float,
              workspace: torch.Tensor, *, result: Optional[torch.Tensor] = None, node: int = 0,
              after_step: bool = False, stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Top-K tokens / probabilities per position of one node, from what the preceding decode_head
    (after_step=False) or verify_step (after_step=True) call left in `workspace`.  `result` = the device
    accept result (node read on the device) or None to use `node`."""
    G, B = block_tokens.shape
    tok = torch.empty((B, K), dtype=torch.int32, device=block_tokens.device)
    prob = torch.empty((B, K), dtype=torch.float32, device=block_tokens.device)
    wp, wn = _ws(workspace)
    _check(lib.spiffy_head_topk(C.byref(cfg), _ptr(w_vocab), _ptr(block_tokens), G, B,
                                _ptr(result) if result is not None else None, node, K, logit_scale,
                                1 if after_step else 0, _ptr(tok), _ptr(prob), wp, wn, _stream(stream)),
           "spiffy_head_topk")
    return tok, prob


def draft_prune(state: torch.Tensor, mask_id: int, topk_tokens: torch.Tensor, topk_probs: torch.Tensor,
                formula_offsets: torch.Tensor, formula_pairs: torch.Tensor, edges: Optional[torch.Tensor],
                d_star: int, stream=None) -> Dict[str, torch.Tensor]:
    """Draft blocks from formulas and the pruned graph for the next step; every tensor on the device.
    Returns drafts [D+1,B], buildable [D+1], local, score [D+1], kept [d_star+1], states [d_star+1,B],
    edges [E,2], counts [2] (kept nodes, surviving edges)."""
    dev = state.device
    B = int(state.numel())
    K = int(topk_tokens.shape[1])
    D = int(formula_offsets.numel()) - 1
    nnz = int(formula_pairs.shape[0]) if formula_pairs is not None else 0
    E = int(edges.shape[0]) if edges is not None else 0
    out = dict(drafts=torch.empty((D + 1, B), dtype=torch.int32, device=dev),
               buildable=torch.empty(D + 1, dtype=torch.uint8, device=dev),
               local=torch.empty(D + 1, dtype=torch.float32, device=dev),
               score=torch.empty(D + 1, dtype=torch.float32, device=dev),
               kept=torch.full((d_star + 1,), -1, dtype=torch.int32, device=dev),
               states=torch.empty((d_star + 1, B), dtype=torch.int32, device=dev),
               edges=torch.empty((max(E, 1), 2), dtype=torch.int32, device=dev),
               counts=torch.empty(2, dtype=torch.int32, device=dev))
    _check(lib.spiffy_draft_prune(_ptr(state), B, mask_id, _ptr(topk_tokens), _ptr(topk_probs), K,
                                  _ptr(formula_offsets), _ptr(formula_pairs) if nnz else None, D, nnz,
                                  _ptr(edges) if E else None, E, d_star, _ptr(out["drafts"]), _ptr(out["buildable"]),
                                  _ptr(out["local"]), _ptr(out["score"]), _ptr(out["kept"]), _ptr(out["states"]),
                                  _ptr(out["edges"]), _ptr(out["counts"]), _stream(stream)), "spiffy_draft_prune")
    return out


def subgraph_search(count: torch.Tensor, level: torch.Tensor, edges: Optional[torch.Tensor], D: int,
                    workspace: Optional[torch.Tensor] = None, stream=None) -> Dict[str, torch.Tensor]:
    """Best connected node set of size D of a candidate graph (calibration, part 3).  count [N] int64, level [N]
    int32, edges [E,2] int32 (parent, child), all on the device.  Returns device tensors best_mask [1] (int64
    holding the 64-bit mask), best_sum [1], n_connected [1], nodes [D]."""
    dev = count.device
    N = int(count.numel())
    E = int(edges.shape[0]) if edges is not None else 0
    if workspace is None:
        workspace = torch.empty(int(lib.spiffy_subgraph_search_workspace_bytes()) + 256, dtype=torch.uint8, device=dev)
    wp, wn = _ws(workspace)
    out = dict(best_mask=torch.empty(1, dtype=torch.int64, device=dev), best_sum=torch.empty(1, dtype=torch.int64, device=dev),
               n_connected=torch.empty(1, dtype=torch.int64, device=dev),
               nodes=torch.empty(max(1, min(D, 64)), dtype=torch.int32, device=dev))
    _check(lib.spiffy_subgraph_search(_ptr(count), _ptr(level), N, _ptr(edges) if E else None, E, D, _ptr(out["best_mask"]),
                                      _ptr(out["best_sum"]), _ptr(out["n_connected"]), _ptr(out["nodes"]), wp, wn,
                                      _stream(stream)), "spiffy_subgraph_search")
    out["_workspace"] = workspace
    return out


class StepPlan:
    """Pre-marshalled arguments of spiffy_verify_step for repeated calls (weights, prefix KV and
    output buffers are fixed; only the launch happens per call)."""

    def __init__(self, cfg: ModelCfg, layers: Sequence[LayerWeights], prefix: Sequence[PrefixKV],
                 w_embed: torch.Tensor, final_norm: torch.Tensor, w_vocab: torch.Tensor, G: int, B: int,
                 pos0: int, threshold: float, logit_scale: float = 1.0, force_one: bool = True,
                 root: int = 0, device="cuda", keep_hidden: bool = True):
        self.cfg, self.G, self.G_cap, self.B, self.pos0 = cfg, G, G, B, pos0
        self.keep_hidden = keep_hidden      # False: hidden_out = NULL, the last layer runs on the masked rows only
        self.threshold, self.logit_scale, self.force_one, self.root = threshold, logit_scale, int(force_one), root
        self.n_layers = len(layers)
        self._layers = (LayerWeights * max(1, self.n_layers))(*layers)
        self._prefix = (PrefixKV * max(1, self.n_layers))(*prefix)
        self._keep = (list(layers), list(prefix), w_embed, final_norm, w_vocab)
        self.w_embed, self.final_norm, self.w_vocab = w_embed, final_norm, w_vocab
        P_max = max([p.P + p.S for p in prefix], default=0)
        self.workspace = alloc_workspace(cfg, G, B, P_max, device)
        dt = _tdtype(cfg)
        self.out = dict(hidden=torch.empty((G, B, cfg.d), dtype=dt, device=device),
                        argmax=torch.empty((G, B), dtype=torch.int32, device=device),
                        conf=torch.empty((G, B), dtype=torch.float32, device=device),
                        unmask=torch.empty((G, B), dtype=torch.uint8, device=device),
                        margin=torch.empty((G, B), dtype=torch.float32, device=device),
                        target_states=torch.empty((G, B), dtype=torch.int32, device=device),
                        result=torch.empty(4, dtype=torch.int32, device=device),
                        accepted_state=torch.empty(B, dtype=torch.int32, device=device))

    def set_prefix_len(self, P: int, pos0: Optional[int] = None, S: Optional[int] = None) -> None:
        """After commit_block: the caches hold P prefix rows per head (and S suffix rows, if given); the block
        now sits at pos0 (default P)."""
        for l in range(self.n_layers):
            self._prefix[l].P = P
            if S is not None:
                self._prefix[l].S = S
        self.pos0 = P if pos0 is None else pos0

    def commit_block(self, block_tokens: torch.Tensor, stream=None) -> None:
        """Append the finished block's keys / values to every layer's cache (rows P .. P+B-1)."""
        wp, wn = _ws(self.workspace)
        _check(lib.spiffy_commit_block(C.byref(self.cfg), self.n_layers, self._layers, self._prefix,
                                       _ptr(self.w_embed), _ptr(block_tokens), self.B, self.pos0, wp, wn,
                                       _stream(stream)), "spiffy_commit_block")

    def run(self, block_tokens: torch.Tensor, graph_edges: Optional[torch.Tensor], stream=None) -> Dict[str, torch.Tensor]:
        """block_tokens [G,B] with G <= the plan's capacity; rows 0..G-1 of the outputs are written."""
        o = self.out
        G = int(block_tokens.shape[0])
        if G > self.G_cap:
            raise SpiffyError(SPIFFY_ESHAPE, "StepPlan.run: more states than the plan was sized for")
        self.G = G
        E = int(graph_edges.shape[0]) if graph_edges is not None else 0
        wp, wn = _ws(self.workspace)
        _check(lib.spiffy_verify_step(
            C.byref(self.cfg), self.n_layers, self._layers, self._prefix, _ptr(self.w_embed), _ptr(self.final_norm),
            _ptr(self.w_vocab), _ptr(block_tokens), self.G, self.B, self.pos0, _ptr(graph_edges) if E else None, E,
            self.root, self.threshold, self.logit_scale, self.force_one, _ptr(o["hidden"]) if self.keep_hidden else None,
            _ptr(o["argmax"]), _ptr(o["conf"]), _ptr(o["unmask"]), _ptr(o["margin"]), _ptr(o["target_states"]),
            _ptr(o["result"]), _ptr(o["accepted_state"]), wp, wn, _stream(stream)), "spiffy_verify_step")
        return o


    def run_commit(self, prev_block: torch.Tensor, block_tokens: torch.Tensor, graph_edges: Optional[torch.Tensor],
                   stream=None) -> Dict[str, torch.Tensor]:
        """commit_block(prev_block) and run(block_tokens) in one pass over the weights (spiffy_verify_step_commit):
        the plan's prefix length is the one BEFORE prev_block and its pos0 the position of prev_block; afterwards
        the caller calls set_prefix_len(P + B).  Returns the step's outputs (hidden: the states' rows)."""
        o = self.out
        G = int(block_tokens.shape[0])
        if G > self.G_cap:
            raise SpiffyError(SPIFFY_ESHAPE, "StepPlan.run_commit: more states than the plan was sized for")
        self.G = G
        dev = block_tokens.device
        if getattr(self, "_commit_ws", None) is None:
            P_max = max([(p.capacity or p.P) for p in self._keep[1]], default=0)
            n = int(lib.spiffy_workspace_bytes_commit(C.byref(self.cfg), self.G_cap, self.B, P_max))
            if n == 0:
                raise SpiffyError(SPIFFY_EINVAL, "spiffy_workspace_bytes_commit")
            if self.workspace.numel() < n + 256:
                self.workspace = torch.empty(n + 256, dtype=torch.uint8, device=dev)
            self._commit_ws = True
            self._commit_hidden = torch.empty(((self.G_cap + 1) * self.B, self.cfg.d), dtype=_tdtype(self.cfg), device=dev)
        E = int(graph_edges.shape[0]) if graph_edges is not None else 0
        wp, wn = _ws(self.workspace)
        _check(lib.spiffy_verify_step_commit(
            C.byref(self.cfg), self.n_layers, self._layers, self._prefix, _ptr(self.w_embed), _ptr(self.final_norm),
            _ptr(self.w_vocab), _ptr(prev_block), _ptr(block_tokens), G, self.B, self.pos0 + self.B,
            _ptr(graph_edges) if E else None, E, self.root, self.threshold, self.logit_scale, self.force_one,
            _ptr(self._commit_hidden), _ptr(o["argmax"]), _ptr(o["conf"]), _ptr(o["unmask"]), _ptr(o["margin"]),
            _ptr(o["target_states"]), _ptr(o["result"]), _ptr(o["accepted_state"]), wp, wn, _stream(stream)),
            "spiffy_verify_step_commit")
        return dict(o, hidden=self._commit_hidden[:G * self.B].view(G, self.B, self.cfg.d),
                    hidden_prev=self._commit_hidden[G * self.B:(G + 1) * self.B])


class SeqStepPlan(StepPlan):
    """spiffy_verify_step_seq with pre-marshalled arguments: the step of a full-sequence model that caches only
    the prefix.  S true tokens after the block ride along; the caches need capacity >= P + B + S (rows behind
    the prefix are rewritten by every call)."""

    def __init__(self, cfg: ModelCfg, layers: Sequence[LayerWeights], prefix: Sequence[PrefixKV], w_embed: torch.Tensor,
                 final_norm: torch.Tensor, w_vocab: torch.Tensor, G: int, B: int, S: int, pos0: int, threshold: float,
                 logit_scale: float = 1.0, force_one: bool = True, root: int = 0, device="cuda"):
        super().__init__(cfg, layers, prefix, w_embed, final_norm, w_vocab, G, B, pos0, threshold, logit_scale=logit_scale,
                         force_one=force_one, root=root, device=device)
        self.S = self.S_cap = S
        P_max = max([p.capacity or p.P for p in prefix], default=0)      # room for a prefix that grows by committed blocks
        n = int(lib.spiffy_workspace_bytes_seq(C.byref(cfg), G, B, S, P_max))
        if n == 0:
            raise SpiffyError(SPIFFY_EINVAL, "spiffy_workspace_bytes_seq")
        self.workspace = torch.empty(n + 256, dtype=torch.uint8, device=device)
        self.out["hidden"] = torch.empty((G * B + S, cfg.d), dtype=_tdtype(cfg), device=device)

    def run(self, block_tokens: torch.Tensor, suffix_tokens: torch.Tensor, graph_edges: Optional[torch.Tensor],
            stream=None) -> Dict[str, torch.Tensor]:
        """block_tokens [G,B] and suffix_tokens [S], both within the plan's capacity.  out["hidden"] holds the G*B
        block rows, then the S suffix rows."""
        o = self.out
        G = int(block_tokens.shape[0])
        S = int(suffix_tokens.numel()) if suffix_tokens is not None else 0
        if G > self.G_cap or S > self.S_cap:
            raise SpiffyError(SPIFFY_ESHAPE, "SeqStepPlan.run: more states or suffix rows than the plan was sized for")
        self.G, self.S = G, S
        E = int(graph_edges.shape[0]) if graph_edges is not None else 0
        wp, wn = _ws(self.workspace)
        _check(lib.spiffy_verify_step_seq(
            C.byref(self.cfg), self.n_layers, self._layers, self._prefix, _ptr(self.w_embed), _ptr(self.final_norm),
            _ptr(self.w_vocab), _ptr(block_tokens), _ptr(suffix_tokens) if self.S else None, G, self.B, self.S, self.pos0,
            _ptr(graph_edges) if E else None, E, self.root, self.threshold, self.logit_scale, self.force_one,
            _ptr(o["hidden"]), _ptr(o["argmax"]), _ptr(o["conf"]), _ptr(o["unmask"]), _ptr(o["margin"]),
            _ptr(o["target_states"]), _ptr(o["result"]), _ptr(o["accepted_state"]), wp, wn, _stream(stream)),
            "spiffy_verify_step_seq")
        return o

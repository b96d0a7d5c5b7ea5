"""Shared test plumbing: tensor <-> numpy conversion and tiny model assembly.
No method arithmetic lives here."""
from __future__ import annotations

import numpy as np
import torch

from paper_2509_18085_amd import synth


# Counts the parity bar asks to be reported (near-ties, excluded states, disagreements with the plain oracle, error
# growth over the layers): tests append dictionaries here, the session prints them at its end (also under -q) and
# writes them, one JSON line each, to the file named by SPIFFY_TEST_REPORT when that is set.
REPORT = []


def to_np(t):
    if isinstance(t, torch.Tensor):
        return t.detach().cpu().to(torch.float64).numpy()
    return np.asarray(t, np.float64)


def np_weights(w):
    return {k: to_np(v) for k, v in w.items()}


def cfg_kw(cfg, pos0=None):
    return dict(n_q_heads=cfg.Hq, n_kv_heads=cfg.Hkv, head_dim=cfg.hd,
                pos0=cfg.P if pos0 is None else pos0, rms_eps=cfg.rms_eps,
                rope_base=cfg.rope_base)


def tiny_cfg(**kw):
    base = synth.CONFIGS["c1"]
    return base.scaled(**kw) if kw else base


def tiny_model(cfg, seed=synth.DEFAULT_SEED, weight_std_scale=1.0, logit_scale=1.0,
               force_one=True, threshold=None):
    """Oracle-side model dict (numpy fp64) for decode_block / verify_step."""
    layers = []
    for l in range(cfg.L):
        w = np_weights(synth.layer_weights(cfg, l, seed))
        if weight_std_scale != 1.0:
            for k in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down"):
                w[k] = w[k] * weight_std_scale
        layers.append(w)
    prefix = [tuple(to_np(t) for t in synth.prefix_kv(cfg, l, seed)) for l in range(cfg.L)]
    hw = synth.head_weights(cfg, seed)
    return dict(
        layers=layers, prefix=prefix, w_embed=to_np(synth.embed_weights(cfg, seed)),
        final_norm=to_np(hw["final_norm"]), w_vocab=to_np(hw["w_vocab"]),
        kw=dict(n_q_heads=cfg.Hq, n_kv_heads=cfg.Hkv, head_dim=cfg.hd, pos0=cfg.P,
                mask_id=cfg.mask_id, threshold=cfg.threshold if threshold is None else threshold,
                rms_eps=cfg.rms_eps, rope_base=cfg.rope_base, logit_scale=logit_scale,
                force_one=force_one))

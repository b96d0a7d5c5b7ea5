"""Pins for the oracle's dual-cache attention (fixed keys / values of the tokens after the block,
Sec. 4.3 / App. A.2), checked without a GPU: each is chosen so that dropping the suffix, counting it twice,
rotating it again, placing it at the wrong positions or hiding it from the drafts fails one of them."""
import math

import numpy as np
import pytest
import torch

from oracle import spiffy_oracle as O
from paper_2509_18085_amd import synth
from helpers import cfg_kw, np_weights, to_np
from test_oracle_pins import _identity_out_cfg, _tokens_model, layer_np, small_cfg


def _caches(cfg, S, seed=3):
    pk, pv = (to_np(t) for t in synth.prefix_kv(cfg, 0, seed))
    sk, sv = (to_np(t) for t in synth.suffix_kv(cfg, 0, S, seed))
    return pk, pv, sk, sv


def test_empty_suffix_is_no_suffix():
    cfg = small_cfg()
    w = layer_np(cfg, bias=True)
    pk, pv, sk, sv = _caches(cfg, 0)
    x = to_np(synth.hidden_states(cfg, 3))
    a = O.verify_layer(w, pk, pv, x, **cfg_kw(cfg))
    b = O.verify_layer(w, pk, pv, x, suffix_k=sk, suffix_v=sv, **cfg_kw(cfg))
    np.testing.assert_array_equal(a, b)


def test_zero_keys_give_the_mean_over_prefix_block_and_suffix():
    """With all keys zero every score is 0 and the output is the plain mean of all P + B + S values."""
    cfg = _identity_out_cfg()
    S = 4
    w = layer_np(cfg)
    w["wo"] = np.eye(cfg.d)
    w["w_down"][:] = 0
    w["wk"][:] = 0
    _, pv, _, sv = _caches(cfg, S)
    pk, sk = np.zeros_like(pv), np.zeros_like(sv)
    x = to_np(synth.hidden_states(cfg, 3))
    out = O.verify_layer(w, pk, pv, x, suffix_k=sk, suffix_v=sv, **cfg_kw(cfg))
    rep = cfg.Hq // cfg.Hkv
    for g in range(cfg.G):
        n = O.rms_norm(x[g], w["norm1"], cfg.rms_eps)
        v_own = (n @ w["wv"].T).reshape(cfg.B, cfg.Hkv, cfg.hd)
        for h in range(cfg.Hq):
            mean_v = (pv[h // rep].sum(0) + v_own[:, h // rep].sum(0) + sv[h // rep].sum(0)) / (cfg.P + cfg.B + S)
            got = (out[g] - x[g])[:, h * cfg.hd:(h + 1) * cfg.hd]
            np.testing.assert_allclose(got, np.broadcast_to(mean_v, got.shape), rtol=1e-12, atol=1e-13)


def test_suffix_rows_are_context_like_prefix_rows():
    """Cached keys are already rotated, so attention does not care in which of the two caches a row sits."""
    cfg = small_cfg(P=4, B=3, G=2)
    S = 5
    w = layer_np(cfg, bias=True)
    pk, pv, sk, sv = _caches(cfg, S)
    x = to_np(synth.hidden_states(cfg, 3))
    a = O.verify_layer(w, pk, pv, x, suffix_k=sk, suffix_v=sv, **cfg_kw(cfg))
    b = O.verify_layer(w, np.concatenate([pk, sk], 1), np.concatenate([pv, sv], 1), x, **cfg_kw(cfg))
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-13)
    c = O.verify_layer(w, pk, pv, x, **cfg_kw(cfg))
    assert np.abs(a - c).max() > 1e-3                     # and the suffix does matter


@pytest.mark.parametrize("B,S", [(1, 3), (4, 6)])
def test_dual_cache_attention_matches_torch_sdpa(B, S):
    cfg = _identity_out_cfg().scaled(B=B, G=2, P=6)
    w = layer_np(cfg, bias=True)
    w["wo"] = np.eye(cfg.d)
    w["w_down"][:] = 0
    pk, pv, sk, sv = _caches(cfg, S, seed=5)
    x = to_np(synth.hidden_states(cfg, 5))
    out = O.verify_layer(w, pk, pv, x, suffix_k=sk, suffix_v=sv, **cfg_kw(cfg))
    rep = cfg.Hq // cfg.Hkv
    T = torch.from_numpy
    for g in range(cfg.G):
        xt = T(x[g])
        n = xt * torch.rsqrt((xt * xt).mean(-1, keepdim=True) + cfg.rms_eps) * T(w["norm1"])
        q = (n @ T(w["wq"]).T + T(w["bq"])).reshape(B, cfg.Hq, cfg.hd).permute(1, 0, 2)
        k = (n @ T(w["wk"]).T + T(w["bk"])).reshape(B, cfg.Hkv, cfg.hd).permute(1, 0, 2)
        v = (n @ T(w["wv"]).T + T(w["bv"])).reshape(B, cfg.Hkv, cfg.hd).permute(1, 0, 2)
        pos = cfg.P + np.arange(B)
        q = T(O.rope(q.numpy(), pos, cfg.rope_base))
        k = T(O.rope(k.numpy(), pos, cfg.rope_base))
        keys = torch.cat([T(pk), k, T(sk)], dim=1).repeat_interleave(rep, dim=0)
        vals = torch.cat([T(pv), v, T(sv)], dim=1).repeat_interleave(rep, dim=0)
        o = torch.nn.functional.scaled_dot_product_attention(q[None], keys[None], vals[None])[0]
        o = o.permute(1, 0, 2).reshape(B, cfg.d).numpy()
        np.testing.assert_allclose(out[g] - x[g], o, rtol=1e-10, atol=1e-12)


def test_first_layer_of_a_full_bidirectional_forward():
    """One layer: keys / values depend on the token embeddings only, so the cached formulation fed with the
    K/V of a full bidirectional forward over [prefix ; block ; suffix] reproduces that forward's block rows
    exactly (App. A.2: fixed context K/V give the exact distribution).  Pins the suffix positions."""
    cfg = small_cfg(L=1, P=5, B=3, G=1)
    S = 4
    layers, w_embed = _tokens_model(cfg)
    r = np.random.default_rng(5)
    T = cfg.P + cfg.B + S
    tok = r.integers(0, cfg.V - 1, T)
    tok[cfg.P + cfg.B:] = cfg.mask_id                      # the tokens after the block are still masked
    x = w_embed[tok]
    kw = dict(n_q_heads=cfg.Hq, n_kv_heads=cfg.Hkv, head_dim=cfg.hd, rms_eps=cfg.rms_eps, rope_base=cfg.rope_base)
    hs, Ks, Vs = O.masked_forward(layers, x, np.arange(T), np.ones((T, T), bool), **kw)
    blk = slice(cfg.P, cfg.P + cfg.B)
    h = O.verify_layer(layers[0], Ks[0][:, :cfg.P], Vs[0][:, :cfg.P], x[None, blk], pos0=cfg.P,
                       suffix_k=Ks[0][:, cfg.P + cfg.B:], suffix_v=Vs[0][:, cfg.P + cfg.B:], **kw)
    np.testing.assert_allclose(h[0], hs[1][blk], rtol=1e-10, atol=1e-12)
    # suffix keys rotated one position off no longer reproduce it
    _, K_off, _ = O.masked_forward(layers, x, np.arange(T) + (np.arange(T) >= cfg.P + cfg.B), np.ones((T, T), bool), **kw)
    h_bad = O.verify_layer(layers[0], Ks[0][:, :cfg.P], Vs[0][:, :cfg.P], x[None, blk], pos0=cfg.P,
                           suffix_k=K_off[0][:, cfg.P + cfg.B:], suffix_v=Vs[0][:, cfg.P + cfg.B:], **kw)
    assert np.abs(h_bad[0] - hs[1][blk]).max() > 1e-6


def test_dense_mask_formulation_with_suffix():
    """The single-sequence formulation of Fig. 4 with the tokens after the block in the context: every block,
    true or draft, attends to prefix, suffix and itself; through all layers it gives what the cached
    formulation gives with the context's own K/V."""
    cfg = small_cfg(P=5, B=3, G=3)
    S = 4
    layers, w_embed = _tokens_model(cfg)
    r = np.random.default_rng(6)
    prefix_tok = r.integers(0, cfg.V - 1, cfg.P)
    suffix_tok = np.full(S, cfg.mask_id)
    states = synth.random_states(cfg.G, cfg.B, cfg.V, 0.3, 0.7, 10)
    kw = dict(n_q_heads=cfg.Hq, n_kv_heads=cfg.Hkv, head_dim=cfg.hd, rms_eps=cfg.rms_eps, rope_base=cfg.rope_base)
    # context K/V from a context-only forward (prefix and suffix see each other, at their own positions)
    xc = w_embed[np.concatenate([prefix_tok, suffix_tok])]
    pos_c = np.concatenate([np.arange(cfg.P), cfg.P + cfg.B + np.arange(S)])
    _, Kc, Vc = O.masked_forward(layers, xc, pos_c, np.ones((cfg.P + S, cfg.P + S), bool), **kw)
    allow, pos = O.verification_mask(cfg.P, cfg.B, cfg.G, S)
    x = w_embed[np.concatenate([prefix_tok, states.reshape(-1), suffix_tok])]
    hs, _, _ = O.masked_forward(layers, x, pos, allow, **kw)
    h = O.embed(w_embed, states)
    for l, w in enumerate(layers):
        h = O.verify_layer(w, Kc[l][:, :cfg.P], Vc[l][:, :cfg.P], h, pos0=cfg.P,
                           suffix_k=Kc[l][:, cfg.P:], suffix_v=Vc[l][:, cfg.P:], **kw)
    final = hs[-1][cfg.P:cfg.P + cfg.G * cfg.B].reshape(cfg.G, cfg.B, cfg.d)
    np.testing.assert_allclose(h, final, rtol=1e-10, atol=1e-12)
    # the mask: a draft that cannot see the suffix differs
    blind = allow.copy()
    blind[cfg.P + cfg.B:cfg.P + 2 * cfg.B, cfg.P + cfg.G * cfg.B:] = False
    hs_blind, _, _ = O.masked_forward(layers, x, pos, blind, **kw)
    assert np.abs(hs_blind[-1][cfg.P + cfg.B:cfg.P + 2 * cfg.B] - final[1]).max() > 1e-6
    # mask shape facts: symmetric context, G*B block rows each seeing P + S + B columns
    assert allow[:cfg.P].sum(1).tolist() == [cfg.P + S] * cfg.P
    assert allow[cfg.P:cfg.P + cfg.G * cfg.B].sum(1).tolist() == [cfg.P + S + cfg.B] * (cfg.G * cfg.B)
    assert pos[-S:].tolist() == list(range(cfg.P + cfg.B, cfg.P + cfg.B + S))


def test_scalar_brute_force_with_suffix():
    """Attention sums written out with Python scalars on a tiny shape, suffix keys after the block's."""
    cfg = small_cfg(d=8, Hq=2, Hkv=1, hd=4, F=6, P=2, B=2, G=1)
    S = 3
    w = layer_np(cfg, bias=True)
    w["wo"] = np.eye(cfg.d)
    w["w_down"][:] = 0
    pk, pv, sk, sv = _caches(cfg, S, seed=11)
    x = to_np(synth.hidden_states(cfg, 11))
    out = O.verify_layer(w, pk, pv, x, suffix_k=sk, suffix_v=sv, **cfg_kw(cfg))
    hd = cfg.hd

    def rot(vec, pos):
        half = hd // 2
        r = list(vec)
        for i in range(half):
            a = pos * cfg.rope_base ** (-2.0 * i / hd)
            r[i] = vec[i] * math.cos(a) - vec[i + half] * math.sin(a)
            r[i + half] = vec[i + half] * math.cos(a) + vec[i] * math.sin(a)
        return r

    n = O.rms_norm(x[0], w["norm1"], cfg.rms_eps)
    qs, ks, vs = n @ w["wq"].T + w["bq"], n @ w["wk"].T + w["bk"], n @ w["wv"].T + w["bv"]
    for b in range(cfg.B):
        o = []
        for h in range(cfg.Hq):
            q = rot(list(qs[b, h * hd:(h + 1) * hd]), cfg.P + b)
            keys = [list(pk[0, p]) for p in range(cfg.P)] + [rot(list(ks[c]), cfg.P + c) for c in range(cfg.B)] \
                + [list(sk[0, s]) for s in range(S)]
            vals = [list(pv[0, p]) for p in range(cfg.P)] + [list(vs[c]) for c in range(cfg.B)] \
                + [list(sv[0, s]) for s in range(S)]
            sc = [sum(q[i] * kk[i] for i in range(hd)) / math.sqrt(hd) for kk in keys]
            m = max(sc)
            e = [math.exp(s - m) for s in sc]
            z = sum(e)
            o += [sum(e[j] / z * vals[j][i] for j in range(len(keys))) for i in range(hd)]
        np.testing.assert_allclose(out[0, b] - x[0, b], o, rtol=1e-11, atol=1e-13)

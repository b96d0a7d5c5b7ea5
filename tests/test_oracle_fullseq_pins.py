"""Pins for the oracle's full-sequence verification (prefix cache only: the true suffix is recomputed in the call
and every draft attends to it; Sec. 4.3, Fig. 4, App. A.2), checked without a GPU."""
import numpy as np

from oracle import spiffy_oracle as O
from paper_2509_18085_amd import synth
from helpers import to_np
from test_oracle_pins import _tokens_model, layer_np, small_cfg


def _kw(cfg):
    return dict(n_q_heads=cfg.Hq, n_kv_heads=cfg.Hkv, head_dim=cfg.hd, rms_eps=cfg.rms_eps, rope_base=cfg.rope_base)


def fig4_mask(P, B, G, S):
    """[prefix ; block_0 .. block_{G-1} ; suffix]: the prefix is fixed context (sees itself only); block 0 and the
    suffix are the true sequence and see prefix, block 0 and suffix; a draft sees prefix, itself and the suffix."""
    T = P + G * B + S
    allow = np.zeros((T, T), bool)
    pre, suf, b0 = slice(0, P), slice(P + G * B, T), slice(P, P + B)
    allow[pre, pre] = True
    for rows in (b0, suf):
        allow[rows, pre] = allow[rows, b0] = allow[rows, suf] = True
    for g in range(1, G):
        r = slice(P + g * B, P + (g + 1) * B)
        allow[r, pre] = allow[r, r] = allow[r, suf] = True
    pos = np.concatenate([np.arange(P)] + [P + np.arange(B)] * G + [P + B + np.arange(S)])
    return allow, pos


def _setup(G=3, S=4, P=5, B=3):
    cfg = small_cfg(P=P, B=B, G=G)
    layers, w_embed = _tokens_model(cfg)
    r = np.random.default_rng(6)
    prefix_tok = r.integers(0, cfg.V - 1, cfg.P)
    states = synth.random_states(cfg.G, cfg.B, cfg.V, 0.3, 0.7, 10)
    suffix_tok = np.full(S, cfg.mask_id)
    suffix_tok[::3] = 7                                      # not all the same row, so order mistakes show
    return cfg, layers, w_embed, prefix_tok, states, suffix_tok


def test_dense_mask_formulation_through_all_layers():
    cfg, layers, w_embed, prefix_tok, states, suffix_tok = _setup()
    S = len(suffix_tok)
    kw = _kw(cfg)
    _, Kp, Vp = O.masked_forward(layers, w_embed[prefix_tok], np.arange(cfg.P), np.ones((cfg.P, cfg.P), bool), **kw)
    allow, pos = fig4_mask(cfg.P, cfg.B, cfg.G, S)
    x = w_embed[np.concatenate([prefix_tok, states.reshape(-1), suffix_tok])]
    hs, Kd, Vd = O.masked_forward(layers, x, pos, allow, **kw)
    hb, hsuf = O.embed(w_embed, states), O.embed(w_embed, suffix_tok)
    for l, w in enumerate(layers):
        hb, hsuf, k0, v0 = O.verify_layer_fullseq(w, Kp[l], Vp[l], hb, hsuf, pos0=cfg.P, return_kv=True, **kw)
        ref = hs[l + 1]
        # the keys / values handed back for the cache are those of the true block in the dense forward
        np.testing.assert_allclose(k0, Kd[l][:, cfg.P:cfg.P + cfg.B], rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(v0, Vd[l][:, cfg.P:cfg.P + cfg.B], rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(hb, ref[cfg.P:cfg.P + cfg.G * cfg.B].reshape(cfg.G, cfg.B, cfg.d), rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(hsuf, ref[cfg.P + cfg.G * cfg.B:], rtol=1e-10, atol=1e-12)
    # the mask matters where it should: a draft that sees the true block, or a suffix that sees a draft, differs
    for r0, c0 in ((cfg.P + cfg.B, cfg.P), (cfg.P + cfg.G * cfg.B, cfg.P + cfg.B)):
        leaky = allow.copy()
        leaky[r0:r0 + 2, c0:c0 + cfg.B] = True
        hl, _, _ = O.masked_forward(layers, x, pos, leaky, **kw)
        assert np.abs(hl[-1][r0:r0 + 2] - hs[-1][r0:r0 + 2]).max() > 1e-6


def test_one_state_is_a_plain_cached_forward_over_block_and_suffix():
    cfg, layers, w_embed, prefix_tok, states, suffix_tok = _setup(G=1)
    S = len(suffix_tok)
    kw = _kw(cfg)
    pk, pv = (to_np(t) for t in synth.prefix_kv(cfg, 0, 3))
    hb, hsuf = O.embed(w_embed, states), O.embed(w_embed, suffix_tok)
    ob, os_ = O.verify_layer_fullseq(layers[0], pk, pv, hb, hsuf, pos0=cfg.P, **kw)
    both = O.verify_layer(layers[0], pk, pv, np.concatenate([hb[0], hsuf])[None], pos0=cfg.P, **kw)[0]
    np.testing.assert_allclose(ob[0], both[:cfg.B], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(os_, both[cfg.B:], rtol=1e-12, atol=1e-13)
    # without a suffix it is the cached layer itself
    ob0, os0 = O.verify_layer_fullseq(layers[0], pk, pv, hb, hsuf[:0], pos0=cfg.P, **kw)
    np.testing.assert_array_equal(ob0, O.verify_layer(layers[0], pk, pv, hb, pos0=cfg.P, **kw))
    assert os0.shape == (0, cfg.d)


def test_drafts_do_not_reach_each_other_or_the_true_sequence():
    cfg, layers, w_embed, prefix_tok, states, suffix_tok = _setup(G=4)
    kw = _kw(cfg)
    pk, pv = (to_np(t) for t in synth.prefix_kv(cfg, 0, 3))
    hb, hsuf = O.embed(w_embed, states), O.embed(w_embed, suffix_tok)
    ob, os_ = O.verify_layer_fullseq(layers[0], pk, pv, hb, hsuf, pos0=cfg.P, **kw)
    hb2 = hb.copy()
    hb2[2] = hb[2][::-1]                                      # another draft 2
    ob2, os2 = O.verify_layer_fullseq(layers[0], pk, pv, hb2, hsuf, pos0=cfg.P, **kw)
    for g in (0, 1, 3):
        np.testing.assert_array_equal(ob2[g], ob[g])
    np.testing.assert_array_equal(os2, os_)
    assert np.abs(ob2[2] - ob[2]).max() > 1e-6
    # but the true block reaches the drafts through the suffix only from the next layer on: in one layer a
    # change of block 0 changes the suffix rows and block 0, not the drafts
    hb3 = hb.copy()
    hb3[0] = hb[0][::-1]
    ob3, os3 = O.verify_layer_fullseq(layers[0], pk, pv, hb3, hsuf, pos0=cfg.P, **kw)
    np.testing.assert_array_equal(ob3[1:], ob[1:])
    assert np.abs(os3 - os_).max() > 1e-6
    # draft duplicates of block 0 get block 0's output (they see the same keys)
    hb4 = hb.copy()
    hb4[3] = hb[0]
    ob4, _ = O.verify_layer_fullseq(layers[0], pk, pv, hb4, hsuf, pos0=cfg.P, **kw)
    np.testing.assert_allclose(ob4[3], ob4[0], rtol=1e-12, atol=1e-13)


def test_step_head_and_walk_run_on_the_blocks_only():
    cfg, layers, w_embed, prefix_tok, states, suffix_tok = _setup(G=3)
    hw = synth.head_weights(cfg, 5)
    prefix = [tuple(to_np(t) for t in synth.prefix_kv(cfg, l, 3)) for l in range(cfg.L)]
    edges = synth.edges_by_superset(states, cfg.mask_id)
    r = O.verify_step_fullseq(layers, prefix, w_embed, to_np(hw["final_norm"]), to_np(hw["w_vocab"]), states, suffix_tok, edges,
                              pos0=cfg.P, mask_id=cfg.mask_id, threshold=0.0, logit_scale=30.0, **_kw(cfg))
    assert r["hidden"].shape == (cfg.G, cfg.B, cfg.d) and r["hidden_suffix"].shape == (len(suffix_tok), cfg.d)
    head = O.decode_head(r["hidden"], to_np(hw["final_norm"]), to_np(hw["w_vocab"]), states, cfg.mask_id, 0.0,
                         rms_eps=cfg.rms_eps, logit_scale=30.0)
    np.testing.assert_array_equal(r["target_states"], head[4])
    assert (r["node"], r["depth"]) == O.graph_accept(edges, states, head[4], 0)[:2]


def test_decode_loop_of_a_full_sequence_model():
    """The block loop with a recomputed suffix: without a suffix it is the cached loop; with one, every pass is
    verify_step_fullseq on the current state, and the result does not depend on drafts (App. A)."""
    cfg, layers, w_embed, prefix_tok, states, suffix_tok = _setup(G=1, B=4)
    r = np.random.default_rng(0)
    rand_suffix = r.integers(0, cfg.V - 1, size=6)           # tokens that matter: the block decodes differently
    kw = dict(_kw(cfg), pos0=cfg.P, mask_id=cfg.mask_id, threshold=0.95, logit_scale=2.0, force_one=True)
    _, Kp, Vp = O.masked_forward(layers, w_embed[prefix_tok], np.arange(cfg.P), np.ones((cfg.P, cfg.P), bool), **_kw(cfg))
    model = dict(layers=layers, prefix=list(zip(Kp, Vp)), w_embed=w_embed, final_norm=np.ones(cfg.d),
                 w_vocab=r.standard_normal((cfg.V, cfg.d)) / np.sqrt(cfg.d), kw=kw)
    block0 = np.full(cfg.B, cfg.mask_id, np.int32)
    plain = O.decode_block(model, block0)
    empty = O.decode_block(dict(model, suffix_tokens=suffix_tok[:0]), block0)
    np.testing.assert_array_equal(plain[0], empty[0])
    assert plain[2] == empty[2]
    suffix_tok = rand_suffix
    seq_model = dict(model, suffix_tokens=suffix_tok)
    van = O.decode_block(seq_model, block0)
    assert not np.array_equal(van[0], plain[0])
    # every state of the trajectory is one full-sequence step from the one before
    for a, b in zip(van[1][:-1], van[1][1:]):
        step = O.verify_step_fullseq(layers, model["prefix"], w_embed, model["final_norm"], model["w_vocab"], a[None],
                                     suffix_tok, np.zeros((0, 2), np.int32), **kw)
        np.testing.assert_array_equal(step["accepted_state"], b)

    def drafter(state, info):                      # the right next state (a chain of two) and a wrong one
        nxt = O.verify_step_fullseq(layers, model["prefix"], w_embed, model["final_norm"], model["w_vocab"], state[None],
                                    suffix_tok, np.zeros((0, 2), np.int32), **kw)["accepted_state"]
        wrong = state.copy()
        wrong[np.flatnonzero(state == cfg.mask_id)[:1]] = 1
        return np.stack([nxt, wrong]), np.array([[0, 1], [0, 2]], np.int32)

    spec = O.decode_block(seq_model, block0, drafter=drafter)
    np.testing.assert_array_equal(spec[0], van[0])
    assert spec[2] < van[2]

"""GPU-vs-oracle parity through the C ABI (needs an MI355X: pytest -m gpu).

Bar: hidden states and confidences within 1e-4 (fp32) / 2e-2 (bf16) by the metric
|gpu - ref| / (|ref| + rms(ref)); argmax / unmask / next-state / acceptance decisions bit-exact
except where the oracle's top-2 logit margin is below 1e-3 (times the synthetic logit_scale knob
when that is above 1: the knob multiplies the rounding noise of the logits as well) or its
confidence is within 1e-4*tau of the threshold (both counted and printed).  Every call is
compared on identical input bits: bf16 inputs reach the oracle as the same values widened to
float64, and in the bf16 configuration the oracle rounds the normalised row to bf16 before the
vocabulary product, as the kernel's matrix-core operands are (decisions are taken from operands
of the same precision on both sides).
"""
import numpy as np
import pytest
import torch

from paper_2509_18085_amd import synth
import helpers
from helpers import np_weights, to_np

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(scope="module")
def sp():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2509_18085_amd import spiffy
    return spiffy


def O():
    from oracle import spiffy_oracle
    return spiffy_oracle


def rel_err(gpu, ref):
    ref = np.asarray(ref, np.float64)
    gpu = np.asarray(gpu, np.float64)
    rms = float(np.sqrt(np.mean(ref * ref))) + 1e-30
    return float(np.max(np.abs(gpu - ref) / (np.abs(ref) + rms))), float(
        np.linalg.norm(gpu - ref) / (np.linalg.norm(ref) + 1e-30))


def tol(cfg):
    return 1e-4 if cfg.dtype == "f32" else 2e-2


def dev_weights(w):
    return {k: v.to(DEV) for k, v in w.items()}


def oracle_kw(cfg, pos0=None):
    return dict(n_q_heads=cfg.Hq, n_kv_heads=cfg.Hkv, head_dim=cfg.hd, pos0=cfg.P if pos0 is None else pos0,
                rms_eps=cfg.rms_eps, rope_base=cfg.rope_base)


def run_layer(sp, cfg, w, pk, pv, hidden, pos0=None, G=None):
    scfg = sp.cfg_from_synth(cfg)
    G = hidden.shape[0]
    ws = sp.alloc_workspace(scfg, G, cfg.B, pk.shape[1] if pk is not None else 0, DEV)
    dw = dev_weights(w)
    lw = sp.layer_weights(dw)
    pf = sp.prefix_kv(None if pk is None else pk.to(DEV), None if pv is None else pv.to(DEV))
    out = sp.verify_layer(scfg, lw, pf, hidden.to(DEV), cfg.P if pos0 is None else pos0, ws)
    torch.cuda.synchronize()
    return out.cpu()


def check_layer(sp, cfg, seed=synth.DEFAULT_SEED, bias=False, hidden_std=1.0, pos0=None, weight_scale=None):
    w = synth.layer_weights(cfg, 0, seed, bias=bias)
    if weight_scale:
        for k in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down"):
            w[k] = (w[k].float() * weight_scale).to(w[k].dtype)
    pk, pv = synth.prefix_kv(cfg, 0, seed)
    x = synth.hidden_states(cfg, seed, std=hidden_std)
    got = run_layer(sp, cfg, w, pk, pv, x, pos0)
    ref = O().verify_layer(np_weights(w), to_np(pk), to_np(pv), to_np(x), **oracle_kw(cfg, pos0))
    e_max, e_norm = rel_err(to_np(got), ref)
    print("layer %s: max-rel %.3e  normwise %.3e" % (cfg.name, e_max, e_norm))
    assert e_max < tol(cfg), (cfg, e_max, e_norm)
    return got, ref


# ------------------------------------------------------------------ acceptance walk (bit-exact)

def test_accept_golden_and_random(sp):
    import json, os
    cases = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "accept_cases.json")))["cases"]
    for c in cases:
        e = torch.tensor(c["edges"], dtype=torch.int32, device=DEV).reshape(-1, 2)
        ds = torch.tensor(c["draft_states"], dtype=torch.int32, device=DEV)
        ts = torch.tensor(c["target_states"], dtype=torch.int32, device=DEV)
        res, state = sp.graph_accept(e, ds, ts, c.get("root", 0))
        res = res.cpu().tolist()
        assert res[:3] == [c["node"], c["depth"], c["depth"] + 1] and res[3] == 0, c["name"]
        assert state.cpu().tolist() == c["accepted_state"], c["name"]
    r = np.random.default_rng(3)
    for trial in range(60):
        G = int(r.integers(1, 65))
        B = int(r.choice([1, 3, 4, 8, 32, 33, 70]))
        levels = []
        left = G - 1
        while left > 0:
            n = int(min(left, r.integers(1, 9)))
            levels.append(n)
            left -= n
        st, e, _ = synth.grown_dag(levels, B, 50, 0.9, 1, 3, 100 + trial)
        tgt, path = synth.planted_targets(st, e, 50, int(r.integers(0, 6)), 200 + trial)
        if trial % 3 == 0 and len(e):
            e = e[r.permutation(len(e))]                   # edge order must not matter
        root = 0
        ref = O().graph_accept(e, st, tgt, root)
        res, state = sp.graph_accept(torch.from_numpy(np.ascontiguousarray(e)).to(DEV), torch.from_numpy(st).to(DEV),
                                     torch.from_numpy(tgt).to(DEV), root)
        assert tuple(res.cpu().tolist()[:3]) == ref[:3], (trial, G, B)
        assert state.cpu().tolist() == ref[3].tolist()


def test_accept_edge_cases(sp):
    # no edges, G = 1
    ds = torch.tensor([[5, 9, 9]], dtype=torch.int32, device=DEV)
    ts = torch.tensor([[5, 2, 9]], dtype=torch.int32, device=DEV)
    res, state = sp.graph_accept(None, ds, ts, 0)
    assert res.cpu().tolist() == [0, 0, 1, 0] and state.cpu().tolist() == [5, 2, 9]
    # out-of-range endpoints are ignored and flagged; a cycle terminates
    ds = torch.tensor([[9, 9], [1, 9], [1, 2]], dtype=torch.int32, device=DEV)
    ts = torch.tensor([[1, 9], [1, 2], [1, 9]], dtype=torch.int32, device=DEV)
    e = torch.tensor([[0, 1], [1, 2], [2, 1], [7, 1], [0, -1]], dtype=torch.int32, device=DEV)
    res, state = sp.graph_accept(e, ds, ts, 0)
    assert res.cpu().tolist() == [2, 2, 3, 1]
    # full subset lattice of the small-block configuration, walk to the all-unmasked leaf
    cfg = synth.CONFIGS["c5"]
    st, e = synth.draft_graph("c5", cfg)
    tgt = st.copy()
    order = [0, 1, 3, 7, 15]
    for a, b in zip(order[:-1], order[1:]):
        tgt[a] = st[b]
    tgt[15, 0] = 5
    ref = O().graph_accept(e, st, tgt, 0)
    res, state = sp.graph_accept(torch.from_numpy(e).to(DEV), torch.from_numpy(st).to(DEV),
                                 torch.from_numpy(tgt).to(DEV), 0)
    assert tuple(res.cpu().tolist()[:3]) == ref[:3] == (15, 4, 5)


# ------------------------------------------------------------------ embed

@pytest.mark.parametrize("key", ["c1", "bf16"])
def test_embed(sp, key):
    cfg = synth.CONFIGS["c1"] if key == "c1" else synth.CONFIGS["c1"].scaled(dtype="bf16")
    w = synth.embed_weights(cfg)
    st, _ = synth.draft_graph("c1", cfg)
    got = sp.embed(sp.cfg_from_synth(cfg), w.to(DEV), torch.from_numpy(st).to(DEV))
    np.testing.assert_array_equal(to_np(got), O().embed(to_np(w), st))


# ------------------------------------------------------------------ layer parity

def test_layer_config1_fp32(sp):
    check_layer(sp, synth.CONFIGS["c1"])
    check_layer(sp, synth.CONFIGS["c1"], bias=True, weight_scale=3.0)


@pytest.mark.parametrize("shape", [
    dict(d=64, Hq=2, Hkv=1, hd=32, F=40, P=0, B=5, G=3),          # no prefix, odd sizes
    dict(d=96, Hq=6, Hkv=2, hd=16, F=72, P=37, B=7, G=2),         # GQA, ragged everything
    dict(d=128, Hq=2, Hkv=2, hd=64, F=136, P=300, B=1, G=9),      # one-token blocks
])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_layer_generic_shapes(sp, shape, dtype):
    cfg = synth.CONFIGS["c1"].scaled(dtype=dtype, **shape)
    check_layer(sp, cfg, bias=True, weight_scale=4.0)


MFMA_SHAPES = [
    dict(d=512, Hq=4, Hkv=2, hd=128, F=768, P=200, B=32, G=5),    # GQA, ragged prefix tail, ragged row tail
    dict(d=256, Hq=2, Hkv=2, hd=128, F=320, P=64, B=4, G=40),     # small blocks: block-diagonal own keys
    dict(d=256, Hq=2, Hkv=1, hd=128, F=192, P=0, B=8, G=3),       # no prefix at all
    dict(d=256, Hq=2, Hkv=2, hd=128, F=256, P=2100, B=16, G=10),  # two prefix splits (the second a lone ragged tile) + combine
    dict(d=256, Hq=2, Hkv=2, hd=128, F=256, P=4200, B=8, G=20),   # three prefix splits, the last 1 full tile + ragged
    dict(d=256, Hq=2, Hkv=1, hd=128, F=256, P=128, B=32, G=3),    # exactly two full prefix tiles
    dict(d=256, Hq=2, Hkv=1, hd=128, F=256, P=192, B=32, G=9),    # exactly three full prefix tiles, three row tiles
    dict(d=384, Hq=3, Hkv=3, hd=128, F=448, P=1, B=64, G=3),      # block larger than a wave's 32 rows
    dict(d=256, Hq=2, Hkv=2, hd=128, F=256, P=130, B=24, G=7),    # block size that divides nothing
]


@pytest.mark.parametrize("shape", MFMA_SHAPES)
def test_layer_mfma_shapes(sp, shape):
    cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", V=1280, **shape)
    assert sp.uses_mfma(sp.cfg_from_synth(cfg), cfg.B) == 1
    check_layer(sp, cfg, bias=True, weight_scale=2.0)


def test_layer_mfma_batch_invariance_and_duplicates(sp):
    """A state's rows do not depend on which other states are verified with it (Sec. 4.3
    independence; App. A.2 remark on accumulation order): bit-identical across G and position."""
    cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", d=512, Hq=4, Hkv=2, hd=128, F=768, P=333, B=32, G=6, V=1280)
    w = synth.layer_weights(cfg, 0)
    pk, pv = synth.prefix_kv(cfg, 0)
    x = synth.hidden_states(cfg)
    x[4] = x[1]
    full = run_layer(sp, cfg, w, pk, pv, x)
    assert torch.equal(full[4], full[1])
    for g in (0, 3, 5):
        single = run_layer(sp, cfg, w, pk, pv, x[g:g + 1].contiguous())
        assert torch.equal(single[0], full[g]), g
    perm = [5, 2, 0, 4, 1, 3]
    shuffled = run_layer(sp, cfg, w, pk, pv, x[perm].contiguous())
    assert torch.equal(shuffled, full[perm])


def test_layer_rows_are_bit_identical_across_tile_heights(sp):
    """1 to 32 states run the projections on 32-, 64-, 128- and 256-row tiles (weight streaming with few rows):
    the tile shape is scheduling only, every state's rows come out bit-identical."""
    cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", d=1024, Hq=8, Hkv=8, hd=128, F=3072, P=200, B=32, G=32, V=1280)
    w = synth.layer_weights(cfg, 0)
    pk, pv = synth.prefix_kv(cfg, 0)
    x = synth.hidden_states(cfg)
    full = run_layer(sp, cfg, w, pk, pv, x)
    for lo, n in ((5, 1), (2, 2), (29, 3), (8, 4), (16, 8), (0, 16)):
        part = run_layer(sp, cfg, w, pk, pv, x[lo:lo + n].contiguous())
        assert torch.equal(part, full[lo:lo + n]), (lo, n)
    ref = O().verify_layer(np_weights(w), to_np(pk), to_np(pv), to_np(x[5:6]), **oracle_kw(cfg))
    e_max, _ = rel_err(to_np(full[5:6]), ref)
    assert e_max < tol(cfg), e_max


def test_reduction_thread_count_is_scheduling_only(sp):
    """The split-K reduction with its fused RMSNorm runs 1024 threads per row up to 512 rows and 256 beyond (rows of 4096
    elements); the row's sum of squares is taken chunk by chunk in a fixed order, so 32 states (1024 rows) and their
    first 8 or 16 (256 / 512 rows) give bit-identical rows."""
    cfg = synth.CONFIGS["c3"].scaled(L=1, F=512, V=1280, P=64)
    w = synth.layer_weights(cfg, 0)
    pk, pv = synth.prefix_kv(cfg, 0)
    x = synth.hidden_states(cfg)
    full = run_layer(sp, cfg, w, pk, pv, x)
    for n in (8, 16, 1):
        part = run_layer(sp, cfg, w, pk, pv, x[:n].contiguous())
        assert torch.equal(part, full[:n]), n
    ref = O().verify_layer(np_weights(w), to_np(pk), to_np(pv), to_np(x[3:4]), **oracle_kw(cfg))
    e_max, _ = rel_err(to_np(full[3:4]), ref)
    assert e_max < tol(cfg), e_max


@pytest.mark.parametrize("B,G", [(32, 24), (4, 192), (16, 48)])
def test_attention_query_tiles_of_96_rows_are_scheduling_only(sp, B, G):
    """28 query heads over 768 rows are 168 workgroups of 128 query rows, so the launch takes 96-row tiles (224
    workgroups, three wavefront pairs at work); a sixth of the states run 32-row tiles and half of them 64-row tiles.
    The rows of the states they share come out bit-identical, and a state matches the oracle.  Blocks of 32, 4 and 16
    tokens (3, 24 and 6 states per 96-row tile)."""
    cfg = synth.CONFIGS["c4"].scaled(L=1, F=512, V=1280, P=300, B=B, G=G)
    w = synth.layer_weights(cfg, 0)
    pk, pv = synth.prefix_kv(cfg, 0)
    x = synth.hidden_states(cfg)
    full = run_layer(sp, cfg, w, pk, pv, x)
    for lo, n in ((0, G // 6), (G // 4 + 1, G // 2), (G - G // 6, G // 6)):
        part = run_layer(sp, cfg, w, pk, pv, x[lo:lo + n].contiguous())
        assert torch.equal(part, full[lo:lo + n]), (lo, n)
    ref = O().verify_layer(np_weights(w), to_np(pk), to_np(pv), to_np(x[G - 1:G]), **oracle_kw(cfg))
    e_max, _ = rel_err(to_np(full[G - 1:G]), ref)
    assert e_max < tol(cfg), e_max


def test_layer_config2_full_size(sp):
    """One LLaDA-8B-shaped layer at the full configuration-2 size, all 512 rows against the oracle."""
    check_layer(sp, synth.CONFIGS["c2"])


def test_layer_shapes_of_configs_3_4_5_reduced_rows(sp):
    """Configurations 3-5 at their real widths, prefix lengths and block sizes, with fewer states
    so the oracle finishes in seconds; G keeps several row tiles and a ragged tail."""
    check_layer(sp, synth.CONFIGS["c3"].scaled(G=5))
    check_layer(sp, synth.CONFIGS["c4"].scaled(G=5))
    check_layer(sp, synth.CONFIGS["c5"].scaled(G=40, P=2500))


@pytest.mark.parametrize("key", ["c3", "c4", "c5"])
def test_layer_full_size_in_the_bench_launch_configuration(sp, key):
    """Configurations 3-5 at their full sizes (all G states, so the tile widths, K splits and key splits are the
    ones the benchmark times); the oracle computes sampled states, which it can do one by one because a state's
    rows depend on no other state."""
    cfg = synth.CONFIGS[key]
    w = synth.layer_weights(cfg, 0)
    pk, pv = synth.prefix_kv(cfg, 0)
    x = synth.hidden_states(cfg)
    got = run_layer(sp, cfg, w, pk, pv, x)
    sample = sorted({0, cfg.G // 2 - 1, cfg.G - 1})
    ref = O().verify_layer(np_weights(w), to_np(pk), to_np(pv), to_np(x[sample]), **oracle_kw(cfg))
    e_max, e_norm = rel_err(to_np(got[sample]), ref)
    print("full-size layer %s, states %s: max-rel %.3e  normwise %.3e" % (cfg.name, sample, e_max, e_norm))
    assert e_max < tol(cfg), (key, e_max, e_norm)
    assert torch.isfinite(got.float()).all()


@pytest.mark.parametrize("kind", ["mfma", "mfma_gqa_small_blocks", "generic_f32", "generic_bf16"])
def test_last_layer_computes_masked_rows_only(sp, kind):
    """spiffy_verify_layer_last: behind the attention only the rows of masked positions are computed.  Those rows equal
    spiffy_verify_layer's bit for bit (a row's arithmetic does not depend on the rows around it) and the oracle's
    within the layer tolerance; rows of unmasked positions are not written; a state with nothing masked, a fully
    masked state and a ragged row count are in the batch."""
    if kind == "mfma":
        cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", d=512, Hq=4, Hkv=4, hd=128, F=768, P=300, B=32, G=9, V=1280)
    elif kind == "mfma_gqa_small_blocks":
        cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", d=256, Hq=2, Hkv=1, hd=128, F=320, P=2100, B=4, G=70, V=1280)
    elif kind == "generic_f32":
        cfg = synth.CONFIGS["c1"].scaled(G=5)
    else:
        cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", d=96, Hq=6, Hkv=2, hd=16, F=72, P=37, B=7, G=4)
    st = synth.random_states(cfg.G, cfg.B, cfg.V, 0.2, 0.8, 21)
    st[1, :] = 3                     # nothing masked
    st[2, :] = cfg.mask_id           # everything masked
    w = synth.layer_weights(cfg, 0, bias=True)
    pk, pv = synth.prefix_kv(cfg, 0)
    x = synth.hidden_states(cfg)
    full = run_layer(sp, cfg, w, pk, pv, x)
    scfg = sp.cfg_from_synth(cfg)
    ws = sp.alloc_workspace(scfg, cfg.G, cfg.B, cfg.P, DEV)
    out = torch.full_like(x, 777.0).to(DEV)
    sp.verify_layer_last(scfg, sp.layer_weights(dev_weights(w)), sp.prefix_kv(pk.to(DEV), pv.to(DEV)), x.to(DEV),
                         torch.from_numpy(st).to(DEV), cfg.P, ws, out)
    torch.cuda.synchronize()
    out = out.cpu()
    m = torch.from_numpy(st == cfg.mask_id)
    assert torch.equal(out[m], full[m])
    assert (out[~m] == 777.0).all()
    # an explicit mask selects the rows instead of the tokens
    mask = torch.zeros((cfg.G, cfg.B), dtype=torch.uint8)
    mask[0, 0] = mask[cfg.G - 1, cfg.B - 1] = 1
    out2 = torch.full_like(x, 777.0).to(DEV)
    sp.verify_layer_last(scfg, sp.layer_weights(dev_weights(w)), sp.prefix_kv(pk.to(DEV), pv.to(DEV)), x.to(DEV),
                         torch.from_numpy(st).to(DEV), cfg.P, ws, out2, mask=mask.to(DEV))
    torch.cuda.synchronize()
    out2 = out2.cpu()
    assert torch.equal(out2[mask.bool()], full[mask.bool()]) and (out2[~mask.bool()] == 777.0).all()
    g = 2
    ref = O().verify_layer(np_weights(w), to_np(pk), to_np(pv), to_np(x[g:g + 1]), **oracle_kw(cfg))
    e_max, _ = rel_err(to_np(out[g:g + 1]), ref)
    assert e_max < tol(cfg), e_max


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_last_layer_with_nothing_masked_writes_nothing(sp, dtype):
    """Degenerate case: no masked position in the whole batch: the row count on the device is zero, every launch behind the
    attention finds nothing to do and hidden_out keeps what it held."""
    cfg = (synth.CONFIGS["c1"].scaled(dtype="bf16", d=256, Hq=2, Hkv=2, hd=128, F=320, P=70, B=32, G=3, V=1280)
           if dtype == "bf16" else synth.CONFIGS["c1"].scaled(G=3))
    st = np.full((cfg.G, cfg.B), 5, np.int32)
    w = synth.layer_weights(cfg, 0)
    pk, pv = synth.prefix_kv(cfg, 0)
    x = synth.hidden_states(cfg)
    scfg = sp.cfg_from_synth(cfg)
    ws = sp.alloc_workspace(scfg, cfg.G, cfg.B, cfg.P, DEV)
    out = torch.full_like(x, 777.0).to(DEV)
    sp.verify_layer_last(scfg, sp.layer_weights(dev_weights(w)), sp.prefix_kv(pk.to(DEV), pv.to(DEV)), x.to(DEV),
                         torch.from_numpy(st).to(DEV), cfg.P, ws, out)
    torch.cuda.synchronize()
    assert (out == 777.0).all()


@pytest.mark.parametrize("kind", ["mfma", "fp32"])
def test_step_without_hidden_output_decides_the_same(sp, kind):
    """spiffy_verify_step with hidden_out = NULL runs its last layer on the masked rows only: every decision, the
    confidences and the walk are those of the call that returns the hidden states, bit for bit."""
    if kind == "mfma":
        cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", L=2, d=256, Hq=2, Hkv=2, hd=128, F=320, V=1280, P=100, B=32, G=32)
        key, scale = "c3", 30.0
    else:
        cfg, key, scale = synth.CONFIGS["c1"], "c1", 40.0
    plan, layers, prefix, hw, w_embed, states, edges = build_step(sp, cfg, key, 5, scale)
    d_states, d_edges = torch.from_numpy(states).to(DEV), torch.from_numpy(edges).to(DEV)
    ref = {k: v.clone() for k, v in plan.run(d_states, d_edges).items()}
    torch.cuda.synchronize()
    for v in plan.out.values():
        v.fill_(0)
    plan.keep_hidden = False
    out = plan.run(d_states, d_edges)
    torch.cuda.synchronize()
    for k in ("argmax", "conf", "unmask", "margin", "target_states", "result", "accepted_state"):
        assert torch.equal(out[k], ref[k]), k
    assert (out["hidden"] == 0).all()          # not written
    assert int((states == cfg.mask_id).sum()) > 0


def test_step_two_layers_at_config3_size(sp):
    """The chained whole-step path at configuration 3's full row count, prefix length and widths (two layers to
    keep the oracle in seconds): hidden states of sampled states, and the walk on the step's own next states."""
    cfg = synth.CONFIGS["c3"].scaled(L=2, V=2048)
    plan, layers, prefix, hw, w_embed, states, edges = build_step(sp, cfg, "c3", synth.DEFAULT_SEED, 8.0)
    out = plan.run(torch.from_numpy(states).to(DEV), torch.from_numpy(edges).to(DEV))
    torch.cuda.synchronize()
    sample = [0, 13, cfg.G - 1]
    h = O().embed(to_np(w_embed), states[sample])
    for w, (pk, pv) in zip(layers, prefix):
        h = O().verify_layer(np_weights(w), to_np(pk), to_np(pv), h, **oracle_kw(cfg))
    e_max, e_norm = rel_err(to_np(out["hidden"][sample].cpu()), h)
    print("two chained layers at config 3 size: max-rel %.3e  normwise %.3e" % (e_max, e_norm))
    # the second layer adds its own rounding to the first layer's error carried through it: 3 x the one-layer bound
    assert e_max < 6e-2 and e_norm < 1.2e-2, (e_max, e_norm)
    ref = O().graph_accept(edges, states, out["target_states"].cpu().numpy(), 0)
    assert tuple(out["result"].cpu().tolist()[:3]) == ref[:3]
    assert out["accepted_state"].cpu().tolist() == ref[3].tolist()


def test_step_all_32_layers_end_to_end_report(sp):
    """End-to-end chaining at configuration 3: the whole step (32 bf16 layers, head, walk) on the device against the
    float64 oracle carried through all 32 layers on three sampled states (a state's rows depend on no other state).
    Weights are made on the device layer by layer and handed to the oracle one layer at a time.  Reported: the
    normwise error after every layer and the argmax / unmask agreement at the end (a 1e-2 hidden error moves
    logits by far more than the 1e-3 margin, so end-to-end decisions are not gated at bf16).  Gated: everything
    finite, and the error after L layers at most sqrt(L) times the one-layer figure (independent roundings add
    in quadrature; anything faster would be a systematic error)."""
    cfg = synth.CONFIGS["c3"]
    seed, scale = synth.DEFAULT_SEED, 8.0
    states, edges = synth.draft_graph("c3", cfg, seed)
    sample = [0, 13, cfg.G - 1]
    scfg = sp.cfg_from_synth(cfg)
    w_embed = synth.embed_weights(cfg, seed, device=DEV)
    hw = synth.head_weights(cfg, seed, device=DEV)
    d_states = torch.from_numpy(states).to(DEV)
    ws = sp.alloc_workspace(scfg, cfg.G, cfg.B, cfg.P, DEV)
    h_gpu = sp.embed(scfg, w_embed, d_states)
    h_ref = O().embed(to_np(w_embed[torch.from_numpy(np.unique(states)).to(DEV).long()]),
                      np.searchsorted(np.unique(states), states[sample]))      # only the rows in use leave the device
    d_layers, d_prefix, growth = [], [], []
    for l in range(cfg.L):
        w = synth.layer_weights(cfg, l, seed, device=DEV)
        pk, pv = synth.prefix_kv(cfg, l, seed, device=DEV)
        d_layers.append(w)
        d_prefix.append((pk, pv))
        h_gpu = sp.verify_layer(scfg, sp.layer_weights(w), sp.prefix_kv(pk, pv), h_gpu, cfg.P, ws)
        h_ref = O().verify_layer(np_weights(w), to_np(pk), to_np(pv), h_ref, **oracle_kw(cfg))
        e_max, e_norm = rel_err(to_np(h_gpu[sample]), h_ref)
        growth.append(e_norm)
        print("layer %2d: normwise %.3e  max-rel %.3e" % (l + 1, e_norm, e_max), flush=True)
    assert np.isfinite(growth).all() and torch.isfinite(h_gpu.float()).all()
    # the whole step in one call (its normalised rows are rounded at another place than in the layer-by-layer chain)
    plan = sp.StepPlan(scfg, [sp.layer_weights(w) for w in d_layers], [sp.prefix_kv(k, v) for k, v in d_prefix],
                       w_embed, hw["final_norm"], hw["w_vocab"], cfg.G, cfg.B, cfg.P, cfg.threshold, logit_scale=scale,
                       device=DEV)
    out = plan.run(d_states, torch.from_numpy(edges).to(DEV))
    torch.cuda.synchronize()
    e_step = rel_err(to_np(out["hidden"][sample]), h_ref)
    amax, conf, unmask, margin, target = O().decode_head(
        h_ref, to_np(hw["final_norm"]), to_np(hw["w_vocab"]), states[sample], cfg.mask_id, cfg.threshold,
        rms_eps=cfg.rms_eps, logit_scale=scale, force_one=True)
    m = states[sample] == cfg.mask_id
    g_amax, g_unmask = out["argmax"][sample].cpu().numpy(), out["unmask"][sample].cpu().numpy()
    g_conf = out["conf"][sample].cpu().numpy()
    rec = dict(kind="end_to_end_32_layers", config=cfg.name, states=sample, logit_scale=scale,
               normwise_error_per_layer=[float("%.4g" % e) for e in growth],
               step_call_normwise_error=float("%.4g" % e_step[1]), step_call_max_rel=float("%.4g" % e_step[0]),
               masked=int(m.sum()), argmax_agree=int((g_amax == amax)[m].sum()),
               unmask_agree=int((g_unmask == unmask)[m].sum()), oracle_unmasked=int(unmask.sum()),
               conf_median_rel_err=float(np.median(np.abs(g_conf[m] - conf[m]) / np.maximum(conf[m], 1e-30))),
               sqrt_L_times_first_layer=float("%.4g" % (np.sqrt(cfg.L) * growth[0])))
    helpers.REPORT.append(rec)
    print(rec)
    assert np.isfinite(g_conf).all() and np.isfinite(e_step).all()
    assert growth[-1] <= np.sqrt(cfg.L) * growth[0], (growth[0], growth[-1])
    assert e_step[1] <= 1.25 * np.sqrt(cfg.L) * growth[0], e_step
    # the walk is an integer procedure: exact on the step's own next states whatever the hidden error
    ref = O().graph_accept(edges, states, out["target_states"].cpu().numpy(), 0)
    assert tuple(out["result"].cpu().tolist()[:3]) == ref[:3]


# ------------------------------------------------------------------ head parity

def run_head(sp, cfg, hidden, hw, states, threshold, logit_scale, force_one):
    scfg = sp.cfg_from_synth(cfg)
    ws = sp.alloc_workspace(scfg, states.shape[0], cfg.B, 0, DEV)
    out = sp.decode_head(scfg, hidden.to(DEV), hw["final_norm"].to(DEV), hw["w_vocab"].to(DEV),
                         torch.from_numpy(states).to(DEV), threshold, ws, logit_scale=logit_scale,
                         force_one=force_one)
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in out.items()}


def check_head(sp, cfg, states, hidden, hw, threshold, logit_scale, force_one=True, max_excluded=0):
    """Decisions of the head against the oracle.  Gated: argmax where the oracle's top-2 logit margin is at least
    the tie margin; confidences; unmask and next state of every state that holds no near-tie, no confidence next to
    the threshold and no near-tie of the forced position; `max_excluded` is the stated ceiling on the states that
    drop out of that comparison.  Reported, not gated (bf16): the decisions that differ from the plain float64
    oracle, whose operands are not rounded to bf16, outside the literal margin of 1e-3."""
    got = run_head(sp, cfg, hidden, hw, states, threshold, logit_scale, force_one)
    kw = dict(rms_eps=cfg.rms_eps, logit_scale=logit_scale, force_one=force_one)
    amax, conf, unmask, margin, target = O().decode_head(
        to_np(hidden), to_np(hw["final_norm"]), to_np(hw["w_vocab"]), states, cfg.mask_id, threshold,
        operand_dtype="bf16" if cfg.dtype == "bf16" else None, **kw)
    m = states == cfg.mask_id
    tie = 1e-3 * max(1.0, logit_scale)
    near_tie = m & (margin < tie)
    near_tau = m & (np.abs(conf.astype(np.float64) - threshold) < 1e-4 * threshold)
    # force_one picks the best position by confidence: a state whose two best masked positions are
    # within 1e-6 relative is a near-tie of that decision
    ok_state = np.ones(states.shape[0], bool)
    for g in range(states.shape[0]):
        c = np.sort(conf[g][m[g]])[::-1]
        if near_tie[g].any() or near_tau[g].any() or (c.size > 1 and c[0] - c[1] < 1e-5 * c[0]):
            ok_state[g] = False
    rec = dict(config=cfg.name, d=cfg.d, V=cfg.V, states=int(states.shape[0]), logit_scale=logit_scale, tau=threshold,
               masked=int(m.sum()), near_tie=int(near_tie.sum()), near_tie_literal_1e_3=int((m & (margin < 1e-3)).sum()),
               near_threshold=int(near_tau.sum()), excluded_states=int((~ok_state).sum()), unmasked=int(unmask.sum()),
               argmax_mismatch_in_near_ties=int((got["argmax"] != amax)[near_tie].sum()))
    if cfg.dtype == "bf16":
        # the plain oracle: float64 all the way, the normalised row NOT rounded to the matrix cores' bf16
        p_amax, p_conf, p_unmask, p_margin, _ = O().decode_head(
            to_np(hidden), to_np(hw["final_norm"]), to_np(hw["w_vocab"]), states, cfg.mask_id, threshold,
            operand_dtype=None, **kw)
        lit = m & (p_margin >= 1e-3)
        far = m & (np.abs(p_conf.astype(np.float64) - threshold) >= 2e-2 * threshold)
        rec.update(plain_oracle_argmax_mismatch_outside_1e_3=int((got["argmax"] != p_amax)[lit].sum()),
                   plain_oracle_unmask_mismatch_away_from_tau=int((got["unmask"] != p_unmask)[far & lit].sum()),
                   plain_oracle_conf_max_rel=float(np.max(np.abs(got["conf"][m] - p_conf[m]) / np.maximum(p_conf[m], 1e-30)))
                   if m.any() else 0.0)
    helpers.REPORT.append(dict(kind="head_decisions", **rec))
    print("head decisions:", rec)
    clear = m & ~near_tie
    np.testing.assert_array_equal(got["argmax"][clear], amax[clear])
    np.testing.assert_array_equal(got["argmax"][~m], states[~m])
    assert (got["conf"][~m] == 0).all() and (got["unmask"][~m] == 0).all() and np.isinf(got["margin"][~m]).all()
    e_max = np.max(np.abs(got["conf"][m] - conf[m]) / np.maximum(conf[m], 1e-30)) if m.any() else 0.0
    t = 1e-4 if cfg.dtype == "f32" else 2e-2
    assert e_max < t, e_max
    big = clear & (margin > 10 * tie)
    if big.any():
        np.testing.assert_allclose(got["margin"][big], margin[big], rtol=2e-3, atol=tie)
    np.testing.assert_array_equal(got["unmask"][ok_state], unmask[ok_state])
    np.testing.assert_array_equal(got["target_states"][ok_state], target[ok_state])
    assert (~ok_state).sum() <= max_excluded, rec
    got["report"] = rec
    return got


@pytest.mark.parametrize("scale,tau,force", [(1.0, 0.9, True), (40.0, 0.9, True), (40.0, 0.3, False), (15.0, 0.0, False)])
def test_head_config1_fp32(sp, scale, tau, force):
    cfg = synth.CONFIGS["c1"]
    st, _ = synth.draft_graph("c1", cfg)
    check_head(sp, cfg, st, synth.hidden_states(cfg), synth.head_weights(cfg), tau, scale, force)


def test_head_generic_bf16_and_edge_masks(sp):
    cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", d=96, V=777, B=9, G=5)
    st = synth.random_states(cfg.G, cfg.B, cfg.V, 0.2, 0.8, 4)
    st[1, :] = cfg.mask_id          # fully masked state
    st[2, :] = 3                    # nothing masked: nothing to decode, nothing forced
    check_head(sp, cfg, st, synth.hidden_states(cfg), synth.head_weights(cfg), 0.5, 30.0)


@pytest.mark.parametrize("shape,scale,max_excluded", [
    (dict(d=256, V=1280, B=32, G=5), 40.0, 2),      # ragged row tile (at scale 40 the tie margin is 0.04: one near-tie, one forced position next to another)
    (dict(d=512, V=128 * 9, B=4, G=70), 25.0, 2),   # several row tiles, small blocks
    (dict(d=256, V=128, B=16, G=6), 20.0, 0),       # a single vocabulary tile
])
def test_head_mfma_shapes(sp, shape, scale, max_excluded):
    cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", Hq=2, Hkv=2, hd=128, F=256, **shape)
    st = synth.random_states(cfg.G, cfg.B, cfg.V, 0.1, 0.9, 6)
    st[0, :] = 7                    # a state with nothing masked
    check_head(sp, cfg, st, synth.hidden_states(cfg), synth.head_weights(cfg), 0.6, scale, max_excluded=max_excluded)


def test_head_nothing_masked_anywhere(sp):
    cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", d=256, V=1280, B=8, G=3)
    st = np.full((cfg.G, cfg.B), 5, np.int32)
    got = run_head(sp, cfg, synth.hidden_states(cfg), synth.head_weights(cfg), st, 0.9, 1.0, True)
    assert (got["unmask"] == 0).all() and (got["target_states"] == st).all()


@pytest.mark.parametrize("logit_scale", [8.0, 1.0])
def test_head_config3_shape_sampled_rows(sp, logit_scale):
    """Full vocabulary (126464) and width of configuration 3; 320 masked rows checked one by one, with the synthetic
    logit scale of the benchmark and at 1.0, the paper's own setting (Alg. 1 steps 1-3 on the raw logits: with
    random-init weights every confidence is then about 1/V and each state unmasks its single best position)."""
    cfg = synth.CONFIGS["c3"].scaled(G=12)
    st = synth.random_states(cfg.G, cfg.B, cfg.V, 0.8, 0.9, 8)
    hw = synth.head_weights(cfg)
    check_head(sp, cfg, st, synth.hidden_states(cfg), hw, cfg.threshold, logit_scale, max_excluded=1)


@pytest.mark.parametrize("logit_scale", [8.0, 1.0])
def test_head_config4_shape_sampled_rows(sp, logit_scale):
    """The head of configuration 4 (Dream-7B-shaped: d = 3584, V = 152064 = 594 vocabulary tiles of 256 rows), eight
    states, every masked row against the oracle."""
    cfg = synth.CONFIGS["c4"].scaled(G=8)
    st = synth.random_states(cfg.G, cfg.B, cfg.V, 0.7, 0.9, 9)
    hw = synth.head_weights(cfg)
    check_head(sp, cfg, st, synth.hidden_states(cfg), hw, cfg.threshold, logit_scale, max_excluded=2)


# ------------------------------------------------------------------ whole step

def build_step(sp, cfg, key, seed, logit_scale, n_layers=None):
    L = cfg.L if n_layers is None else n_layers
    layers = [synth.layer_weights(cfg, l, seed) for l in range(L)]
    prefix = [synth.prefix_kv(cfg, l, seed) for l in range(L)]
    hw = synth.head_weights(cfg, seed)
    w_embed = synth.embed_weights(cfg, seed)
    states, edges = synth.draft_graph(key, cfg, seed)
    scfg = sp.cfg_from_synth(cfg)
    d_layers = [dev_weights(w) for w in layers]
    d_prefix = [(k.to(DEV), v.to(DEV)) for k, v in prefix]
    plan = sp.StepPlan(scfg, [sp.layer_weights(w) for w in d_layers], [sp.prefix_kv(k, v) for k, v in d_prefix],
                       w_embed.to(DEV), hw["final_norm"].to(DEV), hw["w_vocab"].to(DEV), cfg.G, cfg.B, cfg.P,
                       cfg.threshold, logit_scale=logit_scale, device=DEV)
    return plan, layers, prefix, hw, w_embed, states, edges


@pytest.mark.parametrize("key,logit_scale", [("c1", 1.0), ("c1", 40.0), ("c1_literal", 40.0)])
def test_step_config1_end_to_end(sp, key, logit_scale):
    """Configuration 1 (fp32), the whole step in one call: hidden within 1e-4, every decision and
    the accepted node bit-exact (near-ties excluded and counted)."""
    cfg = synth.CONFIGS["c1"]
    plan, layers, prefix, hw, w_embed, states, edges = build_step(sp, cfg, key, synth.DEFAULT_SEED, logit_scale)
    out = plan.run(torch.from_numpy(states).to(DEV), torch.from_numpy(edges).to(DEV))
    torch.cuda.synchronize()
    ref = O().verify_step([np_weights(w) for w in layers], [(to_np(k), to_np(v)) for k, v in prefix],
                          to_np(w_embed), to_np(hw["final_norm"]), to_np(hw["w_vocab"]), states, edges,
                          n_q_heads=cfg.Hq, n_kv_heads=cfg.Hkv, head_dim=cfg.hd, pos0=cfg.P, mask_id=cfg.mask_id,
                          threshold=cfg.threshold, logit_scale=logit_scale)
    e_max, e_norm = rel_err(to_np(out["hidden"]), ref["hidden"])
    assert e_max < 1e-4, e_max
    m = states == cfg.mask_id
    clear = m & (ref["margin"] > 1e-3)
    print("step %s: hidden %.2e, near-ties %d" % (key, e_max, (m & ~clear).sum()))
    np.testing.assert_array_equal(out["argmax"].cpu().numpy()[clear], ref["argmax"][clear])
    if clear[m].all():
        np.testing.assert_array_equal(out["unmask"].cpu().numpy(), ref["unmask"])
        np.testing.assert_array_equal(out["target_states"].cpu().numpy(), ref["target_states"])
        res = out["result"].cpu().tolist()
        assert res[:3] == [ref["node"], ref["depth"], ref["n_steps"]]
        assert out["accepted_state"].cpu().tolist() == ref["accepted_state"].tolist()


def test_step_accept_follows_device_targets(sp):
    """Chained step on an MFMA shape (2 layers): the walk inside the step equals the oracle walk
    on the step's own next states, and each stage matches the oracle on the stage's own inputs."""
    cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", L=2, d=256, Hq=2, Hkv=2, hd=128, F=320, V=1280, P=100, B=32, G=32)
    plan, layers, prefix, hw, w_embed, states, edges = build_step(sp, cfg, "c3", 5, 30.0)
    out = plan.run(torch.from_numpy(states).to(DEV), torch.from_numpy(edges).to(DEV))
    torch.cuda.synchronize()
    tgt = out["target_states"].cpu().numpy()
    ref = O().graph_accept(edges, states, tgt, 0)
    assert tuple(out["result"].cpu().tolist()[:3]) == ref[:3]
    assert out["accepted_state"].cpu().tolist() == ref[3].tolist()
    # stage-wise: layers from the oracle's fp64 chain stay inside the bf16 tolerance after 2 layers
    h = O().embed(to_np(w_embed), states)
    for w, (pk, pv) in zip(layers, prefix):
        h = O().verify_layer(np_weights(w), to_np(pk), to_np(pv), h, **oracle_kw(cfg))
    e_max, _ = rel_err(to_np(out["hidden"]), h)
    assert e_max < 4e-2, e_max       # two chained bf16 layers
    # and the head on the step's own hidden
    check_head(sp, cfg, states, out["hidden"].cpu(), hw, cfg.threshold, 30.0, max_excluded=5)   # 32 states, 6 near-ties at margin 0.03


# ------------------------------------------------------------------ projection GEMM on its own

@pytest.mark.parametrize("M,N,K,epi", [
    (300, 384, 256, "store"),       # 192-wide tiles, ragged rows, short K
    (1024, 1536, 1024, "store"),    # 192-wide tiles, several row tiles, steady-state pipeline
    (70, 256, 192, "store"),        # 128-wide tiles, K of three tiles
    (100, 12288, 256, "store"),     # 64 x 96 tiles over two rows of tiles (256 workgroups), K shorter than the ring
    (200, 12288, 192, "store"),     # 128 x 96 tiles over two rows of tiles
    (513, 512, 2048, "resid"),      # sliced K (split-K) with residual, ragged rows
    (256, 128, 64, "resid"),        # single K tile
    (64, 192, 512, "resid"),        # N an odd multiple of 64: the unsliced launch must take 64-column tiles
    (300, 320, 1024, "resid"),      # the same with ragged rows and a K that is sliced when scratch is given
    (520, 384, 512, "swiglu"),      # gate/up interleave, 192-wide tiles (96 features per tile)
    (129, 320, 640, "swiglu"),      # 128-wide tiles (64 features per tile)
    (40, 12288, 1024, "swiglu"),    # few rows: 96-wide tiles (48 features, 256 workgroups), three of four wavefronts compute
    (100, 3072, 256, "swiglu"),     # 128 x 96 tiles, K shorter than the ring
    (768, 18944, 256, "swiglu"),    # two-part column schedule: 170 tiles of 96 features, then 128 x 128 tiles (config 4's width and rows)
    (600, 12288, 128, "swiglu"),    # two-part: one round of 256 x 192 tiles, the rest in 128 x 192 tiles; ragged rows
])
def test_gemm_against_float64_matmul(sp, M, N, K, epi):
    g = torch.Generator().manual_seed(M * 7 + N)
    A = (torch.randn((M, K), generator=g) * 0.5).to(torch.bfloat16)
    W0 = (torch.randn((N, K), generator=g) * 0.05).to(torch.bfloat16)
    W1 = (torch.randn((N, K), generator=g) * 0.05).to(torch.bfloat16)
    R = torch.randn((M, N), generator=g).to(torch.bfloat16)
    a, w0, w1, r = to_np(A), to_np(W0), to_np(W1), to_np(R)
    if epi == "store":
        got = sp.gemm(sp.GEMM_STORE, A.to(DEV), W0.to(DEV))
        ref = a @ w0.T
    elif epi == "resid":
        ws = torch.empty(4 * M * N * 4 + 256, dtype=torch.uint8, device=DEV)
        got = sp.gemm(sp.GEMM_RESID, A.to(DEV), W0.to(DEV), R=R.to(DEV), workspace=ws)
        direct = sp.gemm(sp.GEMM_RESID, A.to(DEV), W0.to(DEV), R=R.to(DEV))
        ref = r + a @ w0.T
        assert rel_err(to_np(direct.cpu()), ref)[0] < 1e-2
    else:
        got = sp.gemm(sp.GEMM_SWIGLU, A.to(DEV), W0.to(DEV), W1.to(DEV))
        gg = a @ w0.T
        ref = gg / (1.0 + np.exp(-gg)) * (a @ w1.T)
    torch.cuda.synchronize()
    e_max, e_norm = rel_err(to_np(got.cpu()), ref)
    assert e_max < 1e-2 and e_norm < 4e-3, (e_max, e_norm)


def test_gemm_seeded_random_shapes(sp):
    """Forty seeded shapes across the dispatcher's tile plans (ragged rows, one to five row tiles, widths that are odd
    multiples of 32 / 64, short K, wide gate/up launches that take the two-part schedule) against the float64 product;
    every launch plan is also checked to cover the columns once."""
    rng = np.random.default_rng(20250918)
    cases = []
    for _ in range(28):
        epi = ("store", "resid", "swiglu")[int(rng.integers(0, 3))]
        M = int(rng.integers(1, 1100))
        K = 64 * int(rng.integers(1, 13))
        N = (32 if epi == "swiglu" else 64) * int(rng.integers(1, 40))
        cases.append((epi, M, N, K))
    cases += [("swiglu", 1100, 6144, 64), ("swiglu", 900, 9504, 64), ("swiglu", 640, 12288, 64), ("swiglu", 400, 18944, 64),
              ("swiglu", 513, 18944, 128), ("store", 130, 12288, 64), ("store", 70, 9216, 128), ("store", 1030, 4608, 64),
              ("resid", 770, 3584, 1024), ("resid", 33, 4096, 2048), ("resid", 520, 1152, 640), ("swiglu", 1, 96, 64)]
    code = {"store": sp.GEMM_STORE, "resid": sp.GEMM_RESID, "swiglu": sp.GEMM_SWIGLU}
    for epi, M, N, K in cases:
        plan = sp.gemm_plan(code[epi], M, N, K, True)
        col = 0
        for l in plan["launches"]:
            assert l["col0"] == col
            col += l["n_cols"]
        assert col == N, (epi, M, N, K, plan)
        g = torch.Generator().manual_seed(M * 131 + N * 7 + K)
        A = (torch.randn((M, K), generator=g) * 0.5).to(torch.bfloat16)
        W0 = (torch.randn((N, K), generator=g) * 0.05).to(torch.bfloat16)
        a, w0 = to_np(A), to_np(W0)
        if epi == "store":
            got = sp.gemm(sp.GEMM_STORE, A.to(DEV), W0.to(DEV))
            ref = a @ w0.T
        elif epi == "resid":
            R = torch.randn((M, N), generator=g).to(torch.bfloat16)
            ws = torch.empty(4 * M * N * 4 + 256, dtype=torch.uint8, device=DEV)
            got = sp.gemm(sp.GEMM_RESID, A.to(DEV), W0.to(DEV), R=R.to(DEV), workspace=ws)
            ref = to_np(R) + a @ w0.T
        else:
            W1 = (torch.randn((N, K), generator=g) * 0.05).to(torch.bfloat16)
            got = sp.gemm(sp.GEMM_SWIGLU, A.to(DEV), W0.to(DEV), W1.to(DEV))
            gg = a @ w0.T
            ref = gg / (1.0 + np.exp(-gg)) * (a @ to_np(W1).T)
        torch.cuda.synchronize()
        e_max, e_norm = rel_err(to_np(got.cpu()), ref)
        assert e_max < 1e-2 and e_norm < 4e-3, (epi, M, N, K, plan, e_max, e_norm)


@pytest.mark.parametrize("N,K", [(4096, 4096), (4096, 12288), (1024, 2048)])
def test_split_k_projection_rows_do_not_depend_on_the_row_count(sp, N, K):
    """Output / down projection shapes: 32, 64, 96, 128 and 256 rows run on 32x32 (one wavefront), 64x32 (two),
    64x64 and taller tiles; the K slices and the order inside a slice are the same, so the first rows come out
    bit-identical, and they match the float64 product."""
    g = torch.Generator().manual_seed(N + K)
    A = (torch.randn((256, K), generator=g) * 0.5).to(torch.bfloat16).to(DEV)
    W = (torch.randn((N, K), generator=g) * 0.03).to(torch.bfloat16).to(DEV)
    R = torch.randn((256, N), generator=g).to(torch.bfloat16).to(DEV)
    ws = torch.empty(4 * 256 * N * 4 + 256, dtype=torch.uint8, device=DEV)
    full = sp.gemm(sp.GEMM_RESID, A, W, R=R, workspace=ws).clone()
    for n in (32, 64, 96, 128, 17, 45):
        part = sp.gemm(sp.GEMM_RESID, A[:n].contiguous(), W, R=R[:n].contiguous(), workspace=ws)
        assert torch.equal(part, full[:n]), n
    ref = to_np(R.cpu()) + to_np(A.cpu()) @ to_np(W.cpu()).T
    e_max, e_norm = rel_err(to_np(full.cpu()), ref)
    assert e_max < 1e-2 and e_norm < 4e-3, (e_max, e_norm)


def test_qkv_tile_shapes_are_scheduling_only(sp):
    """12288 columns: 40 rows run 64 x 64 tiles, 100 rows 64 x 96, 200 rows 128 x 96, 300 rows 128 x 192 and 1024 rows
    256 x 192; the common rows come out bit-identical."""
    N, K = 12288, 512
    g = torch.Generator().manual_seed(N + K)
    A = (torch.randn((1024, K), generator=g) * 0.5).to(torch.bfloat16).to(DEV)
    W = (torch.randn((N, K), generator=g) * 0.05).to(torch.bfloat16).to(DEV)
    full = sp.gemm(sp.GEMM_STORE, A, W).clone()
    for n in (40, 100, 200, 300):
        part = sp.gemm(sp.GEMM_STORE, A[:n].contiguous(), W)
        assert torch.equal(part, full[:n]), n


def test_gate_up_two_part_schedule_is_scheduling_only(sp):
    """At 18944 features the gate/up projection of 768 rows runs as two launches (256 x 192 tiles over the leading 16320
    features, 128 x 128 tiles over the rest) and that of 256 rows as one (256 x 128 tiles); 1024 rows take three rounds of
    256 x 192 tiles and 64 x 64 tiles for the last 512 features.  The K order of an element is the same in all of them:
    the common rows come out bit-identical."""
    F, K = 18944, 512
    g = torch.Generator().manual_seed(F + K)
    A = (torch.randn((1024, K), generator=g) * 0.5).to(torch.bfloat16).to(DEV)
    W0 = (torch.randn((F, K), generator=g) * 0.05).to(torch.bfloat16).to(DEV)
    W1 = (torch.randn((F, K), generator=g) * 0.05).to(torch.bfloat16).to(DEV)
    full = sp.gemm(sp.GEMM_SWIGLU, A, W0, W1).clone()
    for n in (768, 512, 256, 40):
        part = sp.gemm(sp.GEMM_SWIGLU, A[:n].contiguous(), W0, W1)
        assert torch.equal(part, full[:n]), n


def test_small_block_duplicates_are_bit_identical(sp):
    """Small-block configuration: every unmask-subset state appears four times; copies must give
    bit-identical rows and (through the whole step) identical decisions."""
    cfg = synth.CONFIGS["c5"].scaled(L=1, d=512, Hq=4, Hkv=4, F=768, V=1280, P=1500)
    st, e = synth.draft_graph("c5", synth.CONFIGS["c5"])
    st = np.where(st == synth.CONFIGS["c5"].mask_id, cfg.mask_id, st % (cfg.V - 1)).astype(np.int32)
    plan, layers, prefix, hw, w_embed, _, _ = build_step(sp, cfg, "c5", 3, 30.0)
    out = plan.run(torch.from_numpy(st).to(DEV), torch.from_numpy(e).to(DEV))
    torch.cuda.synchronize()
    hid = out["hidden"].cpu()
    n = 1 << cfg.B
    for k in range(1, cfg.G // n):
        assert torch.equal(hid[:n], hid[k * n:(k + 1) * n]), k
        for key in ("argmax", "unmask", "target_states"):
            assert torch.equal(out[key][:n], out[key][k * n:(k + 1) * n]), (k, key)
        assert torch.equal(out["conf"][:n], out["conf"][k * n:(k + 1) * n])


# ------------------------------------------------------------------ drafting and pruning (Sec. 4.4)

def _draft_case(rng, B, K, V, D, tie_grid):
    mask_id = V
    state = np.array([mask_id if rng.random() < 0.6 else int(rng.integers(0, V)) for _ in range(B)], np.int32)
    tok = np.stack([rng.choice(V, size=K, replace=False) for _ in range(B)]).astype(np.int32)
    if tie_grid:      # a coarse grid: equal confidences and equal scores do occur, and are exact in float32
        prob = np.sort(rng.integers(1, 9, size=(B, K)) / 16.0, axis=1)[:, ::-1].astype(np.float32)
    else:
        prob = np.sort(rng.uniform(0.01, 1.0, size=(B, K)), axis=1)[:, ::-1].astype(np.float32)
    n_masked = int((state == mask_id).sum())
    formulas = []
    for _ in range(D):
        k = int(rng.integers(1, 5))
        hi = max(1, n_masked + 1)
        ranks = rng.choice(np.arange(1, hi + 1), size=min(k, hi), replace=False)
        f = [(int(i), int(rng.integers(1, K + 2))) for i in ranks]
        if rng.random() < 0.1 and len(f) > 1:
            f[1] = (f[0][0], f[1][1])                       # the same position twice
        formulas.append(f)
    sets = [set()] + [set(f) for f in formulas]
    edges = [(a, c) for a in range(D + 1) for c in range(1, D + 1) if a != c and sets[a] < sets[c]]
    edges += edges[:2]                                      # repeated edges count once
    return state, mask_id, tok, prob, formulas, np.array(edges, np.int32).reshape(-1, 2)


def _run_draft_prune(sp, state, mask_id, tok, prob, formulas, edges, d_star):
    off = np.cumsum([0] + [len(f) for f in formulas]).astype(np.int32)
    pairs = np.array([p for f in formulas for p in f], np.int32).reshape(-1, 2)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    out = sp.draft_prune(t(state), mask_id, t(tok), t(prob), t(off), t(pairs) if len(pairs) else None,
                         t(edges) if len(edges) else None, d_star)
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in out.items()}


@pytest.mark.parametrize("seed", range(10))
def test_draft_prune_parity(sp, seed):
    """Draft blocks, buildability and the kept sub-graph bit-exact; scores to float32 rounding.  The
    decision 'which d_star nodes are kept' is compared where the oracle's scores around the cut are
    separated by more than float32 rounding of the geometric means (equal scores are exact on the tie
    grid and go to the lower node on both sides)."""
    rng = np.random.default_rng(900 + seed)
    B = int(rng.choice([4, 32, 33, 200]))
    K = int(rng.integers(1, 5))
    D = int(rng.choice([0, 1, 7, 23, 63]))
    state, mask_id, tok, prob, formulas, edges = _draft_case(rng, B, K, 1000, D, tie_grid=seed % 2 == 0)
    d_star = int(rng.integers(0, D + 2))
    got = _run_draft_prune(sp, state, mask_id, tok, prob, formulas, edges, d_star)
    ref = O().draft_and_prune(state, mask_id, tok, prob.astype(np.float64), formulas, edges, d_star)
    np.testing.assert_array_equal(got["drafts"], ref["drafts"])
    np.testing.assert_array_equal(got["buildable"].astype(bool), ref["buildable"])
    for name in ("local", "score"):
        g, r = got[name].astype(np.float64), ref[name]
        assert (np.isnan(g) == np.isnan(r)).all(), name
        ok = ~np.isnan(r)
        np.testing.assert_allclose(g[ok], r[ok], rtol=2e-6, atol=1e-12, err_msg=name)
    sc = np.sort(ref["score"][1:][ref["buildable"][1:]])[::-1]
    n_keep = min(d_star, len(sc))
    clear_cut = True
    if 0 < n_keep < len(sc):
        a, b = sc[n_keep - 1], sc[n_keep]
        clear_cut = a == b or (a - b) > 1e-5 * a
    # scores that are equal in exact arithmetic must also be equal in float32 for the index rule to agree
    uniq = np.unique(sc)
    exact_ties_ok = all((b - a) > 1e-5 * b for a, b in zip(uniq, uniq[1:])) or seed % 2 == 0
    assert int(got["counts"][0]) == 1 + n_keep
    if clear_cut and exact_ties_ok:
        np.testing.assert_array_equal(got["kept"][:1 + n_keep], ref["kept"])
        np.testing.assert_array_equal(got["states"][:1 + n_keep], ref["states"])
        assert int(got["counts"][1]) == len(ref["edges"])
        np.testing.assert_array_equal(got["edges"][:len(ref["edges"])], ref["edges"])


def test_draft_prune_golden_and_edge_cases(sp):
    import json, os
    g = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "draft_prune_case.json")))
    formulas = [[tuple(p) for p in f] for f in g["formulas"]]
    got = _run_draft_prune(sp, np.array(g["state"], np.int32), g["mask_id"], np.array(g["topk_tokens"], np.int32),
                           np.array(g["topk_probs"], np.float32), formulas, np.array(g["edges"], np.int32), g["d_star"])
    e = g["expected"]
    np.testing.assert_array_equal(got["drafts"], np.array(e["drafts"]))
    assert got["kept"][:int(got["counts"][0])].tolist() == e["kept"]
    assert got["edges"][:int(got["counts"][1])].tolist() == e["edges"]
    for name in ("local", "score"):
        for a, b in zip(got[name], e[name]):
            assert (b is None and np.isnan(a)) or abs(a - b) < 1e-6
    # nothing masked: no formula can be built, only the root is kept, no edge survives
    st = np.arange(8, dtype=np.int32)
    got = _run_draft_prune(sp, st, 99, np.zeros((8, 1), np.int32), np.ones((8, 1), np.float32),
                           [[(1, 1)], [(1, 1), (2, 1)]], np.array([[0, 1], [1, 2]], np.int32), 2)
    assert got["buildable"].tolist() == [1, 0, 0] and got["counts"].tolist() == [1, 0]
    np.testing.assert_array_equal(got["drafts"], np.tile(st, (3, 1)))
    # no formulas at all, no edges
    got = _run_draft_prune(sp, np.full(5, 7, np.int32), 7, np.zeros((5, 2), np.int32),
                           np.full((5, 2), 0.5, np.float32), [], np.zeros((0, 2), np.int32), 3)
    assert got["counts"].tolist() == [1, 0] and got["kept"][0] == 0
    # offsets that do not increase: that formula is not built, the others are
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    out = sp.draft_prune(t(np.full(4, 9, np.int32)), 9, t(np.arange(4, dtype=np.int32).reshape(4, 1)),
                         t(np.array([[.9], [.8], [.7], [.6]], np.float32)), t(np.array([0, 1, 1, 2], np.int32)),
                         t(np.array([[1, 1], [2, 1]], np.int32)), None, 3)
    torch.cuda.synchronize()
    assert out["buildable"].cpu().tolist() == [1, 1, 0, 1]
    assert out["drafts"].cpu().tolist() == [[9, 9, 9, 9], [0, 9, 9, 9], [9, 9, 9, 9], [9, 1, 9, 9]]


def test_draft_prune_feeds_the_next_step(sp):
    """Closed loop on the device: verify -> draft from the accepted node's top-1 rows -> verify again.
    With formulas 'the s most confident positions' one of the drafts is the target of the accepted
    state (threshold rule, Sec. 3.1) and the walk accepts it at depth >= 1, as the oracle does."""
    cfg = synth.CONFIGS["c1"]
    seed = synth.DEFAULT_SEED
    layers = [synth.layer_weights(cfg, l, seed) for l in range(cfg.L)]
    prefix = [synth.prefix_kv(cfg, l, seed) for l in range(cfg.L)]
    hw = synth.head_weights(cfg, seed)
    we = synth.embed_weights(cfg, seed)
    scfg = sp.cfg_from_synth(cfg)
    scale = 40.0
    plan1 = sp.StepPlan(scfg, [sp.layer_weights(dev_weights(w)) for w in layers],
                        [sp.prefix_kv(k.to(DEV), v.to(DEV)) for k, v in prefix], we.to(DEV),
                        hw["final_norm"].to(DEV), hw["w_vocab"].to(DEV), 1, cfg.B, cfg.P, 0.5,
                        logit_scale=scale, device=DEV)
    state0 = np.full((1, cfg.B), cfg.mask_id, np.int32)
    state0[0, 1] = 5
    out1 = plan1.run(torch.from_numpy(state0).to(DEV), None)
    torch.cuda.synchronize()
    new_state = out1["accepted_state"].clone()
    # formulas: the s most confident masked positions, s = 1..B, chained by inclusion
    formulas = [[(i, 1) for i in range(1, n + 1)] for n in range(1, cfg.B + 1)]
    off = torch.tensor(np.cumsum([0] + [len(f) for f in formulas]).astype(np.int32), device=DEV)
    pairs = torch.tensor(np.array([p for f in formulas for p in f], np.int32), device=DEV)
    edges = torch.tensor(np.array([[a, c] for a in range(cfg.B + 1) for c in range(a + 1, cfg.B + 1)], np.int32),
                         device=DEV)
    d_star = 3
    dp = sp.draft_prune(new_state, cfg.mask_id, out1["argmax"][0].reshape(cfg.B, 1).contiguous(),
                        out1["conf"][0].reshape(cfg.B, 1).contiguous(), off, pairs, edges, d_star)
    torch.cuda.synchronize()
    n_kept, n_edges = [int(x) for x in dp["counts"].cpu()]
    assert n_kept == 1 + min(d_star, int((new_state == cfg.mask_id).sum()))
    plan2 = sp.StepPlan(scfg, [sp.layer_weights(dev_weights(w)) for w in layers],
                        [sp.prefix_kv(k.to(DEV), v.to(DEV)) for k, v in prefix], we.to(DEV),
                        hw["final_norm"].to(DEV), hw["w_vocab"].to(DEV), n_kept, cfg.B, cfg.P, 0.5,
                        logit_scale=scale, device=DEV)
    out2 = plan2.run(dp["states"][:n_kept].contiguous(), dp["edges"][:n_edges].contiguous())
    torch.cuda.synchronize()
    # oracle on the same two steps
    m = dict(layers=[np_weights(w) for w in layers], prefix=[(to_np(k), to_np(v)) for k, v in prefix],
             w_embed=to_np(we), final_norm=to_np(hw["final_norm"]), w_vocab=to_np(hw["w_vocab"]))
    kw = dict(n_q_heads=cfg.Hq, n_kv_heads=cfg.Hkv, head_dim=cfg.hd, pos0=cfg.P, mask_id=cfg.mask_id,
              threshold=0.5, rms_eps=cfg.rms_eps, rope_base=cfg.rope_base, logit_scale=scale, force_one=True)
    r1 = O().verify_step(m["layers"], m["prefix"], m["w_embed"], m["final_norm"], m["w_vocab"], state0,
                         np.zeros((0, 2), np.int32), **kw)
    np.testing.assert_array_equal(new_state.cpu().numpy(), r1["accepted_state"])
    rdp = O().draft_and_prune(r1["accepted_state"], cfg.mask_id, r1["argmax"][0].reshape(-1, 1),
                              r1["conf"][0].reshape(-1, 1).astype(np.float64), formulas, edges.cpu().numpy(), d_star)
    np.testing.assert_array_equal(dp["states"][:n_kept].cpu().numpy(), rdp["states"])
    r2 = O().verify_step(m["layers"], m["prefix"], m["w_embed"], m["final_norm"], m["w_vocab"], rdp["states"],
                         rdp["edges"], **kw)
    res = out2["result"].cpu().tolist()
    assert res[0] == r2["node"] and res[1] == r2["depth"]
    np.testing.assert_array_equal(out2["accepted_state"].cpu().numpy(), r2["accepted_state"])


# ------------------------------------------------------------------ drafting source: top-K per position

def check_head_topk(sp, cfg, states, hidden, hw, logit_scale, K, nodes):
    """spiffy_head_topk after spiffy_decode_head against oracle.head_topk.  Column 0 must be exactly the
    argmax / conf of the head pass; rank j tokens are compared where the oracle's logit gaps to the
    neighbouring ranks exceed the tie margin (the ranking is an integer decided by floats)."""
    scfg = sp.cfg_from_synth(cfg)
    G = states.shape[0]
    ws = sp.alloc_workspace(scfg, G, cfg.B, 0, DEV)
    wv = hw["w_vocab"].to(DEV)
    d_states = torch.from_numpy(states).to(DEV)
    out = sp.decode_head(scfg, hidden.to(DEV), hw["final_norm"].to(DEV), wv, d_states, 0.9, ws,
                         logit_scale=logit_scale, force_one=True)
    tie = 1e-3 * max(1.0, logit_scale)
    n_cmp = 0
    for node in nodes:
        tok, prob = sp.head_topk(scfg, wv, d_states, K, logit_scale, ws, node=node)
        torch.cuda.synchronize()
        tok, prob = tok.cpu().numpy(), prob.cpu().numpy()
        kk = min(K + 1, cfg.V)
        rt, rp = O().head_topk(to_np(hidden)[node], to_np(hw["final_norm"]), to_np(hw["w_vocab"]), kk,
                               rms_eps=cfg.rms_eps, logit_scale=logit_scale,
                               operand_dtype="bf16" if cfg.dtype == "bf16" else "f64")
        amax, conf = out["argmax"][node].cpu().numpy(), out["conf"][node].cpu().numpy()
        for b in range(cfg.B):
            if states[node, b] != cfg.mask_id:
                assert (tok[b] == states[node, b]).all() and (prob[b] == 0).all()
                continue
            assert tok[b, 0] == amax[b] and prob[b, 0] == conf[b]
            logp = np.log(np.maximum(rp[b], 1e-300))
            gaps = logp[:-1] - logp[1:]                       # logit gap between rank j and j+1
            for j in range(min(K, cfg.V)):
                clear = (j == 0 or gaps[j - 1] > tie) and (j >= len(gaps) or gaps[j] > tie)
                if clear:
                    assert tok[b, j] == rt[b, j], (node, b, j, tok[b], rt[b])
                    assert abs(prob[b, j] - rp[b, j]) <= (1e-4 if cfg.dtype == "f32" else 2e-2) * rp[b, j] + 1e-30
                    n_cmp += 1
            assert (np.diff(prob[b][tok[b] >= 0]) <= 1e-7).all()
            assert len(set(tok[b][tok[b] >= 0].tolist())) == int((tok[b] >= 0).sum())
            if K > cfg.V:
                assert (tok[b, cfg.V:] == -1).all() and (prob[b, cfg.V:] == 0).all()
    assert n_cmp > 0
    return n_cmp


def test_head_topk_config1_fp32(sp):
    cfg = synth.CONFIGS["c1"]
    st, _ = synth.draft_graph("c1", cfg)
    for K, scale in ((1, 1.0), (3, 15.0), (8, 40.0)):
        check_head_topk(sp, cfg, st, synth.hidden_states(cfg), synth.head_weights(cfg), scale, K, range(cfg.G))


def test_head_topk_generic_bf16_small_vocab(sp):
    cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", d=96, V=5, B=9, G=3)
    st = synth.random_states(cfg.G, cfg.B, cfg.V, 0.3, 0.9, 4)
    st[1, :] = cfg.mask_id
    check_head_topk(sp, cfg, st, synth.hidden_states(cfg), synth.head_weights(cfg), 3.0, 8, range(cfg.G))


@pytest.mark.parametrize("V,K", [(1280, 2), (1000, 4), (300, 8), (126464, 3)])
def test_head_topk_mfma_refinement(sp, V, K):
    """MFMA head: the K best tokens come from recomputing the K best 128-token chunks of every row (ragged
    last chunk, K larger than the number of chunks, the full LLaDA vocabulary)."""
    cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", d=256, V=V, B=8 if V > 100000 else 32, G=3)
    assert sp.uses_mfma(sp.cfg_from_synth(cfg), cfg.B) in (0, 1)
    st = synth.random_states(cfg.G, cfg.B, cfg.V, 0.2, 0.9, 11)
    st[2, :] = cfg.mask_id
    check_head_topk(sp, cfg, st, synth.hidden_states(cfg), synth.head_weights(cfg), 6.0, K, (0, 2))


def test_head_topk_after_step_with_device_result(sp):
    """After spiffy_verify_step, node taken from the device-side accept result; K = 2 formulas feed
    spiffy_draft_prune and the pruned graph is what the oracle builds from the same distribution."""
    cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", L=2, d=256, Hq=2, Hkv=2, hd=128, F=320, V=1280, P=100, B=32, G=4)
    seed = 5
    layers = [synth.layer_weights(cfg, l, seed) for l in range(cfg.L)]
    prefix = [synth.prefix_kv(cfg, l, seed) for l in range(cfg.L)]
    hw = synth.head_weights(cfg, seed)
    we = synth.embed_weights(cfg, seed)
    scfg = sp.cfg_from_synth(cfg)
    scale = 12.0
    plan = sp.StepPlan(scfg, [sp.layer_weights(dev_weights(w)) for w in layers],
                       [sp.prefix_kv(k.to(DEV), v.to(DEV)) for k, v in prefix], we.to(DEV),
                       hw["final_norm"].to(DEV), hw["w_vocab"].to(DEV), cfg.G, cfg.B, cfg.P, 0.9,
                       logit_scale=scale, device=DEV)
    states = synth.random_states(cfg.G, cfg.B, cfg.V, 0.3, 0.8, 3)
    d_states = torch.from_numpy(states).to(DEV)
    out = plan.run(d_states, None)
    K = 2
    tok, prob = sp.head_topk(scfg, plan.w_vocab, d_states, K, scale, plan.workspace, result=out["result"],
                             after_step=True)
    torch.cuda.synchronize()
    node = int(out["result"][0].item())
    assert node == 0                       # no edges: the root is accepted
    hidden = out["hidden"][node].float().cpu().numpy().astype(np.float64)
    rt, rp = O().head_topk(hidden, to_np(hw["final_norm"]), to_np(hw["w_vocab"]), K + 1, rms_eps=cfg.rms_eps,
                           logit_scale=scale, operand_dtype="bf16")
    tie = 1e-3 * scale
    m = states[node] == cfg.mask_id
    logp = np.log(rp)
    clear = m & (logp[:, 0] - logp[:, 1] > tie) & (logp[:, 1] - logp[:, 2] > tie)
    assert clear.sum() >= 4
    np.testing.assert_array_equal(tok.cpu().numpy()[clear], rt[clear][:, :K])
    np.testing.assert_allclose(prob.cpu().numpy()[clear], rp[clear][:, :K], rtol=2e-2)
    # the drafting kernel takes these rows as they are
    new_state = out["accepted_state"]
    formulas = [[(1, 1)], [(1, 2)], [(1, 1), (2, 1)], [(1, 1), (2, 2)]]
    off = torch.tensor(np.cumsum([0] + [len(f) for f in formulas]).astype(np.int32), device=DEV)
    pairs = torch.tensor(np.array([p for f in formulas for p in f], np.int32), device=DEV)
    edges = torch.tensor(np.array([[0, 1], [0, 2], [1, 3], [1, 4]], np.int32), device=DEV)
    dp = sp.draft_prune(new_state, cfg.mask_id, tok, prob, off, pairs, edges, 3)
    torch.cuda.synchronize()
    ref = O().draft_and_prune(new_state.cpu().numpy(), cfg.mask_id, tok.cpu().numpy(),
                              prob.cpu().numpy().astype(np.float64), formulas, edges.cpu().numpy(), 3)
    np.testing.assert_array_equal(dp["drafts"].cpu().numpy(), ref["drafts"])
    n_kept = int(dp["counts"][0].item())
    np.testing.assert_array_equal(dp["kept"][:n_kept].cpu().numpy(), ref["kept"])


def test_layer_and_head_at_the_row_limit(sp):
    """G = SPIFFY_MAX_G states of 256 tokens = SPIFFY_MAX_ROWS rows (64 row tiles, blocks that span eight
    32-row query groups), narrow model so the oracle finishes in seconds."""
    cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", d=256, Hq=2, Hkv=1, hd=128, F=256, V=640, P=70, B=256, G=64)
    assert cfg.G * cfg.B == 16384
    check_layer(sp, cfg)
    st = synth.random_states(cfg.G, cfg.B, cfg.V, 0.05, 0.3, 9)
    # 64 fully masked states, 2924 rows over a 640-token vocabulary at margin 6e-3: 21 near-ties in 16 states
    check_head(sp, cfg, st, synth.hidden_states(cfg), synth.head_weights(cfg), 0.9, 6.0, max_excluded=18)


def test_single_token_blocks(sp):
    """B = 1: every state is one token that attends to the prefix and to itself."""
    cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", d=256, Hq=2, Hkv=2, hd=128, F=256, V=640, P=150, B=1, G=37)
    check_layer(sp, cfg)


# ------------------------------------------------------------------ prefix-cache extension and the decode loop

def _oracle_commit(m, kw, block, P):
    """Oracle side of spiffy_commit_block: forward of the finished block, its rotated K and V appended."""
    h = O().embed(m["w_embed"], block[None, :])
    new_prefix = []
    for w, (pk, pv) in zip(m["layers"], m["prefix"]):
        h, ks, vs = O().verify_layer(w, pk, pv, h, n_q_heads=kw["n_q_heads"], n_kv_heads=kw["n_kv_heads"],
                                     head_dim=kw["head_dim"], pos0=P, rms_eps=kw["rms_eps"],
                                     rope_base=kw["rope_base"], return_kv=True)
        new_prefix.append((np.concatenate([pk, ks[0]], axis=1), np.concatenate([pv, vs[0]], axis=1)))
    return new_prefix


def _decoder_setup(sp, cfg, seed, n_blocks, threshold, scale, graph, d_star, graph_replay=False):
    from paper_2509_18085_amd import decode
    layers = [synth.layer_weights(cfg, l, seed) for l in range(cfg.L)]
    prefix = [synth.prefix_kv(cfg, l, seed) for l in range(cfg.L)]
    hw = synth.head_weights(cfg, seed)
    we = synth.embed_weights(cfg, seed)
    cap = cfg.P + n_blocks * cfg.B
    ck, cv = [], []
    for k, v in prefix:
        kk = torch.zeros((cfg.Hkv, cap, cfg.hd), dtype=k.dtype, device=DEV)
        vv = torch.zeros_like(kk)
        kk[:, :cfg.P] = k.to(DEV)
        vv[:, :cfg.P] = v.to(DEV)
        ck.append(kk)
        cv.append(vv)
    dec = decode.BlockDecoder(sp.cfg_from_synth(cfg), [dev_weights(w) for w in layers], ck, cv, cfg.P, we.to(DEV),
                              hw["final_norm"].to(DEV), hw["w_vocab"].to(DEV), cfg.B, threshold, logit_scale=scale,
                              graph=graph, d_star=d_star, device=DEV, graph_replay=graph_replay)
    m = dict(layers=[np_weights(w) for w in layers], prefix=[(to_np(k), to_np(v)) for k, v in prefix],
             w_embed=to_np(we), final_norm=to_np(hw["final_norm"]), w_vocab=to_np(hw["w_vocab"]))
    kw = dict(n_q_heads=cfg.Hq, n_kv_heads=cfg.Hkv, head_dim=cfg.hd, pos0=cfg.P, mask_id=cfg.mask_id,
              threshold=threshold, rms_eps=cfg.rms_eps, rope_base=cfg.rope_base, logit_scale=scale, force_one=True)
    return dec, ck, cv, m, kw


@pytest.mark.parametrize("key", ["c1", "bf16_mfma"])
def test_commit_block_appends_the_blocks_keys_and_values(sp, key):
    cfg = synth.CONFIGS["c1"] if key == "c1" else synth.CONFIGS["c1"].scaled(
        dtype="bf16", L=2, d=256, Hq=4, Hkv=2, hd=128, F=320, V=640, P=70, B=32, G=1)
    dec, ck, cv, m, kw = _decoder_setup(sp, cfg, 3, 2, 0.9, 1.0, None, 0)
    before_k = [k.clone() for k in ck]
    block = np.random.default_rng(1).integers(0, cfg.V, size=cfg.B).astype(np.int32)
    dec.commit(torch.from_numpy(block).to(DEV))
    torch.cuda.synchronize()
    ref = _oracle_commit(m, kw, block, cfg.P)
    t = tol(cfg)
    for l in range(cfg.L):
        gk, gv = to_np(ck[l]), to_np(cv[l])
        np.testing.assert_array_equal(gk[:, :cfg.P], to_np(before_k[l])[:, :cfg.P])          # context untouched
        assert (gk[:, cfg.P + cfg.B:] == 0).all() and (gv[:, cfg.P + cfg.B:] == 0).all()       # nothing beyond the block
        for got, want in ((gk, ref[l][0]), (gv, ref[l][1])):
            e_max, _ = rel_err(got[:, cfg.P:cfg.P + cfg.B], want[:, cfg.P:])
            assert e_max < t, (l, e_max)
    assert dec.P == cfg.P + cfg.B


def test_decode_two_blocks_matches_the_oracle_loop(sp):
    """Configuration 1 (fp32): the device loop verify -> top-K -> draft/prune -> verify, with the cache extended
    between blocks, produces the oracle's tokens, forward-pass counts and accepted depths; and the same tokens as
    vanilla decoding on the device (losslessness, App. A) with NFE_vanilla - NFE = accepted drafts that still
    had a MASK."""
    from paper_2509_18085_amd import decode
    cfg = synth.CONFIGS["c1"]
    scale, tau, d_star = 12.0, 0.5, 3
    formulas = [[(i, 1) for i in range(1, n + 1)] for n in range(1, 5)] + [[(1, 2)], [(1, 1), (2, 2)]]
    graph = decode.DraftGraph(formulas, device=DEV)
    dec, _, _, m, kw = _decoder_setup(sp, cfg, synth.DEFAULT_SEED, 2, tau, scale, graph, d_star)
    got = dec.generate(2)
    vdec, _, _, _, _ = _decoder_setup(sp, cfg, synth.DEFAULT_SEED, 2, tau, scale, None, 0)
    van = vdec.generate(2)
    np.testing.assert_array_equal(got["tokens"], van["tokens"])
    assert all(n <= v for n, v in zip(got["nfe"], van["nfe"])) and sum(got["nfe"]) < sum(van["nfe"])

    # the oracle's loop with the same drafter
    def drafter(state, info):
        if not info:
            return np.zeros((0, state.size), np.int32), np.zeros((0, 2), np.int32)
        t, p = O().head_topk(info["hidden"][info["node"]], m["final_norm"], m["w_vocab"], graph.K,
                             rms_eps=kw["rms_eps"], logit_scale=scale)
        out = O().draft_and_prune(state, cfg.mask_id, t, p, formulas, graph.edges_np, d_star)
        return out["states"][1:], out["edges"]

    tokens, nfes, depths = [], [], []
    P = cfg.P
    for _ in range(2):
        model = dict(m, kw=dict(kw, pos0=P))
        block0 = np.full(cfg.B, cfg.mask_id, np.int32)
        final, traj, nfe, dps, _ = O().decode_block(model, block0, drafter=drafter)
        tokens.append(final)
        nfes.append(nfe)
        depths.append(dps)
        m["prefix"] = _oracle_commit(m, model["kw"], final, P)
        P += cfg.B
    np.testing.assert_array_equal(got["tokens"], np.concatenate(tokens))
    assert got["nfe"] == nfes and got["depths"] == depths


def test_decode_is_lossless_on_the_mfma_path(sp):
    """bf16 MFMA kernels: a row's arithmetic does not depend on the states verified with it, so speculative
    decoding reproduces vanilla decoding token for token over several blocks, in fewer forward passes."""
    from paper_2509_18085_amd import decode
    cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", L=2, d=256, Hq=2, Hkv=2, hd=128, F=320, V=1280, P=100, B=32, G=1)
    formulas = [[(i, 1) for i in range(1, n + 1)] for n in (1, 2, 3, 4, 6, 8, 12, 16)] + [[(1, 2)], [(1, 1), (2, 2)]]
    graph = decode.DraftGraph(formulas, device=DEV)
    dec, _, _, _, _ = _decoder_setup(sp, cfg, 11, 3, 0.7, 16.0, graph, 5)
    vdec, _, _, _, _ = _decoder_setup(sp, cfg, 11, 3, 0.7, 16.0, None, 0)
    got, van = dec.generate(3), vdec.generate(3)
    np.testing.assert_array_equal(got["tokens"], van["tokens"])
    assert not (got["tokens"] == cfg.mask_id).any()
    assert sum(got["nfe"]) < sum(van["nfe"])
    assert sum(sum(d) for d in got["depths"]) >= sum(van["nfe"]) - sum(got["nfe"])


@pytest.mark.parametrize("key", ["c1", "bf16_mfma"])
@pytest.mark.parametrize("drafting", [True, False])
def test_decode_passes_replayed_from_a_graph_equal_the_eager_loop(sp, key, drafting):
    """graph_replay: every pass after a block's first is one launch of a HIP graph recorded for that block (verify,
    top-K, drafting, pruning and the next pass's inputs at the fixed shape of 1 + d_star states).  Tokens, forward
    passes, accepted depths and the number of states the pruning kept equal the eager loop's, with and without
    drafts, over three blocks (a new recording per block: the prefix grows)."""
    from paper_2509_18085_amd import decode
    if key == "c1":
        cfg, tau, scale = synth.CONFIGS["c1"].scaled(G=1), 0.6, 40.0
    else:
        cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", L=2, d=256, Hq=2, Hkv=2, hd=128, F=320, V=1280, P=100, B=32, G=1)
        tau, scale = 0.7, 16.0
    n_max = min(cfg.B, 8)
    formulas = [[(i, 1) for i in range(1, n + 1)] for n in range(1, n_max + 1)] + [[(1, 2)], [(1, 1), (2, 2)]]
    mk = lambda replay: _decoder_setup(sp, cfg, 11, 3, tau, scale, decode.DraftGraph(formulas, device=DEV) if drafting else None,
                                       5 if drafting else 0, graph_replay=replay)[0]
    eager, replay = mk(False), mk(True)
    a, b = eager.generate(3), replay.generate(3)
    np.testing.assert_array_equal(a["tokens"], b["tokens"])
    assert a["nfe"] == b["nfe"] and a["depths"] == b["depths"] and a["n_states"] == b["n_states"]
    assert replay.graph_launches == sum(n - 1 for n in b["nfe"]) and replay.graph_launches > 0
    assert not (b["tokens"] == cfg.mask_id).any()


# ------------------------------------------------------------------ dual cache: fixed K/V of the tokens after the block

def _full_cache(cfg, S, seed, layer=0, extra=0):
    """[Hkv, P+B+S+extra, hd] caches: prefix rows, the block's slot (filled with a large value that must never
    be read), suffix rows."""
    pk, pv = synth.prefix_kv(cfg, layer, seed)
    sk, sv = synth.suffix_kv(cfg, layer, S, seed)
    cap = cfg.P + cfg.B + S + extra
    ck = torch.full((cfg.Hkv, cap, cfg.hd), 1e4, dtype=pk.dtype)
    cv = torch.full((cfg.Hkv, cap, cfg.hd), 1e4, dtype=pk.dtype)
    ck[:, :cfg.P], cv[:, :cfg.P] = pk, pv
    ck[:, cfg.P + cfg.B:cfg.P + cfg.B + S], cv[:, cfg.P + cfg.B:cfg.P + cfg.B + S] = sk, sv
    return ck, cv, pk, pv, sk, sv


def check_layer_dual(sp, cfg, S, seed=5, bias=False):
    w = synth.layer_weights(cfg, 0, seed, bias=bias)
    ck, cv, pk, pv, sk, sv = _full_cache(cfg, S, seed, extra=3)
    x = synth.hidden_states(cfg, seed)
    scfg = sp.cfg_from_synth(cfg)
    ws = sp.alloc_workspace(scfg, cfg.G, cfg.B, cfg.P + S, DEV)
    pf = sp.prefix_kv(ck.to(DEV), cv.to(DEV), cfg.P, S)
    got = sp.verify_layer(scfg, sp.layer_weights(dev_weights(w)), pf, x.to(DEV), cfg.P, ws)
    torch.cuda.synchronize()
    ref = O().verify_layer(np_weights(w), to_np(pk), to_np(pv), to_np(x), suffix_k=to_np(sk), suffix_v=to_np(sv),
                           **oracle_kw(cfg))
    e_max, e_norm = rel_err(to_np(got.cpu()), ref)
    print("dual-cache layer %s P=%d S=%d: max-rel %.3e  normwise %.3e" % (cfg.name, cfg.P, S, e_max, e_norm))
    assert e_max < tol(cfg), (cfg, S, e_max, e_norm)
    return got


def test_layer_dual_cache_generic(sp):
    check_layer_dual(sp, synth.CONFIGS["c1"], 24, bias=True)
    check_layer_dual(sp, synth.CONFIGS["c1"].scaled(P=0), 5)
    check_layer_dual(sp, synth.CONFIGS["c1"].scaled(dtype="bf16", P=37, B=5, G=3), 11)


@pytest.mark.parametrize("P,S", [(100, 70), (0, 64), (64, 1), (1024, 224), (2000, 300), (2048, 2049), (4200, 224)])
def test_layer_dual_cache_mfma(sp, P, S):
    """Suffix parts of one and of several key splits, ragged tails in both parts, a split whose rows come from
    both parts (2000 + 300), an empty prefix."""
    cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", d=256, Hq=2, Hkv=1, hd=128, F=256, P=P, B=32, G=5)
    assert sp.uses_mfma(sp.cfg_from_synth(cfg), cfg.B) == 1
    check_layer_dual(sp, cfg, S)


def test_dual_cache_rows_are_context_wherever_they_sit(sp):
    """MFMA path: a suffix of S rows gives the output of a prefix cache that holds the same rows (keys are
    already rotated), to rounding of the different summation order; S = 0 is bit-identical to no suffix."""
    cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", d=256, Hq=2, Hkv=2, hd=128, F=256, P=192, B=32, G=4)
    S = 128
    a = check_layer_dual(sp, cfg, S)
    w = synth.layer_weights(cfg, 0, 5)
    _, _, pk, pv, sk, sv = _full_cache(cfg, S, 5)
    x = synth.hidden_states(cfg, 5)
    b = run_layer(sp, cfg.scaled(P=cfg.P + S), w, torch.cat([pk, sk], 1), torch.cat([pv, sv], 1), x, pos0=cfg.P)
    e_max, _ = rel_err(to_np(a.cpu()), to_np(b))
    assert e_max < 2e-2
    c = run_layer(sp, cfg, w, pk, pv, x)
    scfg = sp.cfg_from_synth(cfg)
    ws = sp.alloc_workspace(scfg, cfg.G, cfg.B, cfg.P, DEV)
    pad = torch.zeros((cfg.Hkv, cfg.P + 40, cfg.hd), dtype=pk.dtype)
    pad[:, :cfg.P] = pk
    padv = pad.clone()
    padv[:, :cfg.P] = pv
    d = sp.verify_layer(scfg, sp.layer_weights(dev_weights(w)), sp.prefix_kv(pad.to(DEV), padv.to(DEV), cfg.P, 0),
                        x.to(DEV), cfg.P, ws)
    assert torch.equal(d.cpu(), c)


@pytest.mark.parametrize("key", ["c1", "bf16_mfma"])
def test_step_and_commit_with_dual_cache(sp, key):
    """Whole step with suffix rows against the oracle; then the block is committed into its slot between prefix
    and suffix, and the appended rows match the oracle's keys / values of a block that attended to both."""
    cfg = synth.CONFIGS["c1"] if key == "c1" else synth.CONFIGS["c1"].scaled(
        dtype="bf16", L=2, d=256, Hq=4, Hkv=2, hd=128, F=320, V=640, P=70, B=32, G=4)
    S, seed, scale = 2 * cfg.B, 9, 8.0
    scfg = sp.cfg_from_synth(cfg)
    layers = [synth.layer_weights(cfg, l, seed) for l in range(cfg.L)]
    caches = [_full_cache(cfg, S, seed, layer=l) for l in range(cfg.L)]
    hw, we = synth.head_weights(cfg, seed), synth.embed_weights(cfg, seed)
    states, edges = synth.draft_graph("c1", cfg.scaled(G=4), seed)
    dk = [c[0].to(DEV) for c in caches]
    dv = [c[1].to(DEV) for c in caches]
    plan = sp.StepPlan(scfg, [sp.layer_weights(dev_weights(w)) for w in layers],
                       [sp.prefix_kv(k, v, cfg.P, S) for k, v in zip(dk, dv)], we.to(DEV), hw["final_norm"].to(DEV),
                       hw["w_vocab"].to(DEV), len(states), cfg.B, cfg.P, 0.5, logit_scale=scale, device=DEV)
    out = plan.run(torch.from_numpy(states).to(DEV), torch.from_numpy(np.ascontiguousarray(edges)).to(DEV))
    torch.cuda.synchronize()
    m = dict(layers=[np_weights(w) for w in layers], prefix=[(to_np(c[2]), to_np(c[3])) for c in caches],
             suffix=[(to_np(c[4]), to_np(c[5])) for c in caches])
    ref = O().verify_step(m["layers"], m["prefix"], to_np(we), to_np(hw["final_norm"]), to_np(hw["w_vocab"]), states, edges,
                          n_q_heads=cfg.Hq, n_kv_heads=cfg.Hkv, head_dim=cfg.hd, pos0=cfg.P, mask_id=cfg.mask_id,
                          threshold=0.5, rms_eps=cfg.rms_eps, rope_base=cfg.rope_base, logit_scale=scale,
                          suffix=m["suffix"])
    e_max, _ = rel_err(to_np(out["hidden"].cpu()), ref["hidden"])
    assert e_max < (1e-4 if cfg.dtype == "f32" else 4e-2), e_max         # bf16: two chained layers
    masked = states == cfg.mask_id
    if cfg.dtype == "f32":
        safe = masked & (ref["margin"] > 1e-3 * max(1.0, scale))
        np.testing.assert_array_equal(out["argmax"].cpu().numpy()[safe], ref["argmax"][safe])
    else:       # decisions from the step's own hidden states, operands of the same precision on both sides
        amax, _, _, margin, _ = O().decode_head(to_np(out["hidden"].cpu()), to_np(hw["final_norm"]), to_np(hw["w_vocab"]),
                                                states, cfg.mask_id, 0.5, rms_eps=cfg.rms_eps, logit_scale=scale,
                                                operand_dtype="bf16")
        safe = masked & (margin > 1e-3 * max(1.0, scale))
        np.testing.assert_array_equal(out["argmax"].cpu().numpy()[safe], amax[safe])
    tgt = out["target_states"].cpu().numpy()
    walk = O().graph_accept(edges, states, tgt, 0)
    assert tuple(out["result"].cpu().tolist()[:3]) == walk[:3]
    # commit a finished block into its slot
    block = np.random.default_rng(2).integers(0, cfg.V - 1, size=cfg.B).astype(np.int32)
    plan.commit_block(torch.from_numpy(block).to(DEV))
    torch.cuda.synchronize()
    h = O().embed(to_np(we), block[None, :])
    for l in range(cfg.L):
        h, ks, vs = O().verify_layer(m["layers"][l], m["prefix"][l][0], m["prefix"][l][1], h, suffix_k=m["suffix"][l][0],
                                     suffix_v=m["suffix"][l][1], return_kv=True, **oracle_kw(cfg))
        gk, gv = to_np(dk[l].cpu()), to_np(dv[l].cpu())
        for got, want in ((gk, ks[0]), (gv, vs[0])):
            e_max, _ = rel_err(got[:, cfg.P:cfg.P + cfg.B], want)
            assert e_max < tol(cfg), (l, e_max)
        np.testing.assert_array_equal(gk[:, cfg.P + cfg.B:], to_np(caches[l][0])[:, cfg.P + cfg.B:])   # suffix untouched
        np.testing.assert_array_equal(gk[:, :cfg.P], to_np(caches[l][0])[:, :cfg.P])


def test_decode_with_dual_cache_matches_the_oracle_loop(sp):
    """Configuration 1 (fp32), two blocks with 2B suffix rows after the first: device loop = oracle loop
    (tokens, forward passes, depths); each committed block takes B rows off the suffix."""
    from paper_2509_18085_amd import decode
    cfg = synth.CONFIGS["c1"]
    scale, tau, d_star, seed, S0 = 12.0, 0.5, 3, synth.DEFAULT_SEED, 2 * cfg.B
    formulas = [[(i, 1) for i in range(1, n + 1)] for n in range(1, 5)] + [[(1, 2)], [(1, 1), (2, 2)]]
    layers = [synth.layer_weights(cfg, l, seed) for l in range(cfg.L)]
    caches = [_full_cache(cfg, S0, seed, layer=l) for l in range(cfg.L)]
    hw, we = synth.head_weights(cfg, seed), synth.embed_weights(cfg, seed)

    def run(graph, d):
        ck = [c[0].clone().to(DEV) for c in caches]
        cv = [c[1].clone().to(DEV) for c in caches]
        dec = decode.BlockDecoder(sp.cfg_from_synth(cfg), [dev_weights(w) for w in layers], ck, cv, cfg.P, we.to(DEV),
                                  hw["final_norm"].to(DEV), hw["w_vocab"].to(DEV), cfg.B, tau, logit_scale=scale,
                                  graph=graph, d_star=d, device=DEV, S0=S0)
        return dec.generate(2)

    graph = decode.DraftGraph(formulas, device=DEV)
    got, van = run(graph, d_star), run(None, 0)
    np.testing.assert_array_equal(got["tokens"], van["tokens"])
    assert sum(got["nfe"]) < sum(van["nfe"])

    lw = [np_weights(w) for w in layers]
    full_k = [to_np(c[0]) for c in caches]
    full_v = [to_np(c[1]) for c in caches]
    w_np = dict(w_embed=to_np(we), final_norm=to_np(hw["final_norm"]), w_vocab=to_np(hw["w_vocab"]))

    def drafter(state, info):
        if not info:
            return np.zeros((0, state.size), np.int32), np.zeros((0, 2), np.int32)
        t, p = O().head_topk(info["hidden"][info["node"]], w_np["final_norm"], w_np["w_vocab"], graph.K,
                             rms_eps=cfg.rms_eps, logit_scale=scale)
        out = O().draft_and_prune(state, cfg.mask_id, t, p, formulas, graph.edges_np, d_star)
        return out["states"][1:], out["edges"]

    tokens, nfes, depths = [], [], []
    P, S = cfg.P, S0
    for _ in range(2):
        prefix = [(k[:, :P], v[:, :P]) for k, v in zip(full_k, full_v)]
        suffix = [(k[:, P + cfg.B:P + cfg.B + S], v[:, P + cfg.B:P + cfg.B + S]) for k, v in zip(full_k, full_v)]
        kw = dict(n_q_heads=cfg.Hq, n_kv_heads=cfg.Hkv, head_dim=cfg.hd, pos0=P, mask_id=cfg.mask_id, threshold=tau,
                  rms_eps=cfg.rms_eps, rope_base=cfg.rope_base, logit_scale=scale, force_one=True, suffix=suffix)
        model = dict(layers=lw, prefix=prefix, kw=kw, **w_np)
        final, _, nfe, dps, _ = O().decode_block(model, np.full(cfg.B, cfg.mask_id, np.int32), drafter=drafter)
        tokens.append(final)
        nfes.append(nfe)
        depths.append(dps)
        h = O().embed(w_np["w_embed"], final[None, :])
        for l in range(cfg.L):
            h, ks, vs = O().verify_layer(lw[l], prefix[l][0], prefix[l][1], h, suffix_k=suffix[l][0], suffix_v=suffix[l][1],
                                         return_kv=True, **oracle_kw(cfg, P))
            full_k[l][:, P:P + cfg.B], full_v[l][:, P:P + cfg.B] = ks[0], vs[0]
        P, S = P + cfg.B, S - cfg.B
    np.testing.assert_array_equal(got["tokens"], np.concatenate(tokens))
    assert got["nfe"] == nfes and got["depths"] == depths


# ------------------------------------------------------------------ calibration: optimal connected subgraph

def _run_subgraph(sp, count, level, edges, D):
    e = np.asarray(edges, np.int32).reshape(-1, 2)
    out = sp.subgraph_search(torch.tensor(np.asarray(count), dtype=torch.int64, device=DEV),
                             torch.tensor(np.asarray(level), dtype=torch.int32, device=DEV),
                             torch.from_numpy(np.ascontiguousarray(e)).to(DEV) if len(e) else None, D)
    torch.cuda.synchronize()
    mask = int(out["best_mask"].cpu().numpy().view(np.uint64)[0])
    return dict(best_mask=mask, best_sum=int(out["best_sum"].item()), n_connected=int(out["n_connected"].item()),
                best_nodes=[q for q in out["nodes"].cpu().tolist()[:D] if q >= 0])


def test_subgraph_search_golden(sp):
    import json, os
    g = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "subgraph_case.json")))
    for c in g["cases"]:
        r = _run_subgraph(sp, g["count"], g["level"], g["edges"], c["D"])
        assert r["n_connected"] == len(c["sets"]), c
        assert (r["best_nodes"], r["best_sum"], r["best_mask"]) == (c["best_nodes"], c["best_sum"], c["best_mask"]), c


@pytest.mark.parametrize("seed", range(8))
def test_subgraph_search_parity(sp, seed):
    """Every output bit-exact against the oracle's enumeration: graphs below and above the 12 tabulated low
    nodes, every D that keeps the oracle within seconds, equal counts (the tie rule decides)."""
    n_levels = [2, 3, 4, 5, 6, 7, 8, 4][seed]
    count, level, edges, _ = synth.candidate_graph(n_levels, seed=100 + seed)
    if seed % 3 == 2:
        count = (count // 500 + 1).astype(np.int64)          # many equal sums
    if seed == 7:
        edges = np.concatenate([edges, [[-1, 2], [3, 99], [5, 5]]]).astype(np.int32)   # ignored rows, a self-loop
    N = len(count)
    import math
    for D in range(1, N + 2):
        if math.comb(N, min(D, N)) > 800000:
            continue
        ref = O().subgraph_search(count, level, edges, D)
        got = _run_subgraph(sp, count, level, edges, D)
        assert got == ref, (seed, N, D, got, ref)


def test_subgraph_search_closed_forms_at_size(sp):
    """Sizes the oracle cannot enumerate: results the structure fixes.  (1) all nodes root-level: every set is
    connected, the optimum is the D largest counts; (2) the D largest counts form a chain from a root, planted
    in a random candidate graph: that chain is the optimum; (3) a star: C(m, D-1) sets."""
    import math
    r = np.random.default_rng(4)
    N, D = 40, 8                                              # 7.7e7 sets
    count = r.integers(1, 10 ** 6, N).astype(np.int64)
    got = _run_subgraph(sp, count, np.ones(N, np.int32) + (np.arange(N) % 2), np.zeros((0, 2), np.int32), D)
    top = sorted(np.argsort(-count, kind="stable")[:D].tolist())
    assert got["n_connected"] == math.comb(N, D) and got["best_nodes"] == top and got["best_sum"] == int(count[top].sum())

    count, level, edges, _ = synth.candidate_graph(15, seed=8)       # 45 nodes
    N, D = len(count), 10                                            # 3.2e9 sets
    chain = [1] + list(r.permutation(np.arange(6, N))[:D - 1])       # node 1 is of level 1
    count = count.copy()
    count[chain] = 10 ** 6 + np.arange(D)
    edges = np.concatenate([edges, [[a, b] for a, b in zip(chain[:-1], chain[1:])]]).astype(np.int32)
    got = _run_subgraph(sp, count, level, edges, D)
    assert got["best_nodes"] == sorted(int(c) for c in chain) and got["best_sum"] == int(count[chain].sum())
    assert 0 < got["n_connected"] < math.comb(N, D)
    # relabelling the nodes changes neither the optimum value nor the number of connected sets
    perm = r.permutation(N)
    inv = np.argsort(perm)
    got_p = _run_subgraph(sp, count[perm], level[perm], inv[edges], D)
    assert got_p["best_sum"] == got["best_sum"] and got_p["n_connected"] == got["n_connected"]
    assert sorted(int(perm[q]) for q in got_p["best_nodes"]) == got["best_nodes"]

    m, D = 50, 6                                              # star: root 0 and 50 leaves of level 3
    count = np.concatenate([[1], r.integers(1, 1000, m)]).astype(np.int64)
    got = _run_subgraph(sp, count, np.array([2] + [3] * m, np.int32), np.array([[0, q] for q in range(1, m + 1)], np.int32), D)
    leaves = sorted((np.argsort(-count[1:], kind="stable")[:D - 1] + 1).tolist())
    assert got["n_connected"] == math.comb(m, D - 1) and got["best_sum"] == 1 + int(count[leaves].sum())


def test_subgraph_search_edge_cases(sp):
    one = _run_subgraph(sp, [7], [1], [], 1)
    assert one == dict(best_mask=1, best_sum=7, n_connected=1, best_nodes=[0])
    none = _run_subgraph(sp, [7], [3], [], 1)                 # a single node that is not root-level
    assert none == dict(best_mask=0, best_sum=0, n_connected=0, best_nodes=[])
    too_many = _run_subgraph(sp, [1, 2, 3], [1, 1, 1], [], 4)
    assert too_many == dict(best_mask=0, best_sum=0, n_connected=0, best_nodes=[])
    # 64 nodes, the highest bit in use; negative counts are sums like any other
    count = -np.arange(1, 65, dtype=np.int64)
    ref = O().subgraph_search(count, np.ones(64, np.int32), np.zeros((0, 2), int), 2)
    got = _run_subgraph(sp, count, np.ones(64, np.int32), [], 2)
    assert got == ref and got["best_nodes"] == [0, 1]
    level = np.array([3] * 63 + [1], np.int32)                # only node 63 is a root, everyone its child
    edges = np.array([[63, q] for q in range(63)], np.int32)
    got = _run_subgraph(sp, np.arange(64, dtype=np.int64), level, edges, 3)
    assert got["best_nodes"] == [61, 62, 63] and got["n_connected"] == 63 * 62 // 2 and got["best_mask"] == 7 << 61


@pytest.mark.parametrize("scale", [1 << 29, 1 << 30, 1 << 41])
def test_subgraph_search_large_counts_take_the_64_bit_path(sp, scale):
    """Counts whose magnitudes add up to 2^30 or more are summed in 64 bits; below that in 32 bits: both against
    the oracle, with negative counts and sums beyond 2^44."""
    count, level, edges, _ = synth.candidate_graph(6, seed=300)
    r = np.random.default_rng(scale % 1000)
    big = (r.integers(-8, 9, len(count)) * (scale // 8)).astype(np.int64) + count
    for D in (1, 4, 9):
        ref = O().subgraph_search(big, level, edges, D)
        got = _run_subgraph(sp, big, level, edges, D)
        assert got == ref, (scale, D, got, ref)


# ------------------------------------------------------------------ the step inside a HIP graph

def test_step_replays_from_a_captured_graph(sp):
    """The whole step allocates nothing, never synchronises and records no memset: captured once into a HIP graph
    it replays with new inputs written into the same buffers, bit-identical to the eager call each time (eager
    work and synchronisations between the replays)."""
    cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", L=2, d=256, Hq=2, Hkv=2, hd=128, F=320, V=1280, P=100, B=32, G=6)
    plan, layers, prefix, hw, w_embed, states, edges = build_step(sp, cfg, "c1_literal", 7, 20.0)
    d_states = torch.from_numpy(states).to(DEV)
    d_edges = torch.from_numpy(np.ascontiguousarray(edges)).to(DEV)
    plan.run(d_states, d_edges)                      # first call outside the capture: one-time kernel attributes
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        plan.run(d_states, d_edges)
    keys = ("hidden", "argmax", "conf", "unmask", "target_states", "result", "accepted_state")
    for trial in range(4):
        new_states = synth.random_states(cfg.G, cfg.B, cfg.V, 0.3, 0.7, 50 + trial)
        d_states.copy_(torch.from_numpy(new_states).to(DEV))
        graph.replay()
        torch.cuda.synchronize()
        got = {k: plan.out[k].clone() for k in keys}
        plan.run(d_states, d_edges)                  # eager, same buffers
        torch.cuda.synchronize()
        for k in keys:
            assert torch.equal(got[k], plan.out[k]), (trial, k)
        assert not torch.equal(got["hidden"], torch.zeros_like(got["hidden"]))


# ------------------------------------------------------------------ full-sequence step: the true suffix recomputed in the call

def _seq_setup(sp, cfg, S, seed, scale, tau):
    layers = [synth.layer_weights(cfg, l, seed) for l in range(cfg.L)]
    prefix = [synth.prefix_kv(cfg, l, seed) for l in range(cfg.L)]
    hw, we = synth.head_weights(cfg, seed), synth.embed_weights(cfg, seed)
    states, edges = synth.draft_graph("c1", cfg.scaled(G=4), seed)
    suffix = np.full(S, cfg.mask_id, np.int32)
    suffix[::5] = 3                                           # a suffix that is not one repeated row
    caches = []
    for k, v in prefix:
        ck = torch.full((cfg.Hkv, cfg.P + cfg.B + S + 2, cfg.hd), 1e4, dtype=k.dtype)
        cv = torch.full_like(ck, 1e4)
        ck[:, :cfg.P], cv[:, :cfg.P] = k, v
        caches.append((ck.to(DEV), cv.to(DEV)))
    plan = sp.SeqStepPlan(sp.cfg_from_synth(cfg), [sp.layer_weights(dev_weights(w)) for w in layers],
                          [sp.prefix_kv(k, v, cfg.P) for k, v in caches], we.to(DEV), hw["final_norm"].to(DEV),
                          hw["w_vocab"].to(DEV), len(states), cfg.B, S, cfg.P, tau, logit_scale=scale, device=DEV)
    return plan, layers, prefix, hw, we, states, edges, suffix, caches


@pytest.mark.parametrize("key,S", [("c1", 16), ("c1", 0), ("bf16_generic", 7), ("bf16_mfma", 96), ("bf16_mfma", 1), ("bf16_mfma_long", 224)])
def test_step_full_sequence(sp, key, S):
    """Hidden states of blocks and suffix, decisions and the walk against the oracle; fp32 end to end, bf16 stage-wise.
    The cache rows behind the prefix are filled with 1e4 before the call: a read of a stale row would show."""
    if key == "c1":
        cfg = synth.CONFIGS["c1"]
    elif key == "bf16_generic":
        cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", P=37, B=5)
    elif key == "bf16_mfma":
        cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", L=2, d=256, Hq=4, Hkv=2, hd=128, F=320, V=640, P=70, B=32)
    else:
        cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", L=2, d=256, Hq=2, Hkv=2, hd=128, F=320, V=640, P=1900, B=32)
    scale, tau = 8.0, 0.5
    plan, layers, prefix, hw, we, states, edges, suffix, caches = _seq_setup(sp, cfg, S, 9, scale, tau)
    out = plan.run(torch.from_numpy(states).to(DEV), torch.from_numpy(suffix).to(DEV),
                   torch.from_numpy(np.ascontiguousarray(edges)).to(DEV))
    torch.cuda.synchronize()
    G = len(states)
    ref = O().verify_step_fullseq([np_weights(w) for w in layers], [(to_np(k), to_np(v)) for k, v in prefix], to_np(we),
                                  to_np(hw["final_norm"]), to_np(hw["w_vocab"]), states, suffix, edges, n_q_heads=cfg.Hq,
                                  n_kv_heads=cfg.Hkv, head_dim=cfg.hd, pos0=cfg.P, mask_id=cfg.mask_id, threshold=tau,
                                  rms_eps=cfg.rms_eps, rope_base=cfg.rope_base, logit_scale=scale)
    hid = to_np(out["hidden"].cpu())
    bound = 1e-4 if cfg.dtype == "f32" else (2e-2 if cfg.L == 1 else 4e-2)
    e_b, _ = rel_err(hid[:G * cfg.B].reshape(G, cfg.B, cfg.d), ref["hidden"])
    assert e_b < bound, e_b
    if S:
        e_s, _ = rel_err(hid[G * cfg.B:], ref["hidden_suffix"])
        assert e_s < bound, e_s
    masked = states == cfg.mask_id
    if cfg.dtype == "f32":
        safe = masked & (ref["margin"] > 1e-3 * scale)
        np.testing.assert_array_equal(out["argmax"].cpu().numpy()[safe], ref["argmax"][safe])
    tgt = out["target_states"].cpu().numpy()
    walk = O().graph_accept(edges, states, tgt, 0)
    assert tuple(out["result"].cpu().tolist()[:3]) == walk[:3]
    # the cache: prefix untouched, the slot of the block and the suffix rows rewritten, nothing beyond
    for (ck, cv), (k, v) in zip(caches, prefix):
        assert torch.equal(ck[:, :cfg.P].cpu(), k) and torch.equal(cv[:, :cfg.P].cpu(), v)
        assert (ck[:, cfg.P + cfg.B + S:].cpu() == 1e4).all()
        if S:
            assert (ck[:, cfg.P:cfg.P + cfg.B + S].float().abs().cpu() < 1e3).all()


def test_step_full_sequence_at_the_suffix_limit(sp):
    """S = SPIFFY_MAX_SUFFIX = 4096 recomputed suffix rows (three key splits for the suffix queries, 128 row tiles
    of suffix rows through every projection), one narrow layer so the oracle finishes in seconds."""
    cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", L=1, d=256, Hq=2, Hkv=1, hd=128, F=256, V=640, P=70, B=32)
    S, scale, tau = 4096, 8.0, 0.5
    plan, layers, prefix, hw, we, states, edges, suffix, caches = _seq_setup(sp, cfg, S, 9, scale, tau)
    out = plan.run(torch.from_numpy(states).to(DEV), torch.from_numpy(suffix).to(DEV),
                   torch.from_numpy(np.ascontiguousarray(edges)).to(DEV))
    torch.cuda.synchronize()
    G = len(states)
    ref = O().verify_step_fullseq([np_weights(w) for w in layers], [(to_np(k), to_np(v)) for k, v in prefix], to_np(we),
                                  to_np(hw["final_norm"]), to_np(hw["w_vocab"]), states, suffix, edges, n_q_heads=cfg.Hq,
                                  n_kv_heads=cfg.Hkv, head_dim=cfg.hd, pos0=cfg.P, mask_id=cfg.mask_id, threshold=tau,
                                  rms_eps=cfg.rms_eps, rope_base=cfg.rope_base, logit_scale=scale)
    hid = to_np(out["hidden"].cpu())
    e_b, _ = rel_err(hid[:G * cfg.B].reshape(G, cfg.B, cfg.d), ref["hidden"])
    e_s, _ = rel_err(hid[G * cfg.B:], ref["hidden_suffix"])
    assert e_b < 2e-2 and e_s < 2e-2, (e_b, e_s)
    for ck, cv in caches:
        assert (ck[:, cfg.P + cfg.B + S:].cpu() == 1e4).all() and (cv[:, cfg.P + cfg.B + S:].cpu() == 1e4).all()


def test_step_full_sequence_without_suffix_is_the_step(sp):
    cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", L=2, d=256, Hq=4, Hkv=2, hd=128, F=320, V=640, P=70, B=32)
    plan, layers, prefix, hw, we, states, edges, suffix, caches = _seq_setup(sp, cfg, 0, 9, 8.0, 0.5)
    d_states, d_edges = torch.from_numpy(states).to(DEV), torch.from_numpy(np.ascontiguousarray(edges)).to(DEV)
    a = {k: v.clone() for k, v in plan.run(d_states, torch.zeros(0, dtype=torch.int32, device=DEV), d_edges).items()}
    base = sp.StepPlan(plan.cfg, plan._keep[0], [sp.prefix_kv(k.to(DEV), v.to(DEV)) for k, v in prefix], we.to(DEV),
                       hw["final_norm"].to(DEV), hw["w_vocab"].to(DEV), len(states), cfg.B, cfg.P, 0.5, logit_scale=8.0,
                       device=DEV)
    b = base.run(d_states, d_edges)
    torch.cuda.synchronize()
    for k in ("hidden", "argmax", "conf", "unmask", "target_states", "result", "accepted_state"):
        assert torch.equal(a[k].reshape(b[k].shape), b[k]), k


@pytest.mark.parametrize("reuse", [False, True])
def test_decode_full_sequence_matches_the_oracle_loop(sp, reuse):
    """Configuration 1 (fp32), three blocks, the first with 2B MASK tokens behind it that every pass recomputes:
    device loop = oracle loop (tokens, forward passes, depths), and the same tokens as vanilla decoding.  A
    finished block's keys / values come from one more pass on its final tokens, with the suffix still behind it.
    reuse: that pass also saw the next block's positions as MASK rows of the same sequence, so the next block's
    first step runs the head on its hidden states and spends no forward pass (same tokens and depths, one pass
    less per later block)."""
    from paper_2509_18085_amd import decode
    cfg = synth.CONFIGS["c1"]
    scale, tau, d_star, seed, S0, n_blocks = 12.0, 0.5, 3, synth.DEFAULT_SEED, 2 * cfg.B, 3
    formulas = [[(i, 1) for i in range(1, n + 1)] for n in range(1, 5)] + [[(1, 2)], [(1, 1), (2, 2)]]
    layers = [synth.layer_weights(cfg, l, seed) for l in range(cfg.L)]
    prefix = [synth.prefix_kv(cfg, l, seed) for l in range(cfg.L)]
    hw, we = synth.head_weights(cfg, seed), synth.embed_weights(cfg, seed)

    def run(graph, d):
        ck, cv = [], []
        for k, v in prefix:
            kk = torch.full((cfg.Hkv, cfg.P + n_blocks * cfg.B, cfg.hd), 1e4, dtype=k.dtype)
            vv = torch.full_like(kk, 1e4)
            kk[:, :cfg.P], vv[:, :cfg.P] = k, v
            ck.append(kk.to(DEV))
            cv.append(vv.to(DEV))
        dec = decode.BlockDecoder(sp.cfg_from_synth(cfg), [dev_weights(w) for w in layers], ck, cv, cfg.P, we.to(DEV),
                                  hw["final_norm"].to(DEV), hw["w_vocab"].to(DEV), cfg.B, tau, logit_scale=scale,
                                  graph=graph, d_star=d, device=DEV, seq_S0=S0, reuse_commit_pass=reuse)
        g = dec.generate(n_blocks)
        assert dec.saved_passes == (n_blocks - 1 if reuse else 0)
        return g, ck, cv

    graph = decode.DraftGraph(formulas, device=DEV)
    (got, ck, cv), (van, _, _) = run(graph, d_star), run(None, 0)
    np.testing.assert_array_equal(got["tokens"], van["tokens"])
    assert sum(got["nfe"]) < sum(van["nfe"])

    lw = [np_weights(w) for w in layers]
    w_np = dict(w_embed=to_np(we), final_norm=to_np(hw["final_norm"]), w_vocab=to_np(hw["w_vocab"]))
    pre = [(to_np(k), to_np(v)) for k, v in prefix]

    def drafter(state, info):
        if not info:
            return np.zeros((0, state.size), np.int32), np.zeros((0, 2), np.int32)
        t, p = O().head_topk(info["hidden"][info["node"]], w_np["final_norm"], w_np["w_vocab"], graph.K,
                             rms_eps=cfg.rms_eps, logit_scale=scale)
        out = O().draft_and_prune(state, cfg.mask_id, t, p, formulas, graph.edges_np, d_star)
        return out["states"][1:], out["edges"]

    tokens, nfes, depths = [], [], []
    P, S = cfg.P, S0
    for _ in range(n_blocks):
        kw = dict(n_q_heads=cfg.Hq, n_kv_heads=cfg.Hkv, head_dim=cfg.hd, pos0=P, mask_id=cfg.mask_id, threshold=tau,
                  rms_eps=cfg.rms_eps, rope_base=cfg.rope_base, logit_scale=scale, force_one=True)
        suffix = np.full(S, cfg.mask_id, np.int32)
        model = dict(layers=lw, prefix=pre, kw=kw, suffix_tokens=suffix, **w_np)
        final, _, nfe, dps, _ = O().decode_block(model, np.full(cfg.B, cfg.mask_id, np.int32), drafter=drafter)
        tokens.append(final)
        nfes.append(nfe)
        depths.append(dps)
        hb, hs = O().embed(w_np["w_embed"], final[None, :]), O().embed(w_np["w_embed"], suffix)
        new_pre = []
        for l in range(cfg.L):
            hb, hs, k0, v0 = O().verify_layer_fullseq(lw[l], pre[l][0], pre[l][1], hb, hs, return_kv=True,
                                                      **oracle_kw(cfg, P))
            new_pre.append((np.concatenate([pre[l][0], k0], axis=1), np.concatenate([pre[l][1], v0], axis=1)))
        pre = new_pre
        P, S = P + cfg.B, max(0, S - cfg.B)
    np.testing.assert_array_equal(got["tokens"], np.concatenate(tokens))
    assert got["nfe"] == ([nfes[0]] + [n - 1 for n in nfes[1:]] if reuse else nfes) and got["depths"] == depths
    # the caches now hold the oracle's prefix: context and the three committed blocks
    for l in range(cfg.L):
        for got_c, want in ((ck[l], pre[l][0]), (cv[l], pre[l][1])):
            e_max, _ = rel_err(to_np(got_c.cpu()), want)
            assert e_max < 1e-4, (l, e_max)


# ------------------------------------------------------------------ commit of the finished block folded into the next block's first pass

@pytest.mark.parametrize("key", ["c1", "bf16_generic", "bf16_mfma", "bf16_mfma_long", "bf16_mfma_dual", "bf16_mfma_b4"])
def test_step_commit_is_commit_block_then_step(sp, key):
    """spiffy_verify_step_commit = spiffy_commit_block of the finished block, then spiffy_verify_step of the next
    block's states with the prefix grown by B: same cache rows and same outputs, bit for bit (a row's arithmetic
    does not depend on what is verified with it); and the oracle's two steps within the usual bounds."""
    S = 0
    if key == "c1":
        cfg = synth.CONFIGS["c1"]
    elif key == "bf16_generic":
        cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", P=37, B=5)
    elif key == "bf16_mfma_long":
        cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", L=2, d=256, Hq=2, Hkv=2, hd=128, F=320, V=640, P=2040, B=32)
    elif key == "bf16_mfma_b4":          # small blocks: the finished block and the four states share one 32-row group
        cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", L=2, d=256, Hq=4, Hkv=2, hd=128, F=320, V=640, P=70, B=4)
    else:
        cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", L=2, d=256, Hq=4, Hkv=2, hd=128, F=320, V=640, P=70, B=32)
        S = 3 * cfg.B if key == "bf16_mfma_dual" else 0
    seed, scale, tau = 9, 8.0, 0.5
    layers = [synth.layer_weights(cfg, l, seed) for l in range(cfg.L)]
    caches = [_full_cache(cfg, S + cfg.B, seed, layer=l) for l in range(cfg.L)]     # room for both blocks (and the suffix)
    hw, we = synth.head_weights(cfg, seed), synth.embed_weights(cfg, seed)
    states, edges = synth.draft_graph("c1", cfg.scaled(G=4), seed)
    d_states = torch.from_numpy(states).to(DEV)
    d_edges = torch.from_numpy(np.ascontiguousarray(edges)).to(DEV)
    prev = torch.from_numpy(np.random.default_rng(4).integers(0, cfg.V - 1, size=cfg.B).astype(np.int32)).to(DEV)

    def make():
        dk = [c[0].clone().to(DEV) for c in caches]
        dv = [c[1].clone().to(DEV) for c in caches]
        plan = sp.StepPlan(sp.cfg_from_synth(cfg), [sp.layer_weights(dev_weights(w)) for w in layers],
                           [sp.prefix_kv(k, v, cfg.P, S) for k, v in zip(dk, dv)], we.to(DEV), hw["final_norm"].to(DEV),
                           hw["w_vocab"].to(DEV), len(states), cfg.B, cfg.P, tau, logit_scale=scale, device=DEV)
        return plan, dk, dv

    plan_a, ka, va = make()
    plan_a.workspace = sp.alloc_workspace(plan_a.cfg, len(states), cfg.B, cfg.P + cfg.B + S, DEV)
    plan_a.commit_block(prev)
    plan_a.set_prefix_len(cfg.P + cfg.B, S=max(0, S - cfg.B))
    a = {k: v.clone() for k, v in plan_a.run(d_states, d_edges).items()}
    plan_b, kb, vb = make()
    b = plan_b.run_commit(prev, d_states, d_edges)
    torch.cuda.synchronize()
    for k in ("hidden", "argmax", "conf", "unmask", "margin", "target_states", "result", "accepted_state"):
        assert torch.equal(a[k], b[k]), k
    for l in range(cfg.L):
        assert torch.equal(ka[l], kb[l]) and torch.equal(va[l], vb[l]), l
    # the oracle: forward of the finished block (its keys / values join the prefix), then the step
    lw = [np_weights(w) for w in layers]
    pre = [(to_np(c[2]), to_np(c[3])) for c in caches]
    suf = [(to_np(c[4])[:, :S], to_np(c[5])[:, :S]) for c in caches]
    h = O().embed(to_np(we), prev.cpu().numpy()[None, :])
    new_pre = []
    for l in range(cfg.L):
        h, ks, vs = O().verify_layer(lw[l], pre[l][0], pre[l][1], h, suffix_k=suf[l][0] if S else None,
                                     suffix_v=suf[l][1] if S else None, return_kv=True, **oracle_kw(cfg))
        new_pre.append((np.concatenate([pre[l][0], ks[0]], axis=1), np.concatenate([pre[l][1], vs[0]], axis=1)))
    e_prev, _ = rel_err(to_np(b["hidden_prev"].cpu()), h[0])
    bound = 1e-4 if cfg.dtype == "f32" else (2e-2 if cfg.L == 1 else 4e-2)
    assert e_prev < bound, e_prev
    ref = O().verify_step(lw, new_pre, to_np(we), to_np(hw["final_norm"]), to_np(hw["w_vocab"]), states, edges,
                          n_q_heads=cfg.Hq, n_kv_heads=cfg.Hkv, head_dim=cfg.hd, pos0=cfg.P + cfg.B, mask_id=cfg.mask_id,
                          threshold=tau, rms_eps=cfg.rms_eps, rope_base=cfg.rope_base, logit_scale=scale,
                          suffix=[(k[:, cfg.B:], v[:, cfg.B:]) for k, v in suf] if S else None)
    e_max, _ = rel_err(to_np(b["hidden"].cpu()), ref["hidden"])
    assert e_max < bound, e_max
    if cfg.dtype == "f32":
        safe = (states == cfg.mask_id) & (ref["margin"] > 1e-3 * scale)
        np.testing.assert_array_equal(b["argmax"].cpu().numpy()[safe], ref["argmax"][safe])
        assert tuple(b["result"].cpu().tolist()[:3]) == (ref["node"], ref["depth"], ref["n_steps"])


def test_decode_full_sequence_is_lossless_on_the_mfma_path(sp):
    """bf16 MFMA kernels, full-sequence model (3B MASK tokens recomputed behind the first block), four blocks:
    speculative decoding reproduces vanilla decoding token for token, with and without the commit pass standing
    in for the next block's first pass; that shortcut changes no token here and saves one pass per later block."""
    from paper_2509_18085_amd import decode
    cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", L=2, d=256, Hq=2, Hkv=2, hd=128, F=320, V=1280, P=100, B=32, G=1)
    formulas = [[(i, 1) for i in range(1, n + 1)] for n in (1, 2, 3, 4, 6, 8, 12, 16)] + [[(1, 2)], [(1, 1), (2, 2)]]
    seed, n_blocks = 11, 4
    layers = [synth.layer_weights(cfg, l, seed) for l in range(cfg.L)]
    prefix = [synth.prefix_kv(cfg, l, seed) for l in range(cfg.L)]
    hw, we = synth.head_weights(cfg, seed), synth.embed_weights(cfg, seed)

    def run(graph, d, reuse):
        ck, cv = [], []
        for k, v in prefix:
            kk = torch.zeros((cfg.Hkv, cfg.P + n_blocks * cfg.B, cfg.hd), dtype=k.dtype)
            vv = torch.zeros_like(kk)
            kk[:, :cfg.P], vv[:, :cfg.P] = k, v
            ck.append(kk.to(DEV))
            cv.append(vv.to(DEV))
        dec = decode.BlockDecoder(sp.cfg_from_synth(cfg), [dev_weights(w) for w in layers], ck, cv, cfg.P, we.to(DEV),
                                  hw["final_norm"].to(DEV), hw["w_vocab"].to(DEV), cfg.B, 0.7, logit_scale=16.0,
                                  graph=graph, d_star=d, device=DEV, seq_S0=(n_blocks - 1) * cfg.B, reuse_commit_pass=reuse)
        return dec.generate(n_blocks)

    graph = decode.DraftGraph(formulas, device=DEV)
    res = {(spec, reuse): run(graph if spec else None, 5 if spec else 0, reuse) for spec in (0, 1) for reuse in (0, 1)}
    for reuse in (0, 1):
        np.testing.assert_array_equal(res[(1, reuse)]["tokens"], res[(0, reuse)]["tokens"])
        assert sum(res[(1, reuse)]["nfe"]) < sum(res[(0, reuse)]["nfe"])
    assert not (res[(1, 1)]["tokens"] == cfg.mask_id).any()
    np.testing.assert_array_equal(res[(0, 1)]["tokens"], res[(0, 0)]["tokens"])
    assert sum(res[(0, 1)]["nfe"]) == sum(res[(0, 0)]["nfe"]) - (n_blocks - 1)


def test_machine_probes_run(sp):
    """The roofline probes launch, finish, and report the work they did (their rates are bench.py's business)."""
    sink = torch.full((1024,), -1.0, dtype=torch.float32, device=DEV)
    from paper_2509_18085_amd import probe
    flop = probe.probe_mfma(100, False, sink)
    torch.cuda.synchronize()
    assert flop == 1024 * 4 * 100 * 4 * 2.0 * 32 * 32 * 16
    assert (sink == 0).all()                                   # zero operands: every accumulator stays zero
    probe.probe_mfma(100, True, sink)
    torch.cuda.synchronize()
    assert torch.isfinite(sink).all() and (sink != 0).any()
    src = torch.ones(3 * (1 << 20) + 48, dtype=torch.uint8, device=DEV)
    assert probe.probe_hbm_read(src, torch.zeros(1, dtype=torch.int32, device=DEV)) == src.numel()
    torch.cuda.synchronize()


def test_attention_with_scores_that_jump(sp):
    """Keys late in the prefix that dwarf everything before them (rows scaled 25x, spread over tiles and over both
    key halves of a tile), a prefix that starts with such a key, and one in the very last, ragged tile: the
    online-softmax reference has to move (by far more than the 2^8 it tolerates without moving) at arbitrary
    points of the stream, and small probabilities before the jump must vanish as in the oracle."""
    cfg = synth.CONFIGS["c1"].scaled(dtype="bf16", L=1, d=256, Hq=2, Hkv=1, hd=128, F=256, V=640, P=2300, B=32, G=5)
    w = synth.layer_weights(cfg, 0, 21)
    pk, pv = synth.prefix_kv(cfg, 0, 21)
    x = synth.hidden_states(cfg, 21)
    cases = [([0], 25.0), ([300, 345, 1000, 1500, 2047, 2048, 2299], 25.0), ([64 * 7 + 31, 64 * 7 + 32], 25.0),
             (list(range(100, 2300, 37)), 4.0)]      # the last: maxima that creep up, below and beyond 2^8 in turn
    for big, factor in cases:
        k = pk.clone()
        for i, r in enumerate(big):
            k[:, r] = (k[:, r].float() * (factor if factor > 5 else 1.0 + (factor - 1.0) * (i + 1) / len(big))).to(k.dtype)
        got = run_layer(sp, cfg, w, k, pv, x)
        ref = O().verify_layer(np_weights(w), to_np(k), to_np(pv), to_np(x), **oracle_kw(cfg))
        e_max, e_norm = rel_err(to_np(got), ref)
        assert e_max < tol(cfg), (big, e_max, e_norm)

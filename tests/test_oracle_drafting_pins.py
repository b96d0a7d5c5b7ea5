"""Pins for the oracle's drafting and pruning functions (Sec. 4.4.2 drafting source, Sec. 4.4.4
pruning).  None of them re-types the oracle's formula: a hand-worked example stored as text, an
independent implementation on exact fractions with counting ranks, the parent-child conditions of
Eqs. (4)-(6), algebraic properties of the geometric mean, and the link to Next(X, p) of Alg. 1 /
Sec. 3.1 (a formula made of the positions the threshold rule unmasks is the next state, and the
walk accepts it).
"""
import json
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import spiffy_oracle as O
from helpers import tiny_cfg, tiny_model

HERE = os.path.dirname(os.path.abspath(__file__))


def _golden():
    with open(os.path.join(HERE, "golden", "draft_prune_case.json")) as f:
        return json.load(f)


def test_worked_example():
    """tests/golden/draft_prune_case.json: ranks, draft blocks, scores and the kept sub-graph worked
    out by hand from Sec. 4.4.2 / 4.4.4 (derivation inside the file)."""
    g = _golden()
    r = O.draft_and_prune(np.array(g["state"]), g["mask_id"], np.array(g["topk_tokens"]),
                          np.array(g["topk_probs"]), [[tuple(p) for p in f] for f in g["formulas"]],
                          np.array(g["edges"]), g["d_star"])
    e = g["expected"]
    assert r["order"] == e["position_order"]
    np.testing.assert_array_equal(r["drafts"], np.array(e["drafts"]))
    assert r["buildable"].tolist() == e["buildable"]
    for name in ("local", "child", "score"):
        for got, want in zip(r[name], e[name]):
            if want is None:
                assert math.isnan(got), name
            else:
                assert abs(got - want) < 5e-7, (name, got, want)
    assert r["kept"].tolist() == e["kept"]
    assert r["edges"].tolist() == e["edges"]
    np.testing.assert_array_equal(r["states"], np.array(e["drafts"])[e["kept"]])


# ---------------------------------------------------------------- independent implementation

def _independent(state, mask_id, tok, prob, formulas, edges, d_star):
    """Same quantities from the definitions, by other means: rank by counting (a position's rank
    is 1 + the number of masked positions that beat it), scores compared through exact powers
    (local^k = product of probabilities; score^2 = local * child; child^n = product of locals),
    selection by repeatedly taking the maximum."""
    B = len(state)
    masked = [b for b in range(B) if state[b] == mask_id]
    rank = {}
    for b in masked:
        beat = sum(1 for c in masked if prob[c][0] > prob[b][0] or (prob[c][0] == prob[b][0] and c < b))
        rank[beat + 1] = b
    D = len(formulas)
    drafts, ok, prods = [list(state)], [True], [None]
    for f in formulas:
        d = list(state)
        good = len(f) > 0 and len({i for i, _ in f}) == len(f)
        pr = Fraction(1)
        for i, j in f:
            if i not in rank or not (1 <= j <= len(tok[0])):
                good = False
                break
            d[rank[i]] = tok[rank[i]][j - 1]
            pr *= Fraction(prob[rank[i]][j - 1])
        drafts.append(d if good else list(state))
        ok.append(good)
        prods.append((pr, len(f)) if good else None)
    local = [None] + [float(prods[m][0]) ** (1.0 / prods[m][1]) if ok[m] else None for m in range(1, D + 1)]
    score = [None] * (D + 1)
    for m in range(1, D + 1):
        if not ok[m]:
            continue
        kids = sorted({c for a, c in edges if a == m and 1 <= c <= D and ok[c]})
        if kids:
            child = math.prod(local[c] for c in kids) ** (1.0 / len(kids))
            score[m] = math.sqrt(local[m] * child)
        else:
            score[m] = local[m]
    pool = [m for m in range(1, D + 1) if ok[m]]
    kept = []
    while pool and len(kept) < d_star:
        best = max(pool, key=lambda m: (score[m], -m))
        kept.append(best)
        pool.remove(best)
    return drafts, ok, local, score, sorted(kept)


def _random_case(rng, B, K, V, D):
    mask_id = V
    state = [int(mask_id) if rng.random() < 0.6 else int(rng.integers(0, V)) for _ in range(B)]
    tok = [[int(t) for t in rng.choice(V, size=K, replace=False)] for _ in range(B)]
    # a coarse grid of probabilities: ties in confidence and in scores do occur
    prob = []
    for _ in range(B):
        p = sorted((float(rng.integers(1, 9)) / 16.0 for _ in range(K)), reverse=True)
        prob.append(p)
    n_masked = sum(1 for s in state if s == mask_id)
    formulas = []
    for _ in range(D):
        k = int(rng.integers(1, 4))
        hi = max(1, n_masked + 1)            # sometimes one rank too many: an unbuildable formula
        ranks = rng.choice(np.arange(1, hi + 1), size=min(k, hi), replace=False)
        formulas.append([(int(i), int(rng.integers(1, K + 2))) for i in ranks])   # sometimes j = K+1
    sets = [set()] + [set(f) for f in formulas]
    edges = [(a, c) for a in range(D + 1) for c in range(1, D + 1) if a != c and sets[a] < sets[c]]
    return state, mask_id, tok, prob, formulas, edges


@pytest.mark.parametrize("seed", range(12))
def test_against_independent_implementation(seed):
    rng = np.random.default_rng(100 + seed)
    B, K, V, D = int(rng.integers(3, 9)), int(rng.integers(1, 4)), 50, int(rng.integers(1, 9))
    state, mask_id, tok, prob, formulas, edges = _random_case(rng, B, K, V, D)
    d_star = int(rng.integers(0, D + 2))
    r = O.draft_and_prune(np.array(state), mask_id, np.array(tok), np.array(prob), formulas,
                          np.array(edges, np.int64).reshape(-1, 2), d_star)
    drafts, ok, local, score, kept = _independent(state, mask_id, tok, prob, formulas, edges, d_star)
    assert r["buildable"].tolist() == ok
    np.testing.assert_array_equal(r["drafts"], np.array(drafts))
    for m in range(1, D + 1):
        if ok[m]:
            assert abs(r["local"][m] - local[m]) < 1e-12 and abs(r["score"][m] - score[m]) < 1e-12
        else:
            assert math.isnan(r["score"][m])
    # equal scores are decided by node index on both sides; scores closer than rounding are not compared
    vals = sorted(score[m] for m in range(1, D + 1) if ok[m])
    if all(b - a == 0 or b - a > 1e-9 for a, b in zip(vals, vals[1:])):
        assert r["kept"].tolist() == [0] + kept
    assert r["kept"][0] == 0 and len(r["kept"]) == 1 + min(d_star, sum(ok[1:]))
    pos = {int(m): i for i, m in enumerate(r["kept"])}
    want_edges = [(pos[a], pos[c]) for a, c in edges if a in pos and c in pos]
    assert r["edges"].tolist() == [list(e) for e in want_edges]


# ---------------------------------------------------------------- Eqs. (4)-(6)

def test_formula_inclusion_gives_parent_child_blocks():
    """If formula A is a subset of formula B then block B only adds unmasked tokens to block A:
    unmasked(A) is a subset of unmasked(B), the tokens of A are untouched, and B has exactly
    |B \\ A| more unmasked positions (the conditions under which B can be a child of A)."""
    rng = np.random.default_rng(5)
    for _ in range(20):
        state, mask_id, tok, prob, formulas, edges = _random_case(rng, 8, 3, 40, 8)
        r = O.draft_and_prune(np.array(state), mask_id, np.array(tok), np.array(prob), formulas,
                              np.array(edges, np.int64).reshape(-1, 2), 8)
        sets = [set()] + [set(f) for f in formulas]
        for a, c in edges:
            if not (r["buildable"][a] and r["buildable"][c]):
                continue
            A, Bk = r["drafts"][a], r["drafts"][c]
            ua, ub = A != mask_id, Bk != mask_id
            assert (ub | ~ua).all()                      # unmasked(A) subset of unmasked(B)
            assert (A[ua] == Bk[ua]).all()
            assert int(ub.sum()) - int(ua.sum()) == len(sets[c] - sets[a])
        for m in range(1, len(formulas) + 1):            # every block extends the current one
            if r["buildable"][m]:
                keep = np.array(state) != mask_id
                assert (r["drafts"][m][keep] == np.array(state)[keep]).all()
                assert int((r["drafts"][m] != mask_id).sum()) == int(keep.sum()) + len(formulas[m - 1])


# ---------------------------------------------------------------- geometric mean

def test_geometric_mean_properties():
    rng = np.random.default_rng(3)
    for _ in range(50):
        k = int(rng.integers(1, 7))
        v = rng.uniform(0.01, 1.0, size=k)
        g = O.geometric_mean(v)
        assert min(v) - 1e-15 <= g <= max(v) + 1e-15
        assert abs(g ** k - float(np.prod(v))) < 1e-12                      # g^k = product
        assert abs(O.geometric_mean(0.5 * v) - 0.5 * g) < 1e-12              # homogeneous of degree 1
        assert abs(O.geometric_mean(np.concatenate([v, v])) - g) < 1e-12     # repeating the sample
        assert g <= float(np.mean(v)) + 1e-12                                # AM-GM
    assert O.geometric_mean([0.37]) == pytest.approx(0.37, abs=1e-15)
    assert O.geometric_mean([0.25, 0.25, 0.25]) == pytest.approx(0.25, abs=1e-15)
    assert O.geometric_mean([0.5, 0.0]) == 0.0
    assert O.geometric_mean([4.0, 9.0]) == pytest.approx(6.0, abs=1e-12)


def test_prune_budget_edges_and_nesting():
    rng = np.random.default_rng(9)
    state, mask_id, tok, prob, formulas, edges = _random_case(rng, 8, 2, 30, 7)
    E = np.array(edges, np.int64).reshape(-1, 2)
    args = (np.array(state), mask_id, np.array(tok), np.array(prob), formulas, E)
    full = O.draft_and_prune(*args, len(formulas))
    n_ok = int(full["buildable"][1:].sum())
    assert full["kept"].tolist() == [0] + [m for m in range(1, len(formulas) + 1) if full["buildable"][m]]
    assert O.draft_and_prune(*args, 0)["kept"].tolist() == [0]
    prev = {0}
    for d in range(1, n_ok + 1):                   # budgets are nested: D*+1 keeps a superset of D*
        cur = set(O.draft_and_prune(*args, d)["kept"].tolist())
        assert prev <= cur and len(cur) == d + 1
        prev = cur


# ---------------------------------------------------------------- drafting source

def test_head_topk_first_column_is_the_head_and_rows_are_sorted():
    rng = np.random.default_rng(2)
    B, d, V, K = 5, 16, 37, 4
    hidden = rng.standard_normal((1, B, d))
    fn = rng.uniform(0.5, 1.5, size=d)
    wv = rng.standard_normal((V, d))
    tokens = np.full((1, B), V, np.int32)        # everything masked
    amax, conf, _, _, _ = O.decode_head(hidden, fn, wv, tokens, V, 0.9, rms_eps=1e-5, logit_scale=3.0)
    tok, pr = O.head_topk(hidden[0], fn, wv, K, rms_eps=1e-5, logit_scale=3.0)
    np.testing.assert_array_equal(tok[:, 0], amax[0])
    np.testing.assert_allclose(pr[:, 0], conf[0], rtol=1e-6)
    assert (np.diff(pr, axis=1) <= 0).all()
    allt, allp = O.head_topk(hidden[0], fn, wv, V, rms_eps=1e-5, logit_scale=3.0)
    np.testing.assert_allclose(allp.sum(axis=1), 1.0, atol=1e-12)
    assert all(sorted(row.tolist()) == list(range(V)) for row in allt)
    # equal logits: the lower token id ranks first
    wv2 = wv.copy()
    wv2[9] = wv2[4]
    t2, _ = O.head_topk(hidden[0], fn, wv2, V, rms_eps=1e-5)
    for row in t2:
        row = row.tolist()
        assert row.index(4) + 1 == row.index(9)


def test_threshold_formula_is_the_next_state_and_is_accepted():
    """Link to Next(X, p) (Alg. 1 steps 1-4 with the threshold rule, Sec. 3.1): the positions the rule
    unmasks are exactly the s most confident masked positions, so the formula {(1,1),...,(s,1)} built
    from the current distribution is the next state; drafted from the accepted node's distribution
    it is accepted by the walk whenever the model's next step agrees (and decoding stays lossless)."""
    cfg = tiny_cfg(d=64, Hq=2, Hkv=2, hd=32, F=96, V=64, P=6, B=6, L=2)
    model = tiny_model(cfg, seed=31, weight_std_scale=6.0, logit_scale=20.0, threshold=0.5, force_one=True)
    kw = model["kw"]
    block0 = np.full(cfg.B, cfg.mask_id, np.int32)
    block0[2] = 7
    r0 = O.verify_step(model["layers"], model["prefix"], model["w_embed"], model["final_norm"],
                       model["w_vocab"], block0[None, :], np.zeros((0, 2), np.int32), **kw)
    s = int(r0["unmask"][0].sum())
    assert s >= 1
    tok, pr = O.head_topk(r0["hidden"][0], model["final_norm"], model["w_vocab"], 2,
                          rms_eps=kw["rms_eps"], logit_scale=kw["logit_scale"])
    formula = [(i, 1) for i in range(1, s + 1)]
    dp = O.draft_and_prune(block0, cfg.mask_id, tok, pr, [formula], np.array([[0, 1]]), 1)
    np.testing.assert_array_equal(dp["drafts"][1], r0["target_states"][0])

    # as a drafter inside the decode loop: formulas "the s best" for s = 1..B, chained, pruned to 3
    formulas = [[(i, 1) for i in range(1, n + 1)] for n in range(1, cfg.B + 1)]
    edges = np.array([[a, c] for a in range(0, cfg.B + 1) for c in range(a + 1, cfg.B + 1)])

    def drafter(state, info):
        if not info:
            return np.zeros((0, state.size), np.int32), np.zeros((0, 2), np.int32)
        t, p = O.head_topk(info["hidden"][info["node"]], model["final_norm"], model["w_vocab"], 1,
                           rms_eps=kw["rms_eps"], logit_scale=kw["logit_scale"])
        out = O.draft_and_prune(state, cfg.mask_id, t, p, formulas, edges, 3)
        return out["states"][1:], out["edges"]

    final_v, traj_v, nfe_v, _, _ = O.decode_block(model, block0)
    final_s, traj_s, nfe_s, depths, saved = O.decode_block(model, block0, drafter=drafter)
    np.testing.assert_array_equal(final_s, final_v)
    assert nfe_v - nfe_s == sum(saved)


def test_equal_scores_and_repeated_rank():
    """Readings pinned by construction: equal scores keep the lower node index; a formula naming one
    position rank twice (two tokens for one position) cannot be built."""
    state = np.array([9, 9, 9, 9])
    tok = np.array([[1, 2], [3, 4], [5, 6], [7, 8]])
    prob = np.array([[0.8, 0.1], [0.6, 0.2], [0.6, 0.3], [0.4, 0.3]])
    # ranks: pos0 (0.8), pos1 and pos2 tie at 0.6 -> pos1 then pos2, pos3 (0.4)
    formulas = [[(2, 1)], [(3, 1)], [(1, 1), (1, 2)], [(4, 1), (1, 1)]]
    r = O.draft_and_prune(state, 9, tok, prob, formulas, np.zeros((0, 2), np.int64), 1)
    assert r["buildable"].tolist() == [True, True, True, False, True]
    assert r["score"][1] == r["score"][2] == pytest.approx(0.6)
    assert r["kept"].tolist() == [0, 1]                       # node 1 beats node 2 on index, both beat node 4
    assert r["drafts"][1].tolist() == [9, 3, 9, 9] and r["drafts"][2].tolist() == [9, 9, 5, 9]
    assert r["drafts"][3].tolist() == [9, 9, 9, 9]
    assert O.draft_and_prune(state, 9, tok, prob, formulas, np.zeros((0, 2), np.int64), 2)["kept"].tolist() == [0, 1, 2]

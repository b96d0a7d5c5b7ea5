"""The pins must notice mistakes.  Each case plants one plausible mistake in the oracle's source text (on the
CPU, in a copy of the module that only this test sees) and runs the pins named for it: at least one must fail.
The untouched source is run through the same harness first, so a failure is the mutation's and not the harness's.
"""
import os
import types

import pytest

import test_oracle_drafting_pins as drafting
import test_oracle_fullseq_pins as fullseq
import test_oracle_pins as pins
import test_oracle_subgraph_pins as subgraph
import test_oracle_suffix_pins as suffix

SRC_PATH = os.path.join(os.path.dirname(__file__), "..", "oracle", "spiffy_oracle.py")
SRC = open(SRC_PATH).read()


def build(src):
    mod = types.ModuleType("spiffy_oracle_under_test")
    exec(compile(src, SRC_PATH, "exec"), mod.__dict__)
    return mod


def run(mod, checks, monkeypatch):
    """Run the pins against `mod`; returns the names of those that failed."""
    failed = []
    for m in (pins, drafting, subgraph, suffix, fullseq):
        monkeypatch.setattr(m, "O", mod)
    for fn, kwargs in checks:
        try:
            fn(**kwargs)
        except Exception:                                    # an assertion, or a shape error the mistake causes
            failed.append(fn.__name__)
    return failed


P = lambda fn, **kw: (fn, kw)

CASES = [
    ("rmsnorm: sum instead of mean", "ms = np.mean(x * x, axis=-1, keepdims=True)", "ms = np.sum(x * x, axis=-1, keepdims=True)",
     [P(pins.test_rmsnorm_closed_form)]),
    ("rmsnorm: eps dropped", "return x / np.sqrt(ms + eps) * np.asarray(gain, F64)", "return x / np.sqrt(ms) * np.asarray(gain, F64)",
     [P(pins.test_rmsnorm_closed_form)]),
    ("rope: rotation the other way", "[x1 * c - x2 * s, x2 * c + x1 * s]", "[x1 * c + x2 * s, x2 * c - x1 * s]",
     [P(pins.test_rope_known_rotation_and_identity)]),
    ("rope: wrong frequency exponent", "inv_freq = base ** (-2.0 * i / hd)", "inv_freq = base ** (-1.0 * i / hd)",
     [P(pins.test_rope_known_rotation_and_identity)]),
    ("silu: sign of the exponent", "return z / (1.0 + np.exp(-z))", "return z / (1.0 + np.exp(z))", [P(pins.test_silu_values)]),
    ("softmax: not normalised", "return e / np.sum(e, axis=-1, keepdims=True)", "return e / np.max(e, axis=-1, keepdims=True)",
     [P(pins.test_softmax_rows_sum_to_one)]),
    ("bf16 rounding: half up instead of half to even", "b = ((b + 0x7FFF + ((b >> 16) & 1)) >> 16) << 16", "b = ((b + 0x8000) >> 16) << 16",
     [P(pins.test_round_to_bf16_matches_torch)]),
    ("attention: scale 1/hd", "s = (q[h] @ keys.T) / np.sqrt(float(hd))            # [B, P+B+S]", "s = (q[h] @ keys.T) / float(hd)",
     [P(pins.test_attention_matches_torch_sdpa, B=4, pos0=9)]),
    ("attention: wrong KV head for a query head", "            kvh = h // rep\n", "            kvh = h % Hkv\n",
     [P(pins.test_attention_matches_torch_sdpa, B=4, pos0=9)]),
    ("attention: own keys not rotated", "k = rope(k.reshape(B, Hkv, hd).transpose(1, 0, 2), pos, rope_base)   # [Hkv,B,hd]",
     "k = k.reshape(B, Hkv, hd).transpose(1, 0, 2)", [P(pins.test_layer_scalar_brute_force)]),
    ("layer: block positions start at 0", "    pos = pos0 + np.arange(B)\n", "    pos = np.arange(B)\n",
     [P(pins.test_prefix_cache_equals_full_recomputation)]),
    ("layer: residual of the attention dropped", "h1 = x + o.reshape(B, Hq * hd) @ wo.T", "h1 = o.reshape(B, Hq * hd) @ wo.T",
     [P(pins.test_layer_zero_output_projections_is_identity)]),
    ("layer: gate and up swapped", "y = h1 + (silu(n2 @ wg.T) * (n2 @ wu.T)) @ wd.T", "y = h1 + (silu(n2 @ wu.T) * (n2 @ wg.T)) @ wd.T",
     [P(pins.test_layer_scalar_brute_force)]),
    ("layer: second norm applied to the input instead of the attention output", "n2 = rms_norm(h1, w[\"norm2\"], rms_eps)\n        y = h1 +",
     "n2 = rms_norm(x, w[\"norm2\"], rms_eps)\n        y = h1 +", [P(pins.test_layer_scalar_brute_force)]),
    ("dual cache: suffix ignored", "sk, sv = np.asarray(suffix_k, F64), np.asarray(suffix_v, F64)",
     "sk, sv = np.asarray(suffix_k, F64)[:, :0], np.asarray(suffix_v, F64)[:, :0]",
     [P(suffix.test_zero_keys_give_the_mean_over_prefix_block_and_suffix)]),
    ("dual cache: suffix keys rotated again", "sk, sv = np.asarray(suffix_k, F64), np.asarray(suffix_v, F64)",
     "sk, sv = rope(np.asarray(suffix_k, F64), pos0 + B + np.arange(np.shape(suffix_k)[1]), rope_base), np.asarray(suffix_v, F64)",
     [P(suffix.test_first_layer_of_a_full_bidirectional_forward)]),
    ("mask: drafts see each other", "        allow[r, r] = True\n", "        allow[r, P:P + G * B] = True\n",
     [P(pins.test_one_call_equals_many_calls_and_draft_independence)]),
    ("head: threshold not strict", "unmask[g, b] = 1 if conf[g, b] > tau32 else 0", "unmask[g, b] = 1 if conf[g, b] >= tau32 else 0",
     [P(pins.test_head_threshold_strict_force_one_and_monotone)]),
    ("head: forced position is the least confident", "best = masked[int(np.argmax(conf[g, masked]))]", "best = masked[int(np.argmin(conf[g, masked]))]",
     [P(pins.test_head_threshold_strict_force_one_and_monotone)]),
    ("head: logit scale dropped", "logits_all = logit_scale * (n @ wv.T)", "logits_all = (n @ wv.T)",
     [P(pins.test_unmask_counts_vary_with_logit_scale), P(pins.test_head_matches_torch_softmax_and_bounds)]),
    ("head: final norm dropped", "n = rms_norm(hid[g, masked_pos], final_norm, rms_eps)   # [n_masked, d]", "n = hid[g, masked_pos]",
     [P(pins.test_head_matches_torch_softmax_and_bounds), P(pins.test_head_planted_one_hot_logit)]),
    ("head: unmasked positions overwritten", "target = np.where(unmask == 1, amax, tok).astype(np.int32)", "target = amax.astype(np.int32)",
     [P(pins.test_config1_step_shapes_and_invariants), P(pins.test_head_threshold_strict_force_one_and_monotone)]),
    ("walk: child compared with its own target", "if int(p) == cur and np.array_equal(ds[int(c)], ts[cur]))", "if int(p) == cur and np.array_equal(ts[int(c)], ts[cur]))",
     [P(pins.test_accept_golden_cases)]),
    ("walk: edges followed backwards", "cand = sorted(int(c) for p, c in e\n", "cand = sorted(int(c) for c, p in e\n", [P(pins.test_accept_golden_cases)]),
    ("walk: returns the draft, not its next state", "return cur, depth, depth + 1, ts[cur].astype(np.int32).copy()", "return cur, depth, depth + 1, ds[cur].astype(np.int32).copy()",
     [P(pins.test_accept_golden_cases)]),
    ("walk: any matching state accepted, edge or not", "if int(p) == cur and np.array_equal(ds[int(c)], ts[cur]))", "if np.array_equal(ds[int(c)], ts[cur]))",
     [P(pins.test_accept_child_equal_to_target_always_accepted_non_child_never), P(pins.test_accept_brute_force_small_graphs)]),
    ("top-k: ascending", "order = sorted(range(V), key=lambda v: (-logits[b, v], v))[:k]", "order = sorted(range(V), key=lambda v: (logits[b, v], v))[:k]",
     [P(drafting.test_head_topk_first_column_is_the_head_and_rows_are_sorted)]),
    ("position rank: equal confidences to the higher position", "return sorted(masked, key=lambda b: (-float(conf[b]), b))", "return sorted(masked, key=lambda b: (-float(conf[b]), -b))",
     [P(drafting.test_equal_scores_and_repeated_rank), P(drafting.test_worked_example)]),
    ("position rank: unmasked positions ranked too", "masked = [b for b in range(len(state)) if int(state[b]) == mask_id]", "masked = [b for b in range(len(state))]",
     [P(drafting.test_worked_example), P(drafting.test_against_independent_implementation, seed=0)]),
    ("scores: arithmetic mean", "return float(np.exp(np.mean(np.log(np.asarray(v, F64)))))", "return float(np.mean(np.asarray(v, F64)))",
     [P(drafting.test_geometric_mean_properties)]),
    ("scores: unbuildable children counted", "if int(a) == m and 1 <= int(c) <= D and buildable[int(c)]})", "if int(a) == m and 1 <= int(c) <= D})",
     [P(drafting.test_worked_example), P(drafting.test_against_independent_implementation, seed=1),
      P(drafting.test_against_independent_implementation, seed=2), P(drafting.test_against_independent_implementation, seed=3)]),
    ("scores: child score alone", "score[m] = geometric_mean([local[m], child[m]])               # score", "score[m] = child[m]",
     [P(drafting.test_worked_example)]),
    ("drafts: vocabulary rank off by one", "drafts[m, b] = int(topk_tokens[b, j - 1])", "drafts[m, b] = int(topk_tokens[b, min(j, K - 1)])",
     [P(drafting.test_worked_example)]),
    ("full sequence: drafts see the true block instead of themselves", "keys = np.concatenate([pk[c], kg[c], ks[c]], axis=0)",
     "keys = np.concatenate([pk[c], blocks[0][1][c], ks[c]], axis=0)", [P(fullseq.test_dense_mask_formulation_through_all_layers)]),
    ("full sequence: suffix at the block's positions", "pos_s = pos0 + B + np.arange(S)", "pos_s = pos0 + np.arange(S)",
     [P(fullseq.test_dense_mask_formulation_through_all_layers)]),
    ("full sequence: the suffix sees a draft instead of the true block", "    _, k0, v0 = blocks[0]  ", "    _, k0, v0 = blocks[-1]  ",
     [P(fullseq.test_dense_mask_formulation_through_all_layers)]),
    ("full sequence: the suffix is not updated", "out_s = rest(xs, o.reshape(S, Hq * hd)) if S else xs.copy()", "out_s = xs.copy()",
     [P(fullseq.test_one_state_is_a_plain_cached_forward_over_block_and_suffix)]),
    ("full sequence: values handed back for the cache are the keys", "        return out_b, out_s, k0, v0", "        return out_b, out_s, k0, k0",
     [P(fullseq.test_dense_mask_formulation_through_all_layers)]),
    ("full sequence: the decode loop ignores the suffix", '        if "suffix_tokens" in model:', '        if "suffix_tokens_" in model:',
     [P(fullseq.test_decode_loop_of_a_full_sequence_model)]),
    ("subgraph: only level 1 is a root", "return all(level[q] in (1, 2) or (parents[q] & g) for q in g)", "return all(level[q] in (1,) or (parents[q] & g) for q in g)",
     [P(subgraph.test_hand_worked_example)]),
    ("subgraph: edges reversed", "            parents[q].add(int(p))\n    best, best_mask", "            parents[p].add(int(q))\n    best, best_mask",
     [P(subgraph.test_hand_worked_example)]),
    ("subgraph: every parent required", "return all(level[q] in (1, 2) or (parents[q] & g) for q in g)", "return all(level[q] in (1, 2) or (parents[q] and parents[q] <= g) for q in g)",
     [P(subgraph.test_one_parent_in_the_set_is_enough_and_direction_matters)]),
    ("subgraph: equal sums to the larger mask", "(total == best_sum and mask < best_mask)", "(total == best_sum and mask > best_mask)",
     [P(subgraph.test_equal_sums_go_to_the_smallest_mask_and_level_three_is_not_a_root)]),
    ("subgraph: disconnected sets counted", "        if not subgraph_is_connected(nodes, level, parents):\n            continue\n", "",
     [P(subgraph.test_hand_worked_example)]),
]


def test_untouched_oracle_passes_every_pin_used_here(monkeypatch):
    checks = {(fn.__name__, tuple(sorted(kw.items()))): (fn, kw) for _, _, _, cs in CASES for fn, kw in cs}
    assert run(build(SRC), list(checks.values()), monkeypatch) == []


@pytest.mark.parametrize("label,old,new,checks", CASES, ids=[c[0] for c in CASES])
def test_planted_mistake_fails_a_pin(label, old, new, checks, monkeypatch):
    assert SRC.count(old) == 1, "the text to replace must occur exactly once: %r" % old
    failed = run(build(SRC.replace(old, new)), checks, monkeypatch)
    assert failed, "no pin noticed: " + label

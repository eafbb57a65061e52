"""Are the pins of the attention oracle sharp?  Each case plants ONE plausible mistake in a copy of the
oracle's source (a dropped factor, an off-by-one in the causal bound, a wrong head mapping, a wrong block or
slot, a transposed tile, a forgotten normalisation, ...) and runs the pins of tests/test_oracle_pins.py against
the mutant: the brute-force comparison must reject it, and so must at least one pin that does not lean on
the brute force (a library routine, a closed form or an invariant).  Everything here runs on the CPU."""
import inspect
import re

import numpy as np
import pytest

from oracle import ref_numpy

import test_oracle_pins as P

SOURCE = inspect.getsource(ref_numpy.attn_mixed)

# (name, text of the oracle, text of the mistake)
MUTANTS = [
    ("scale dropped", "scale * (kt @ qv)", "(kt @ qv)"),
    ("scale squared", "scale * (kt @ qv)", "scale * scale * (kt @ qv)"),
    ("own key left out (causal bound one short)", "n = pos + 1 ", "n = max(pos, 1) "),
    ("one key too many (causal bound one long)", "n = pos + 1 ", "n = min(pos + 2, ctx + (q1 - q0)) "),
    ("chunk rows all see the whole chunk (no causal mask inside the step)", "n = pos + 1 ", "n = ctx + (q1 - q0) "),
    ("position ignores the cached prefix", "pos = ctx + t", "pos = t if q1 - q0 > 1 else ctx + t"),
    ("kv head by interleaving instead of contiguous groups", "kap = h // g", "kap = h % Hkv"),
    ("kv head always 0", "kap = h // g", "kap = 0"),
    ("logical block used as physical block", "blk = int(block_tables[i][jb])", "blk = jb % NB"),
    ("block table row of the wrong sequence", "blk = int(block_tables[i][jb])", "blk = int(block_tables[0][jb])"),
    ("K tile read without the transpose of its 8-element groups", ".transpose(1, 0, 2).reshape(cnt, hd)",
     ".reshape(hd // 8 * cnt, 8).reshape(cnt, hd)"),
    ("V tile not transposed back (dims and slots swapped)", "vt = widen_bf16(v_cache[blk, kap, :, :cnt]).T",
     "vt = widen_bf16(v_cache[blk, kap, :, :cnt]).reshape(cnt, hd)"),
    ("V taken from the K pool", "vt = widen_bf16(v_cache[blk, kap, :, :cnt]).T",
     "vt = widen_bf16(k_cache[blk, kap, :, :cnt, :]).transpose(1, 0, 2).reshape(cnt, hd)"),
    ("weights not normalised", "p = e / e.sum()", "p = e"),
    ("normalised by the largest weight", "p = e / e.sum()", "p = e / e.max()"),
    # (the same function on moderate scores: only the pin that drives exp() out of range can tell)
    ("no maximum subtracted", "e = np.exp(s - s.max())", "e = np.exp(s)", "overflow only"),
    ("softmax over the negated scores", "e = np.exp(s - s.max())", "e = np.exp(s.min() - s)"),
    ("weights applied in reverse key order", "out[q0 + t, h] = p @ vals", "out[q0 + t, h] = p[::-1] @ vals"),
    ("query row of the wrong token", "qv = widen_bf16(q[q0 + t, h])", "qv = widen_bf16(q[q0 + (q1 - q0 - 1 - t), h])"),
    ("query head of the neighbour", "qv = widen_bf16(q[q0 + t, h])", "qv = widen_bf16(q[q0 + t, (h + 1) % Hq])"),
    ("output row of the wrong token", "out[q0 + t, h] = p @ vals", "out[q0 + (q1 - q0 - 1 - t), h] = p @ vals"),
    ("partial last block dropped", "for jb in range((n + BS - 1) // BS):", "for jb in range(max(1, n // BS)):"),
]

BRUTE = [lambda: P.test_config1_matches_dense_bruteforce_and_c()] + \
        [lambda s=s: P.test_random_tiny_cases_match_dense_bruteforce(s) for s in (0, 2, 9)] + \
        [lambda: P.test_grouped_head_shapes_match_dense_bruteforce(8, 2)]
# pins that stand on a library routine, a closed form or an invariant
OTHER = [
    P.test_prefill_without_context_equals_torch_sdpa_causal,
    P.test_decode_equals_torch_sdpa_single_query_no_mask,
    P.test_chunk_on_prior_context_equals_sdpa_with_explicit_mask_and_gqa_repeat,
    P.test_probability_rows_sum_to_one_and_have_causal_length,
    P.test_adding_a_constant_to_every_score_changes_nothing,
    P.test_golden_two_key_rational_example,
    P.test_constant_v_returns_v,
    P.test_zero_query_gives_mean_of_visible_values,
    P.test_single_key_decode_returns_v0,
    P.test_dominant_key_selects_its_value_row,
    P.test_output_is_invariant_under_permuting_physical_blocks_and_poison,
    P.test_causal_future_keys_do_not_matter,
    P.test_decode_equals_last_row_of_full_prefill,
    P.test_chunk_rows_equal_rows_of_full_prefill,
    P.test_gqa_equals_mha_with_repeated_kv_heads,
    P.test_kv_head_mapping_is_contiguous_groups,
    P.test_sequences_are_independent_and_order_permutes_rows,
]


def mutant_of(old, new):
    assert SOURCE.count(old) == 1, f"the oracle no longer contains {old!r} exactly once"
    ns = dict(vars(ref_numpy))
    exec(compile(SOURCE.replace(old, new), "<mutant>", "exec"), ns)
    return ns["attn_mixed"]


def rejects(pin):
    with np.errstate(all="ignore"):
        try:
            pin()
        except AssertionError:
            return True
        except (ValueError, IndexError, FloatingPointError):   # a mistake may also break shapes or indices
            return True
    return False


def test_every_pin_accepts_the_oracle_as_it_stands():
    for pin in BRUTE + OTHER:
        pin()


@pytest.mark.parametrize("case", MUTANTS, ids=[re.sub(r"\W+", "_", m[0]) for m in MUTANTS])
def test_a_planted_mistake_is_rejected(monkeypatch, case):
    name, old, new = case[:3]
    monkeypatch.setattr(ref_numpy, "attn_mixed", mutant_of(old, new))
    if len(case) == 3:
        assert any(rejects(pin) for pin in BRUTE), f"'{name}' passes the brute-force comparison"
    caught = [pin.__name__ for pin in OTHER if rejects(pin)]
    assert caught, f"'{name}' passes every pin that does not use the brute force"

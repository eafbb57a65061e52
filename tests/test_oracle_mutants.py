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


# ------------------------------------------------------------------------------------------------------------
# The same for the other oracles: KV append, the latency model (Table 2, Equation 1), Mix Decoding Selection
# (Algorithm 2), the migration decision (Algorithm 1) and the eviction rule.  A mutant must be rejected by at
# least one of the module's pins.
from oracle import migration, mix_select, perf_model  # noqa: E402

APPEND_PINS = [P.test_kv_append_offsets_of_a_hand_worked_example, P.test_kv_append_rebuilds_the_cache_and_touches_nothing_else,
               P.test_kv_append_reads_back_through_the_independent_gather]
MODEL_PINS = [P.test_model_operator_counts_equal_hand_evaluated_table2_rows, P.test_model_equation1_regimes_and_crossing,
              P.test_model_iteration_is_the_sum_of_operators_plus_overheads,
              P.test_model_causal_count_is_the_number_of_visible_pairs]
MIX_PINS = [P.test_mix_selection_hand_worked_example, P.test_mix_selection_equal_lengths_closed_form,
            P.test_mix_selection_invariants_by_exhaustive_scan, P.test_mix_selection_bounds_are_inclusive]
MIG_PINS = [P.test_migration_hand_worked_examples, P.test_migration_preference_closed_forms_in_the_memory_bound_regime,
            P.test_migration_preference_is_the_maximum_by_direct_evaluation, P.test_eviction_victims_against_every_subset]

# (module, function, pins, name, text of the oracle, text of the mistake)
OTHER_MUTANTS = [
    (ref_numpy, "kv_append", APPEND_PINS, "slot from the row index instead of the position", "), pos % BS", "), t % BS"),
    (ref_numpy, "kv_append", APPEND_PINS, "position ignores the cached prefix", "pos = int(ctx_lens[i]) + t", "pos = t"),
    (ref_numpy, "kv_append", APPEND_PINS, "K written in V's layout", "k_cache[blk, kv, d // 8, slot, d % 8]",
     "k_cache[blk, kv, d % (hd // 8), slot, d // (hd // 8)]"),
    (ref_numpy, "kv_append", APPEND_PINS, "row of the wrong sequence", "k_new[q0 + t, kv, d]", "k_new[t, kv, d]"),
    (ref_numpy, "kv_append", APPEND_PINS, "V of the neighbouring kv head", "v_new[q0 + t, kv, d]", "v_new[q0 + t, (kv + 1) % Hkv, d]"),
    (perf_model, "attention_flops", MODEL_PINS, "one of the two matrix products forgotten", "4.0 *", "2.0 *"),
    (perf_model, "attention_bytes", MODEL_PINS, "K/V bytes per query head instead of per kv head", "S_kv * D_h * Hkv / Hq", "S_kv * D_h"),
    (perf_model, "attention_bytes", MODEL_PINS, "only K counted", "2.0 * d * (S_q * D_h + S_kv * D_h * Hkv / Hq)",
     "d * (2.0 * S_q * D_h + S_kv * D_h * Hkv / Hq)"),
    (perf_model, "attention_bytes", MODEL_PINS, "group ratio upside down", "Hkv / Hq", "Hq / Hkv"),
    (perf_model, "op_latency", MODEL_PINS, "sum instead of maximum", "max(flops / F, nbytes / M)", "flops / F + nbytes / M"),
    (perf_model, "op_latency", MODEL_PINS, "minimum instead of maximum", "max(flops / F, nbytes / M)", "min(flops / F, nbytes / M)"),
    (perf_model, "attention_flops_causal", MODEL_PINS, "own key not counted", "pairs += ctx + t + 1", "pairs += ctx + t"),
    (perf_model, "predict", MODEL_PINS, "decode rate used for prefill", 'F = params["F_ap"] if ql > 1 else params["F_ad"]',
     'F = params["F_ad"]'),
    (perf_model, "predict", MODEL_PINS, "overheads charged whether or not the kind of work is there",
     '(params["O_p"] if any_p else 0.0) + (params["O_d"] if any_d else 0.0)', 'params["O_p"] + params["O_d"]'),
    (perf_model, "predict", MODEL_PINS, "overhead left out", "latency=t_prefill + t_decode + overhead", "latency=t_prefill + t_decode"),
    (perf_model, "predict", MODEL_PINS, "S_kv without the new tokens", "attention_bytes(Hq, Hkv, hd, ql, ctx + ql, d)",
     "attention_bytes(Hq, Hkv, hd, ql, ctx, d)"),
    (mix_select, "mix_decoding_select", MIX_PINS, "a request that reaches the bound exactly is refused",
     "batch + [int(offline_lens[r])]) <= S", "batch + [int(offline_lens[r])]) < S"),
    # (not planted: letting refused requests back into the sorted phase changes nothing, because the predictor
    # grows with a request's length: whatever was refused once stops the prefix exactly where the oracle stops)
    (mix_select, "mix_decoding_select", MIX_PINS, "sorted by descending length", "key=lambda i: (int(offline_lens[i]), i))",
     "key=lambda i: (-int(offline_lens[i]), i))"),
    (mix_select, "mix_decoding_select", MIX_PINS, "prefix one short", "for i in rest[:lo]:", "for i in rest[:max(lo - 1, 0)]:"),
    (mix_select, "mix_decoding_select", MIX_PINS, "admitted request not added to the batch", "            batch.append(int(offline_lens[r]))\n",
     "            pass\n"),
    (mix_select, "mix_decoding_select", MIX_PINS, "bisection keeps the first admissible prefix", "                lo = mid\n",
     "                lo = mid\n                break\n"),
    (mix_select, "latency", MIX_PINS, "length counted without the new token twice", "[int(n) - 1 for n in lens]", "[int(n) - 2 for n in lens]"),
    (migration, "migration_preference", MIG_PINS, "headroom test inverted", "if not (L(B) < S and all_included):", "if L(B) < S and all_included:"),
    (migration, "migration_preference", MIG_PINS, "node not required to be drained", "L(B) < S and all_included", "L(B) < S"),
    (migration, "migration_preference", MIG_PINS, "memory not checked when saturated",
     "if L(B + [l]) <= S and u_mem(B + [l], block_size, capacity_blocks) <= 1.0]", "if L(B + [l]) <= S]"),
    (migration, "migration_preference", MIG_PINS, "shortest that fits instead of longest (saturated)",
     'pref=max(fits) if fits else None, branch="saturated"', 'pref=min(fits) if fits else None, branch="saturated"'),
    (migration, "migration_preference", MIG_PINS, "one request assumed instead of the missing n", "if L(B + [l] * n) <= S]", "if L(B + [l]) <= S]"),
    (migration, "migration_preference", MIG_PINS, "saturation test off by one", "if len(B) >= bs_sat:", "if len(B) > bs_sat:"),
    (migration, "migration_preference", MIG_PINS, "longest instead of shortest when saturation is out of reach",
     'return dict(pref=len_min, branch="shortest")', 'return dict(pref=len_max, branch="shortest")'),
    (migration, "migration_select", MIG_PINS, "longest first instead of closest to the preference",
     "key=lambda i: (abs(int(relaxed_lens[i]) - pref), int(relaxed_lens[i]), i))", "key=lambda i: (-int(relaxed_lens[i]), i))"),
    (migration, "migration_select", MIG_PINS, "batch not grown by what was taken", "            B = cand\n", ""),
    (migration, "eviction_victims", MIG_PINS, "long requests evicted when memory-bound", "compute_bound = batch_size >= bs_sat",
     "compute_bound = batch_size < bs_sat"),
    (migration, "eviction_victims", MIG_PINS, "victims that are not needed are kept", "            if freed - b >= need_blocks:",
     "            if False:"),
    (migration, "eviction_victims", MIG_PINS, "stops one victim early", "        if freed >= need_blocks:\n            break",
     "        if freed + blocks(offline_lens[i], block_size) >= need_blocks:\n            break"),
    (migration, "blocks", MIG_PINS, "blocks rounded down", "(int(length) + block_size - 1) // block_size", "int(length) // block_size"),
]


@pytest.mark.parametrize("case", OTHER_MUTANTS, ids=[f"{m[1]}__" + re.sub(r"\W+", "_", m[3]) for m in OTHER_MUTANTS])
def test_a_planted_mistake_in_the_other_oracles_is_rejected(monkeypatch, case):
    module, func, pins, name, old, new = case
    src = inspect.getsource(getattr(module, func))
    assert src.count(old) == 1, f"{func} no longer contains {old!r} exactly once"
    ns = dict(vars(module))
    exec(compile(src.replace(old, new), "<mutant>", "exec"), ns)
    monkeypatch.setattr(module, func, ns[func])
    caught = [pin.__name__ for pin in pins if rejects(pin)]
    assert caught, f"'{name}' in {func} passes every pin of its module"


# ------------------------------------------------------------------------------------------------------------
# Would the GPU parity tests notice?  The kernels are held to max-abs 2e-2 / mean-abs 2e-3 / relative L2 1e-2
# against the oracle.  On the inputs of the GPU parity cases (tests/test_gpu_parity.py, the smaller ones) every
# planted mistake, with its output rounded to bf16 like a kernel's, must break those gates: the tolerance is
# wide enough for bf16 rounding and not wide enough to hide a wrong kernel.
def test_the_parity_gates_on_the_gpu_cases_reject_every_planted_mistake():
    import gpu_util
    import test_gpu_parity as G
    from paper_2511_21862_amd import workloads as W

    cases = []
    for case in (0, 9, 6, 5, 4, 7, 1):
        Hq, Hkv, hd, ql, ctx = G.RAGGED[case]
        nblk = int(sum((c + q + 15) // 16 for c, q in zip(ctx, ql))) + 7
        b = W.build_batch(Hq=Hq, Hkv=Hkv, hd=hd, q_lens=ql, ctx_lens=ctx, num_blocks=nblk, seed=1000 + case, poison=True)
        cases.append((case, b, P.run(b)))
    # the oracle itself, rounded to bf16, passes
    for case, b, ref in cases:
        e = gpu_util.errors(W.f32_to_bf16_bits(ref.astype(np.float32)), ref)
        assert e["max_abs"] <= gpu_util.MAX_ABS / 2 and e["mean_abs"] <= gpu_util.MEAN_ABS / 2 and e["rel_l2"] <= gpu_util.REL_L2 / 2
    for m in MUTANTS:
        if len(m) > 3:
            continue
        fn = mutant_of(m[1], m[2])
        broke = None
        for case, b, ref in cases:
            with np.errstate(all="ignore"):
                try:
                    out = P.run(b, fn)
                except (ValueError, IndexError):
                    broke = case
                    break
            with np.errstate(all="ignore"):
                e = gpu_util.errors(W.f32_to_bf16_bits(np.nan_to_num(out, nan=np.inf).astype(np.float32)), ref)
            if not (e["finite"] and e["max_abs"] <= gpu_util.MAX_ABS and e["mean_abs"] <= gpu_util.MEAN_ABS
                    and e["rel_l2"] <= gpu_util.REL_L2):
                broke = case
                break
        assert broke is not None, f"'{m[0]}' stays within the parity gates on every case"

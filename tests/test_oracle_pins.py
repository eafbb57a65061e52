"""Pins for the CPU oracle: things fixed by the paper's operator definition and by mathematics,
none of which restate the oracle's own formula.  All run without a GPU."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import dense_bruteforce, ref_c, ref_numpy
from paper_2511_21862_amd import accounting
from paper_2511_21862_amd import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def run(b, fn=None, **kw):
    fn = fn or ref_numpy.attn_mixed   # (looked up at call time: tests/test_oracle_mutants.py swaps it)
    return fn(b.q, b.k_cache, b.v_cache, b.block_tables, b.seq_lens, b.query_start_loc, b.ctx_lens, **kw)


def bits(x):
    out = W.f32_to_bf16_bits(np.atleast_1d(np.asarray(x, dtype=np.float32)))
    return out[0] if np.ndim(x) == 0 else out


def f64(u):
    return W.bf16_bits_to_f32(u).astype(np.float64)


def tiny(seed, Hq=4, Hkv=2, hd=16, q_lens=(1, 5, 1), ctx_lens=(20, 7, 0), nblk=16, poison=False, **kw):
    return W.build_batch(Hq=Hq, Hkv=Hkv, hd=hd, q_lens=q_lens, ctx_lens=ctx_lens, num_blocks=nblk, seed=seed,
                         poison=poison, **kw)


# --------------------------------------------------------------------------- brute force
def test_config1_matches_dense_bruteforce_and_c():
    b = W.config1(poison=True)
    o = run(b)
    assert np.isfinite(o).all()
    assert np.abs(o - run(b, dense_bruteforce.attn_mixed_dense)).max() <= 1e-12
    assert np.abs(o - run(b, ref_c.attn_mixed)).max() <= 1e-12


@pytest.mark.parametrize("seed", range(12))
def test_random_tiny_cases_match_dense_bruteforce(seed):
    rng = np.random.default_rng(100 + seed)
    Hq = int(rng.choice([1, 4, 8]))
    Hkv = int(rng.choice([h for h in (1, 2, 4, 8) if Hq % h == 0]))
    hd = int(rng.choice([8, 16, 64])) if seed % 4 else 128
    n = int(rng.integers(1, 4))
    ql = [int(rng.choice([1, 1, int(rng.integers(1, 49))])) for _ in range(n)]
    ctx = [int(rng.integers(0, 71)) for _ in range(n)]
    if seed == 0:
        ql, ctx = [1, 1], [129, 0]          # seq 130 and the one-key decode
    b = W.build_batch(Hq=Hq, Hkv=Hkv, hd=hd, q_lens=ql, ctx_lens=ctx, num_blocks=24, seed=seed, poison=True)
    o = run(b)
    assert np.abs(o - run(b, dense_bruteforce.attn_mixed_dense)).max() <= 1e-12
    assert np.abs(o - run(b, ref_c.attn_mixed)).max() <= 1e-12


# --------------------------------------------------------------------------- library special cases
@pytest.mark.parametrize("Hq,Hkv", [(8, 2), (8, 4), (6, 3), (12, 4), (14, 2)])
def test_grouped_head_shapes_match_dense_bruteforce(Hq, Hkv):
    """1 < Hkv < Hq, where a contiguous and an interleaved head-to-kv-head mapping differ."""
    b = W.build_batch(Hq=Hq, Hkv=Hkv, hd=16, q_lens=[1, 7, 1], ctx_lens=[21, 18, 0], num_blocks=12, seed=Hq * 31 + Hkv,
                      poison=True)
    o = run(b)
    assert np.abs(o - run(b, dense_bruteforce.attn_mixed_dense)).max() <= 1e-12
    assert np.abs(o - run(b, ref_c.attn_mixed)).max() <= 1e-12


def test_prefill_without_context_equals_torch_sdpa_causal():
    b = tiny(1, Hq=2, Hkv=2, hd=16, q_lens=(23,), ctx_lens=(0,))
    k, v = W.gather_logical(b, 0)
    Q = torch.from_numpy(f64(b.q)).permute(1, 0, 2)[None]          # [1, H, L, hd]
    K = torch.from_numpy(f64(k)).permute(1, 0, 2)[None]
    V = torch.from_numpy(f64(v)).permute(1, 0, 2)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(Q, K, V, is_causal=True)[0].permute(1, 0, 2).numpy()
    assert np.abs(run(b) - ref).max() <= 1e-12


def test_decode_equals_torch_sdpa_single_query_no_mask():
    b = tiny(2, Hq=4, Hkv=4, hd=32, q_lens=(1,), ctx_lens=(52,))
    k, v = W.gather_logical(b, 0)
    Q = torch.from_numpy(f64(b.q)).permute(1, 0, 2)[None]
    K = torch.from_numpy(f64(k)).permute(1, 0, 2)[None]
    V = torch.from_numpy(f64(v)).permute(1, 0, 2)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(Q, K, V, is_causal=False)[0].permute(1, 0, 2).numpy()
    assert np.abs(run(b) - ref).max() <= 1e-12


def test_chunk_on_prior_context_equals_sdpa_with_explicit_mask_and_gqa_repeat():
    b = tiny(3, Hq=4, Hkv=2, hd=16, q_lens=(9,), ctx_lens=(30,))
    k, v = W.gather_logical(b, 0)
    L, c, ctx = 39, 9, 30
    Q = torch.from_numpy(f64(b.q)).permute(1, 0, 2)[None]
    K = torch.from_numpy(f64(k)).permute(1, 0, 2).repeat_interleave(2, dim=0)[None]   # kv head h//2
    V = torch.from_numpy(f64(v)).permute(1, 0, 2).repeat_interleave(2, dim=0)[None]
    mask = torch.arange(L)[None, :] <= (torch.arange(c)[:, None] + ctx)
    ref = torch.nn.functional.scaled_dot_product_attention(Q, K, V, attn_mask=mask)[0].permute(1, 0, 2).numpy()
    assert np.abs(run(b) - ref).max() <= 1e-12


# --------------------------------------------------------------------------- softmax
def test_probability_rows_sum_to_one_and_have_causal_length():
    b = W.config1()
    _, probs = run(b, return_probs=True)
    expect_len = []
    for i in range(b.num_seqs):
        for t in range(int(b.q_lens[i])):
            expect_len += [int(b.ctx_lens[i]) + t + 1] * b.Hq
    assert [len(p) for p in probs] == expect_len
    assert max(abs(p.sum() - 1.0) for p in probs) <= 1e-14
    assert all((p >= 0).all() for p in probs)


def test_adding_a_constant_to_every_score_changes_nothing():
    b = tiny(4, Hq=2, Hkv=1, hd=16, q_lens=(1, 6), ctx_lens=(33, 12))
    for s in range(b.num_seqs):
        k, v = W.gather_logical(b, s)
        k[:, :, 15] = bits(1.0)                       # every key carries a 1 in the last feature
        W.scatter_logical(b, s, k, v)
    b.q[:, :, 15] = bits(0.0)
    base = run(b)
    b.q[:, :, 15] = bits(96.0)                        # +96*scale on every score of every row
    shifted = run(b)
    assert np.abs(base - shifted).max() <= 1e-12
    b.q[:, :, 15] = bits(3000.0)                      # would overflow exp() without max-subtraction
    assert np.abs(base - run(b)).max() <= 1e-9


# --------------------------------------------------------------------------- closed forms
def test_golden_two_key_rational_example():
    exp = np.loadtxt(os.path.join(GOLD, "two_key_softmax.txt"))
    b = W.build_batch(Hq=1, Hkv=1, hd=8, q_lens=[1], ctx_lens=[1], num_blocks=2, seed=0)
    k = np.zeros((2, 1, 8), np.float32)
    k[1, 0, 0] = 1.0
    v = np.zeros((2, 1, 8), np.float32)
    v[0, 0, :4] = [1, -2, 4, 0]
    v[1, 0, :4] = [-3, 2, 0.5, 8]
    W.scatter_logical(b, 0, bits(k), bits(v))
    b.q[:] = bits(np.eye(1, 8, dtype=np.float32))[None]
    for fn in (ref_numpy.attn_mixed, ref_c.attn_mixed, dense_bruteforce.attn_mixed_dense):
        o = run(b, fn, scale=math.log(3.0))
        assert np.abs(o[0, 0, :4] - exp[:, 1]).max() <= 1e-15
        assert np.abs(o[0, 0, 4:]).max() == 0.0


def test_constant_v_returns_v():
    b = tiny(5, q_lens=(1, 7), ctx_lens=(40, 3))
    row = bits(np.linspace(-2, 2, b.hd, dtype=np.float32))
    for s in range(b.num_seqs):
        k, v = W.gather_logical(b, s)
        v[:] = row
        W.scatter_logical(b, s, k, v)
    o = run(b)
    assert np.abs(o - f64(row)[None, None, :]).max() <= 1e-14


def test_zero_query_gives_mean_of_visible_values():
    b = tiny(6, Hq=2, Hkv=1, hd=8, q_lens=(4,), ctx_lens=(10,))
    b.q[:] = 0
    _, v = W.gather_logical(b, 0)
    o = run(b)
    for t in range(4):
        assert np.abs(o[t, 0] - f64(v[: 10 + t + 1, 0]).mean(axis=0)).max() <= 1e-14
        assert np.abs(o[t, 1] - o[t, 0]).max() == 0.0
    assert np.abs(run(b, scale=0.0) - o).max() <= 1e-14      # scale 0 with any q: same thing


def test_single_key_decode_returns_v0():
    b = tiny(7, Hq=2, Hkv=2, hd=8, q_lens=(1,), ctx_lens=(0,))
    _, v = W.gather_logical(b, 0)
    o = run(b)
    assert np.array_equal(o[0], f64(v[0]))


def test_dominant_key_selects_its_value_row():
    b = tiny(8, Hq=1, Hkv=1, hd=8, q_lens=(1,), ctx_lens=(19,))
    k, v = W.gather_logical(b, 0)
    k[:] = 0
    k[11, 0, 0] = bits(1.0)
    W.scatter_logical(b, 0, k, v)
    b.q[:] = 0
    b.q[0, 0, 0] = bits(1.0)
    o = run(b, scale=50.0)                                    # key 11 scores 50 above the rest
    assert np.abs(o[0, 0] - f64(v[11, 0])).max() <= 20 * math.exp(-50.0) * 10


# --------------------------------------------------------------------------- paging
def test_output_is_invariant_under_permuting_physical_blocks_and_poison():
    clean = W.config1(poison=False)
    dirty = W.config1(poison=True)
    o = run(clean)
    assert np.array_equal(o, run(dirty))                      # unowned slots are never read
    assert np.array_equal(o, run(W.permute_blocks(clean, 9)))
    assert np.array_equal(run(dirty, ref_c.attn_mixed), run(W.permute_blocks(dirty, 10), ref_c.attn_mixed))


def test_causal_future_keys_do_not_matter():
    b = tiny(9, Hq=2, Hkv=1, hd=8, q_lens=(6,), ctx_lens=(5,))
    o = run(b)
    k, v = W.gather_logical(b, 0)
    k[8:] = bits(np.full_like(k[8:], 7.0, dtype=np.float32))   # keys 8.. are invisible to rows 0..2 (pos 5..7)
    v[8:] = bits(np.full_like(v[8:], -9.0, dtype=np.float32))
    W.scatter_logical(b, 0, k, v)
    o2 = run(b)
    assert np.array_equal(o[:3], o2[:3])
    assert not np.array_equal(o[3], o2[3])                     # row 3 (pos 8) does see key 8


# --------------------------------------------------------------------------- decode == prefill row, chunking
def _same_sequence(Hq, Hkv, hd, L, splits, seed):
    """The same L-token sequence presented as chunks [ctx, ctx+c) for each (ctx, c) in splits."""
    rng = np.random.default_rng(seed)
    k = bits(rng.standard_normal((L, Hkv, hd), dtype=np.float32))
    v = bits(rng.standard_normal((L, Hkv, hd), dtype=np.float32))
    qfull = bits(rng.standard_normal((L, Hq, hd), dtype=np.float32))
    outs = []
    for n, (ctx, c) in enumerate(splits):
        b = W.build_batch(Hq=Hq, Hkv=Hkv, hd=hd, q_lens=[c], ctx_lens=[ctx], num_blocks=8, seed=seed + n)
        W.scatter_logical(b, 0, k[: ctx + c], v[: ctx + c])
        b.q[:] = qfull[ctx: ctx + c]
        outs.append(run(b))
    return outs


def test_decode_equals_last_row_of_full_prefill():
    full, dec = _same_sequence(4, 2, 16, 45, [(0, 45), (44, 1)], 11)
    assert np.abs(full[-1] - dec[0]).max() <= 1e-13


def test_chunk_rows_equal_rows_of_full_prefill():
    full, a, b2, c = _same_sequence(4, 1, 16, 50, [(0, 50), (0, 17), (17, 20), (37, 13)], 12)
    assert np.abs(np.concatenate([a, b2, c]) - full).max() <= 1e-13


# --------------------------------------------------------------------------- GQA
def test_gqa_equals_mha_with_repeated_kv_heads():
    b = tiny(13, Hq=8, Hkv=2, hd=16, q_lens=(1, 5), ctx_lens=(21, 9))
    o = run(b)
    m = W.build_batch(Hq=8, Hkv=8, hd=16, q_lens=b.q_lens, ctx_lens=b.ctx_lens, num_blocks=16, seed=99)
    m.q[:] = b.q
    for s in range(b.num_seqs):
        k, v = W.gather_logical(b, s)
        W.scatter_logical(m, s, np.repeat(k, 4, axis=1), np.repeat(v, 4, axis=1))   # head h uses kv head h//4
    assert np.abs(o - run(m)).max() <= 1e-14


def test_kv_head_mapping_is_contiguous_groups():
    # heads 0,1 must read kv head 0 and heads 2,3 kv head 1: make kv head 1 constant
    b = tiny(14, Hq=4, Hkv=2, hd=8, q_lens=(1,), ctx_lens=(9,))
    k, v = W.gather_logical(b, 0)
    v[:, 1, :] = bits(5.0)
    W.scatter_logical(b, 0, k, v)
    o = run(b)
    assert np.abs(o[0, 2:] - 5.0).max() <= 1e-14 and np.abs(o[0, :2] - 5.0).min() > 1e-3


# --------------------------------------------------------------------------- batch structure
def test_sequences_are_independent_and_order_permutes_rows():
    b = tiny(15, q_lens=(1, 5, 1, 3), ctx_lens=(20, 7, 0, 31), nblk=24)
    o = run(b)
    order = [2, 0, 3, 1]
    s = W.subset(b, order)
    os_ = run(s)
    assert np.array_equal(os_, o[s.extra["rows"]])
    one = W.subset(b, [3])
    assert np.array_equal(run(one), o[one.extra["rows"]])


def test_empty_cases():
    b = tiny(16, q_lens=(0, 1), ctx_lens=(5, 8))
    o = run(b)
    assert o.shape == (1, 4, 16)
    e = W.build_batch(Hq=4, Hkv=2, hd=16, q_lens=[], ctx_lens=[], num_blocks=4, seed=0)
    assert run(e).shape == (0, 4, 16) and run(e, ref_c.attn_mixed).shape == (0, 4, 16)


# --------------------------------------------------------------------------- block copy
def test_block_copy_oracles_agree_and_leave_other_blocks_alone():
    b = tiny(17, nblk=12)
    src = np.array([3, 7, 0, 11], np.int64)
    dst = np.array([1, 2, 5, 4], np.int64)
    outs = []
    for fn in (ref_numpy.block_copy, ref_c.block_copy):
        kd = np.full((8,) + b.k_shape()[1:], 0xABCD, np.uint16)
        vd = np.full((8,) + b.v_shape()[1:], 0xABCD, np.uint16)
        fn(b.k_cache, b.v_cache, kd, vd, src, dst)
        outs.append((kd, vd))
        for s, d in zip(src, dst):
            assert kd[d].tobytes() == b.k_cache[s].tobytes() and vd[d].tobytes() == b.v_cache[s].tobytes()
        for d in (0, 3, 6, 7):
            assert (kd[d] == 0xABCD).all() and (vd[d] == 0xABCD).all()
    assert np.array_equal(outs[0][0], outs[1][0]) and np.array_equal(outs[0][1], outs[1][1])


# --------------------------------------------------------------------------- accounting vs Table 2
def test_accounting_matches_table2_golden_values():
    rows = np.loadtxt(os.path.join(GOLD, "table2_attention.txt"), dtype=np.int64)
    for Hq, Hkv, hd, Sq, Skv, flops, nbytes in rows:
        D_h = int(Hq * hd)
        assert accounting.table2_flops(D_h, int(Sq), int(Skv)) == flops
        assert accounting.table2_bytes(D_h, int(Sq), int(Skv), int(Hq), int(Hkv)) == nbytes
        w = accounting.batch_work(int(Hq), int(Hkv), int(hd), 16, [int(Skv)], [int(Sq)])
        assert w["flops_table2"] == flops
        # batch_work adds only the block-table entries on top of the Table-2 bytes
        assert w["bytes_total"] - ((int(Skv) + 15) // 16) * 4 == nbytes


def test_causal_flops_count_visible_pairs():
    w = accounting.batch_work(4, 1, 64, 16, [32], [32])
    assert w["flops_causal"] == 4 * 256 * (32 * 33 // 2)       # 0.54 MFLOP for the tiny prefill chunk
    w = accounting.batch_work(32, 8, 128, 16, [100 + 512], [512])
    assert w["flops_causal"] == 4 * 4096 * (512 * 100 + 512 * 513 // 2)


def test_row_sample_reproduces_rows_of_the_full_batch():
    # the sampled-row batches handed to the oracle by the full-size GPU tests: row t of a chunk, recast as a
    # single-query sequence over its visible keys, gives exactly the row of the whole-batch result
    b = W.build_batch(Hq=8, Hkv=2, hd=64, q_lens=[1, 5, 33, 0, 1], ctx_lens=[40, 3, 20, 9, 0], num_blocks=40, seed=5)
    full = ref_numpy.attn_mixed(b.q, b.k_cache, b.v_cache, b.block_tables, b.seq_lens, b.query_start_loc, b.ctx_lens)
    pairs = [(0, 0), (1, 0), (1, 4), (2, 0), (2, 15), (2, 16), (2, 32), (4, 0)]
    s = W.row_sample(b, pairs)
    assert (s.q_lens == 1).all() and s.num_blocks == 3 + 1 + 4 + 1
    got = ref_numpy.attn_mixed(s.q, s.k_cache, s.v_cache, s.block_tables, s.seq_lens, s.query_start_loc, s.ctx_lens)
    rows = [int(b.query_start_loc[q]) + t for q, t in pairs]
    assert (s.extra["rows"] == rows).all()
    np.testing.assert_allclose(got, full[rows], rtol=0, atol=1e-13)



# ----------------------------------------------------------------------------- KV append
def _step_kv(b):
    """K/V vectors ([T][Hkv][hd] bit patterns) of the step's tokens, read out of a filled host batch."""
    k_new = np.zeros((b.total_q, b.Hkv, b.hd), np.uint16)
    v_new = np.zeros_like(k_new)
    for i in range(b.num_seqs):
        k, v = W.gather_logical(b, i)
        q0, ql, c = int(b.query_start_loc[i]), int(b.q_lens[i]), int(b.ctx_lens[i])
        k_new[q0:q0 + ql] = k[c:c + ql]
        v_new[q0:q0 + ql] = v[c:c + ql]
    return k_new, v_new


def test_kv_append_offsets_of_a_hand_worked_example():
    # Hkv=1, hd=8, BS=16: one sequence with 17 cached tokens appends 2 tokens -> positions 17, 18 live in the
    # sequence's second block (id 5), slots 1 and 2.  K element d of slot s is word [blk][0][0][s][d] of the
    # K pool (flat offset blk*128 + s*8 + d); V element d of slot s is [blk][0][d][s] (flat blk*128 + d*16 + s).
    k_cache = np.zeros((8, 1, 1, 16, 8), np.uint16)
    v_cache = np.zeros((8, 1, 8, 16), np.uint16)
    k_new = (np.arange(16, dtype=np.uint16) + 100).reshape(2, 1, 8)
    v_new = (np.arange(16, dtype=np.uint16) + 200).reshape(2, 1, 8)
    ref_numpy.kv_append(k_new, v_new, k_cache, v_cache, np.array([[3, 5, -1]]), np.array([0, 2]), np.array([17]))
    kf, vf = k_cache.reshape(-1), v_cache.reshape(-1)
    expect_k = {5 * 128 + 1 * 8 + d: 100 + d for d in range(8)}
    expect_k.update({5 * 128 + 2 * 8 + d: 108 + d for d in range(8)})
    expect_v = {5 * 128 + d * 16 + 1: 200 + d for d in range(8)}
    expect_v.update({5 * 128 + d * 16 + 2: 208 + d for d in range(8)})
    assert {int(i): int(kf[i]) for i in np.flatnonzero(kf)} == expect_k
    assert {int(i): int(vf[i]) for i in np.flatnonzero(vf)} == expect_v


def test_kv_append_rebuilds_the_cache_and_touches_nothing_else():
    for seed, (Hq, Hkv, hd, ql, cx) in enumerate([(4, 1, 64, [1, 1, 5, 0, 40], [36, 15, 16, 7, 3]),
                                                  (8, 2, 128, [33, 1, 2], [0, 31, 47]),
                                                  (14, 2, 64, [16, 17], [16, 15])]):
        b = W.build_batch(Hq=Hq, Hkv=Hkv, hd=hd, q_lens=ql, ctx_lens=cx, num_blocks=24, seed=40 + seed)
        k_new, v_new = _step_kv(b)
        # wipe the slots of the step's tokens (and only those), then append: the pools must come back bit for bit
        k0, v0 = b.k_cache.copy(), b.v_cache.copy()
        hole_k, hole_v = b.k_cache.copy(), b.v_cache.copy()
        for i in range(b.num_seqs):
            for t in range(int(b.q_lens[i])):
                pos = int(b.ctx_lens[i]) + t
                blk, s = int(b.block_tables[i, pos // 16]), pos % 16
                hole_k[blk, :, :, s, :] = 0xDEAD
                hole_v[blk, :, :, s] = 0xDEAD
        assert (hole_k != k0).any()
        ref_numpy.kv_append(k_new, v_new, hole_k, hole_v, b.block_tables, b.query_start_loc, b.ctx_lens)
        assert (hole_k == k0).all() and (hole_v == v0).all()
        # attention over the rebuilt pools is the attention over the original ones
        o0 = ref_numpy.attn_mixed(b.q, k0, v0, b.block_tables, b.seq_lens, b.query_start_loc, b.ctx_lens)
        o1 = ref_numpy.attn_mixed(b.q, hole_k, hole_v, b.block_tables, b.seq_lens, b.query_start_loc, b.ctx_lens)
        assert (o0 == o1).all()


def test_kv_append_reads_back_through_the_independent_gather():
    # append distinctive vectors, read the sequence back with workloads.gather_logical (separate code)
    b = W.build_batch(Hq=4, Hkv=2, hd=64, q_lens=[3, 1], ctx_lens=[14, 0], num_blocks=8, seed=50)
    rng = np.random.default_rng(7)
    k_new = rng.integers(0, 65536, size=(4, 2, 64)).astype(np.uint16)
    v_new = rng.integers(0, 65536, size=(4, 2, 64)).astype(np.uint16)
    ref_numpy.kv_append(k_new, v_new, b.k_cache, b.v_cache, b.block_tables, b.query_start_loc, b.ctx_lens)
    k, v = W.gather_logical(b, 0)
    assert (k[14:17] == k_new[0:3]).all() and (v[14:17] == v_new[0:3]).all()
    k, v = W.gather_logical(b, 1)
    assert (k[0] == k_new[3]).all() and (v[0] == v_new[3]).all()


# ----------------------------------------------------------------------------- roofline latency model
from oracle import perf_model  # noqa: E402

PARAMS = dict(F_ap=1.0e15, F_ad=2.0e14, M_a=5.0e12, O_p=30e-6, O_d=20e-6)


def test_model_operator_counts_equal_hand_evaluated_table2_rows():
    path = os.path.join(os.path.dirname(__file__), "golden", "table2_attention.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) >= 5
    for Hq, Hkv, hd, Sq, Skv, flops, nbytes in (map(int, r) for r in rows):
        assert perf_model.attention_flops(Hq, hd, Sq, Skv) == flops
        assert perf_model.attention_bytes(Hq, Hkv, hd, Sq, Skv) == nbytes


def test_model_equation1_regimes_and_crossing():
    # decode operator, Hq 32 / Hkv 8 / hd 128: FLOPs = 16384*S, bytes = 4096*S + 16384: intensity < 4 FLOP/B,
    # far below F_ad/M_a = 40 -> memory-bound, time = bytes / M_a exactly
    r = perf_model.predict(PARAMS, 32, 8, 128, [1], [999])
    assert r["decode"] == (4096 * 1000 + 16384) / 5.0e12 and r["memory_bound"] == r["decode"] and r["compute_bound"] == 0
    assert r["latency"] == r["decode"] + 20e-6 and r["prefill"] == 0
    # prefill operator of c rows over c keys: FLOPs = 16384 c^2, bytes = 4096 c + 16384 c = 20480 c; compute-bound iff
    # 16384 c^2 / 1e15 >= 20480 c / 5e12, i.e. c >= 250
    lo = perf_model.predict(PARAMS, 32, 8, 128, [249], [0])
    hi = perf_model.predict(PARAMS, 32, 8, 128, [250], [0])
    assert lo["memory_bound"] > 0 and lo["compute_bound"] == 0 and lo["prefill"] == 20480 * 249 / 5.0e12
    assert hi["compute_bound"] > 0 and hi["memory_bound"] == 0 and hi["prefill"] == 16384 * 250 * 250 / 1.0e15
    assert math.isclose(hi["prefill"], 20480 * 250 / 5.0e12, rel_tol=1e-12)       # the two roofs meet at c = 250
    # a slower decode roof turns the same decode operator compute-bound
    slow = perf_model.predict({**PARAMS, "F_ad": 1.0e12}, 32, 8, 128, [1], [999])
    assert slow["decode"] == 16384 * 1000 / 1.0e12 and slow["compute_bound"] == slow["decode"]


def test_model_iteration_is_the_sum_of_operators_plus_overheads():
    ql, cx = [1, 512, 1, 0, 2048, 1], [4095, 100, 0, 7, 4096, 70000]
    whole = perf_model.predict(PARAMS, 64, 8, 128, ql, cx)
    parts = [perf_model.predict(PARAMS, 64, 8, 128, [q], [c]) for q, c in zip(ql, cx)]
    assert math.isclose(whole["prefill"], sum(p["prefill"] for p in parts), rel_tol=1e-14)
    assert math.isclose(whole["decode"], sum(p["decode"] for p in parts), rel_tol=1e-14)
    assert whole["overhead"] == 50e-6                                              # each kind of work once
    assert math.isclose(whole["latency"], whole["prefill"] + whole["decode"] + 50e-6, rel_tol=1e-14)
    assert parts[3]["latency"] == 0.0                                              # empty sequence: no operator
    assert perf_model.predict(PARAMS, 64, 8, 128, [1, 1], [10, 20])["overhead"] == 20e-6
    assert perf_model.predict(PARAMS, 64, 8, 128, [5], [10])["overhead"] == 30e-6
    # decode attention latency grows in proportion to the batch's total token count (Section 3.3.3)
    a = perf_model.predict(PARAMS, 32, 8, 128, [1] * 10, [1023] * 10)["decode"]
    b = perf_model.predict(PARAMS, 32, 8, 128, [1] * 20, [1023] * 20)["decode"]
    assert math.isclose(b, 2 * a, rel_tol=1e-14)


def test_model_causal_count_is_the_number_of_visible_pairs():
    # closed forms: c rows on an empty cache see 1 + 2 + ... + c keys; on ctx cached keys c*ctx more; decode unchanged
    assert perf_model.attention_flops_causal(32, 128, 512, 0) == 4 * 4096 * (512 * 513 // 2)
    assert perf_model.attention_flops_causal(32, 128, 512, 1000) == 4 * 4096 * (512 * 1000 + 512 * 513 // 2)
    assert perf_model.attention_flops_causal(32, 128, 1, 999) == perf_model.attention_flops(32, 128, 1, 1000)
    assert perf_model.attention_flops_causal(8, 64, 3, 2) == 4 * 512 * (3 + 4 + 5)
    a = perf_model.predict(PARAMS, 32, 8, 128, [2048, 1], [0, 500], causal=True)
    b = perf_model.predict(PARAMS, 32, 8, 128, [2048, 1], [0, 500], causal=False)
    assert a["decode"] == b["decode"] and a["bytes"] == b["bytes"]
    assert math.isclose(a["prefill"] / b["prefill"], (2049 / 2) / 2048, rel_tol=1e-12)   # both compute-bound
    # the accounting used by bench.py for MFMA utilisation counts the same pairs
    w = accounting.batch_work(32, 8, 128, 16, [2048, 501], [2048, 1])
    assert w["flops_causal"] == a["flops"]


# ----------------------------------------------------------------------------- Mix Decoding Selection (Algorithm 2)
from oracle import mix_select  # noqa: E402

MIXP = dict(F_ap=1e18, F_ad=1e18, M_a=4.096e9, O_p=0.0, O_d=10e-6)


def test_mix_selection_hand_worked_example():
    path = os.path.join(os.path.dirname(__file__), "golden", "mix_selection.txt")
    cases = [l.split() for l in open(path) if l.startswith("S_us")]
    assert len(cases) == 3
    for c in cases:
        S = float(c[1]) * 1e-6
        order = [int(x) for x in c[c.index("order") + 1:c.index("selected")]]
        want = [bool(int(x)) for x in c[c.index("selected") + 1:c.index("latency_us")]]
        lat = float(c[-1]) * 1e-6
        r = mix_select.mix_decoding_select(MIXP, 32, 8, 128, S, [100, 200], [50, 400, 30, 120, 60, 500], order)
        assert r["selected"] == want
        assert math.isclose(r["latency"], lat, rel_tol=1e-12)


def test_mix_selection_equal_lengths_closed_form():
    # every request costs (n + 4) us: with no online requests and no random looks the number admitted is
    # floor((S - 10 us) / (n + 4) us), capped by the number of candidates
    for n, S_us, cand in ((96, 1010.5, 20), (96, 1009.5, 20), (996, 5000.0, 3), (46, 9.0, 5), (46, 59.5, 5), (46, 60.5, 5)):
        r = mix_select.mix_decoding_select(MIXP, 32, 8, 128, S_us * 1e-6, [], [n] * cand, [])
        want = min(cand, int(math.floor((S_us - 10.0) / (n + 4)))) if S_us > 10.0 else 0        # (no value sits on a tie)
        assert sum(r["selected"]) == want, (n, S_us, cand)


def test_mix_selection_bounds_are_inclusive():
    """Algorithm 2 admits on L <= S in both phases: a bound that equals a predicted latency bit for bit admits
    that batch and nothing beyond it."""
    p = dict(F_ap=9e14, F_ad=2e14, M_a=6e12, O_p=1e-5, O_d=9e-6)
    L = lambda lens: mix_select.latency(p, 32, 8, 128, lens)
    on, off = [700, 1500], [900, 300, 5000, 1200, 650]
    # random phase: the first request looked at lands exactly on the bound
    r = mix_select.mix_decoding_select(p, 32, 8, 128, L(on + [off[2]]), on, off, [2])
    assert r["selected"] == [False, False, True, False, False] and r["latency"] == L(on + [off[2]])
    # sorted phase: the bound is the latency of the three shortest candidates
    S = L(on + [300, 650, 900])
    r = mix_select.mix_decoding_select(p, 32, 8, 128, S, on, off, [])
    assert r["selected"] == [True, True, False, False, True] and r["latency"] == S


def test_mix_selection_invariants_by_exhaustive_scan():
    rng = np.random.default_rng(8)
    p = dict(F_ap=9e14, F_ad=2e14, M_a=6e12, O_p=1e-5, O_d=9e-6)
    L = lambda lens: mix_select.latency(p, 32, 8, 128, lens)
    for trial in range(60):
        on = [int(x) for x in rng.integers(16, 4000, size=rng.integers(0, 4))]
        off = [int(x) for x in rng.integers(16, 30000, size=rng.integers(0, 12))]
        K = int(rng.integers(0, 6))
        order = [int(x) for x in rng.integers(0, max(1, len(off)), size=K)] if off else []
        S = float(rng.uniform(0.5, 3.0)) * L(on + off[: len(off) // 2 + 1])
        r = mix_select.mix_decoding_select(p, 32, 8, 128, S, on, off, order)
        sel = [i for i, s in enumerate(r["selected"]) if s]
        chosen = on + [off[i] for i in sel]
        assert math.isclose(r["latency"], L(chosen), rel_tol=1e-12)
        if L(on) <= S:
            assert r["latency"] <= S                                     # the bound holds whenever it can
        else:
            assert not sel                                               # best effort: online only
        # the random phase, replayed one look at a time
        b, looked, acc = list(on), set(), set()
        for i in order:
            if i in looked:
                continue
            looked.add(i)
            if L(b + [off[i]]) <= S:
                b.append(off[i])
                acc.add(i)
        assert {i for i in sel if i in looked} == acc and all(r["looked"][i] for i in looked)
        # the sorted phase: exactly the longest admissible prefix, found here by scanning every prefix
        rest = sorted((i for i in range(len(off)) if i not in looked), key=lambda i: (off[i], i))
        best = 0
        if L(b) < S:
            for m in range(1, len(rest) + 1):
                if L(b + [off[i] for i in rest[:m]]) <= S:
                    best = m
        assert [i for i in sel if i not in looked] == sorted(rest[:best])


# ---------------------------------------------------------------- migration decision and eviction rule
from oracle import migration  # noqa: E402


def golden_lines(name, tag):
    path = os.path.join(os.path.dirname(__file__), "golden", name)
    return [l.split() for l in open(path) if l.startswith(tag + " ")]


def test_migration_hand_worked_examples():
    B = [100, 200]
    prefs = golden_lines("migration.txt", "pref")
    assert len(prefs) == 8
    for c in prefs:
        S, inc, sat, cap, lo, hi = float(c[1]) * 1e-6, bool(int(c[2])), int(c[3]), int(c[4]), int(c[5]), int(c[6])
        r = migration.migration_preference(MIXP, 32, 8, 128, S, B, inc, sat, 16, cap, lo, hi)
        assert (r["branch"], -1 if r["pref"] is None else r["pref"]) == (c[8], int(c[9])), c
    sels = golden_lines("migration.txt", "select")
    assert len(sels) == 3
    for c in sels:
        lens = [int(x) for x in c[c.index(":") + 1:c.index("->")]]
        want = [int(x) for x in c[c.index("->") + 1:]]
        got = migration.migration_select(MIXP, 32, 8, 128, float(c[1]) * 1e-6, B, lens, int(c[2]), 16, 10 ** 6, int(c[3]))
        assert got == want, c
    evs = golden_lines("migration.txt", "evict")
    assert len(evs) == 4
    for c in evs:
        lens = [int(x) for x in c[c.index(":") + 1:c.index("->")]]
        want = [int(x) for x in c[c.index("->") + 1:]]
        r = migration.eviction_victims(lens, int(c[1]), 16, int(c[2]), int(c[3]))
        assert [int(r["enough"])] + r["victims"] == want, c


def test_migration_preference_closed_forms_in_the_memory_bound_regime():
    # k requests of length n0 cost 10 + k (n0 + 4) us; S is chosen off every tie
    for k, n0, S_us, sat in ((4, 96, 1000.5, 4), (4, 96, 1000.5, 3), (4, 96, 1000.5, 9), (1, 500, 9000.5, 40),
                             (6, 30, 400.5, 8), (3, 1000, 3100.5, 2)):
        room = S_us - (10 + k * (n0 + 4))
        r = migration.migration_preference(MIXP, 32, 8, 128, S_us * 1e-6, [n0] * k, True, sat, 16, 10 ** 9, 8, 3000)
        if room <= 0:
            assert r["pref"] is None
        elif k >= sat:
            want = min(3000, int(math.floor(room - 4)))
            assert (r["pref"], r["branch"]) == ((want, "saturated") if want >= 8 else (None, "none"))
        else:
            n = sat - k
            if n * (8 + 4) <= room:
                assert (r["pref"], r["branch"]) == (min(3000, int(math.floor(room / n - 4))), "reach")
            else:
                assert (r["pref"], r["branch"]) == (8, "shortest")


def test_migration_preference_is_the_maximum_by_direct_evaluation():
    # compute-bound decode operators too (small F_ad): the preferred length fits, the next one does not
    rng = np.random.default_rng(21)
    p = dict(F_ap=9e14, F_ad=3e12, M_a=6e12, O_p=1e-5, O_d=9e-6)
    L = lambda lens: mix_select.latency(p, 32, 8, 128, lens)
    seen = set()
    for trial in range(80):
        B = [int(x) for x in rng.integers(16, 3000, size=rng.integers(1, 7))]
        sat = int(rng.integers(1, 16))
        S = L(B) * float(rng.uniform(0.9, 1.5) if trial % 2 else rng.uniform(1.0, 2.5))
        cap = int(rng.integers(50, 1500))
        lo = 16 if trial % 3 else 1200
        r = migration.migration_preference(p, 32, 8, 128, S, B, True, sat, 16, cap, lo, 2048)
        seen.add(r["branch"])
        n = max(1, sat - len(B))
        if r["branch"] == "none":
            ok = L(B) < S and len(B) >= sat
            assert not ok or L(B + [lo]) > S or migration.u_mem(B + [lo], 16, cap) > 1
        elif r["branch"] == "shortest":
            assert r["pref"] == lo and L(B + [lo] * n) > S
        else:
            l = r["pref"]
            mem = (lambda x: migration.u_mem(B + [x], 16, cap) <= 1) if r["branch"] == "saturated" else (lambda x: True)
            assert L(B + [l] * n) <= S and mem(l)
            assert l == 2048 or L(B + [l + 1] * n) > S or not mem(l + 1)
    assert seen == {"none", "saturated", "reach", "shortest"}


def test_eviction_victims_against_every_subset():
    rng = np.random.default_rng(5)
    for trial in range(80):
        lens = [int(x) for x in rng.integers(1, 400, size=rng.integers(1, 9))]
        blk = [migration.blocks(n, 16) for n in lens]
        need = int(rng.integers(0, sum(blk) + 8))
        for compute_bound in (False, True):
            r = migration.eviction_victims(lens, need, 16, 10 if compute_bound else 3, 10)
            v = r["victims"]
            assert r["compute_bound"] == compute_bound and len(set(v)) == len(v)
            assert r["enough"] == (sum(blk) >= need)
            if not r["enough"]:
                assert sorted(v) == list(range(len(lens)))
                continue
            freed = sum(blk[i] for i in v)
            assert freed >= need
            assert all(freed - blk[i] < need for i in v)                      # nobody is evicted needlessly
            order = sorted(range(len(lens)), key=lambda i: (-lens[i], i) if compute_bound else (lens[i], i))
            k = next(k for k in range(len(lens) + 1) if sum(blk[i] for i in order[:k]) >= need)
            assert set(v) <= set(order[:k])                                   # only from the preferred end
            if compute_bound:                                                 # fewest victims of all feasible subsets
                best = min(bin(m).count("1") for m in range(1 << len(lens))
                           if sum(blk[i] for i in range(len(lens)) if m >> i & 1) >= need)
                assert len(v) == best

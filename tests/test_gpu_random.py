"""Seeded random batches through every entry point of the library: head shapes, numbers of sequences, the mix of
empty / decode / short-chunk / long-chunk sequences, prior contexts (a fifth of them empty), pool sizes, poison in
the unused cache slots and a random choice of planner options are all drawn per case.  Each case checks
  * ooco_attn_mixed against the float64 C oracle (the parity gates),
  * ooco_attn_mixed_static against ooco_attn_mixed with the same kernels (bit-identical),
  * ooco_kv_append and ooco_kv_block_copy against the numpy oracle (bit-exact)."""
import os

import numpy as np
import pytest
import torch

from oracle import ref_c, ref_numpy
from paper_2511_21862_amd import binding as B
from paper_2511_21862_amd import workloads as W

from gpu_util import assert_parity, device_meta, run_gpu, say

pytestmark = pytest.mark.gpu

SHAPES = [(32, 8, 128), (28, 4, 128), (8, 1, 128), (16, 16, 64), (8, 2, 64), (64, 8, 128), (4, 4, 128), (2, 1, 64)]
# options every batch may be run under (values inside the documented ranges; the planner ignores what does not apply)
OPTIONS = [{}, {}, {"prefill_split": 2}, {"prefill_split": 5}, {"prefill_sorted": 0}, {"prefill_sorted": 2}, {"overlap": 0},
           {"overlap": 2}, {"decode_nbi": 2}, {"decode_nbi": 4}, {"decode_segments": 3}, {"decode_segments": 10 ** 6},
           {"decode_tail_pct": 30, "decode_tail_blocks": 2}, {"mixed_lean": 2}, {"mixed_lean": 2, "overlap": 2},
           {"prefill_waves": 8}, {"mixed_fused": 1}, {"rotate_heads": 0}, {"decode_piece_pad": 5}, {"xcd_weights": sum(w << (8 * k) for k, w in enumerate([100, 60, 140, 95, 105, 85, 115, 100])), "decode_segments": 16}, {"decode_first": 0}]
bits = lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16)
N_CASES = int(os.environ.get("OOCO_RANDOM_CASES", "24"))      # set higher for a longer run (400 cases take 90 s)
FIRST = int(os.environ.get("OOCO_RANDOM_FIRST", "0"))         # first case number (other seeds for a longer run)
N_LARGER = int(os.environ.get("OOCO_RANDOM_LARGER", "6"))     # larger batches (a few seconds of oracle time each)
N_LONG = int(os.environ.get("OOCO_RANDOM_LONG", "10"))        # batches of long and short contexts


def draw(case):
    rng = np.random.default_rng(52000 + case)
    Hq, Hkv, hd = SHAPES[rng.integers(len(SHAPES))]
    n = int(rng.integers(1, 36))
    kinds = rng.choice(4, size=n, p=[0.1, 0.5, 0.3, 0.1])
    ql = np.where(kinds == 0, 0, np.where(kinds == 1, 1, np.where(kinds == 2, rng.integers(2, 70, size=n),
                                                                 rng.integers(70, 300, size=n)))).astype(np.int32)
    cx = np.where(rng.random(n) < 0.2, 0, (2.0 ** rng.uniform(0, 11, size=n)).astype(np.int64)).astype(np.int32)
    if ql.sum() == 0:
        ql[0] = 1
    nblk = int(((cx + ql + 15) // 16).sum()) + int(rng.integers(1, 30))
    opts = dict(OPTIONS[rng.integers(len(OPTIONS))])
    if hd != 128:      # the eight-wave prefill workgroups, the lean pair and the one-launch kernel are head_dim-128 paths
        for k in ("mixed_lean", "prefill_waves", "mixed_fused"):
            opts.pop(k, None)
    b = W.build_batch(Hq=Hq, Hkv=Hkv, hd=hd, q_lens=ql, ctx_lens=cx, num_blocks=nblk, seed=7000 + case, poison=True)
    return rng, b, opts


@pytest.mark.parametrize("case", range(FIRST, FIRST + N_CASES))
def test_random_batch_attention(case):
    rng, b, opts = draw(case)
    say(f"case: random {case}: {b.Hq}/{b.Hkv}/{b.hd} q_lens={b.q_lens.tolist()} ctx={b.ctx_lens.tolist()} options={opts}")
    ref = ref_c.attn_mixed(b.q, b.k_cache, b.v_cache, b.block_tables, b.seq_lens, b.query_start_loc, b.ctx_lens)
    assert_parity(run_gpu(b, options=opts), ref, f"random {case}")
    # the entry point that allocates nothing: the same kernels one after the other, tiles never split
    d = W.to_device(b)
    bt, sl, qsl, cl = device_meta(b)
    out = torch.full((b.total_q, b.Hq, b.hd), float("nan"), dtype=torch.bfloat16, device="cuda")
    B.ooco_attn_mixed_static(b.Hq, b.Hkv, b.hd, b.BS, b.max_blocks_per_seq, 0.0, b.seq_lens, b.query_start_loc, b.ctx_lens,
                             d.q, d.k_cache, d.v_cache, bt, sl, qsl, cl, out, b.num_seqs, b.total_q)
    torch.cuda.synchronize()
    want = run_gpu(b, options={"prefill_split": 1, "mixed_lean": 0})
    assert np.array_equal(bits(out), want), "the entry point that allocates nothing differs from ooco_attn_mixed"


@pytest.mark.parametrize("case", range(N_LARGER))
def test_random_larger_batch_attention(case):
    # batches that fill the GPU for more than one round of workgroups: up to 150 sequences, contexts up to 16K tokens,
    # chunks up to 700 rows (capped so that the oracle stays within a few seconds per case)
    rng = np.random.default_rng(53000 + case)
    Hq, Hkv, hd = [(32, 8, 128), (28, 4, 128), (64, 8, 128), (16, 2, 64)][case % 4]
    n = int(rng.integers(40, 150))
    kinds = rng.choice(3, size=n, p=[0.05, 0.85, 0.10])
    ql = np.where(kinds == 0, 0, np.where(kinds == 1, 1, rng.integers(16, 700, size=n))).astype(np.int64)
    cx = (2.0 ** rng.uniform(4, 14, size=n)).astype(np.int64)
    budget = 6.0e6 * 32 / Hq                                   # (row, key) pairs the oracle is given
    pairs = ql * cx + ql * (ql + 1) // 2
    while pairs.sum() > budget:                                # shorten the costliest chunk until the batch fits
        i = int(np.argmax(pairs))
        ql[i] = max(1, ql[i] // 2)
        pairs = ql * cx + ql * (ql + 1) // 2
    nblk = int(((cx + ql + 15) // 16).sum()) + 64
    opts = [{}, {"mixed_lean": 2}, {"overlap": 2}, {}, {"mixed_fused": 1}, {"prefill_split": 3}][case % 6]
    b = W.build_batch(Hq=Hq, Hkv=Hkv, hd=hd, q_lens=ql.astype(np.int32), ctx_lens=cx.astype(np.int32), num_blocks=nblk,
                      seed=7100 + case, poison=True)
    say(f"case: larger random {case}: {Hq}/{Hkv}/{hd}, {n} sequences, {int(ql.sum())} query rows in chunks of up to "
        f"{int(ql.max())}, {int(cx.sum())} cached tokens, options={opts}")
    ref = ref_c.attn_mixed(b.q, b.k_cache, b.v_cache, b.block_tables, b.seq_lens, b.query_start_loc, b.ctx_lens)
    assert_parity(run_gpu(b, options=opts), ref, f"larger random {case}")


@pytest.mark.parametrize("case", range(N_LONG))
def test_random_long_and_short_contexts(case):
    # one to three chunks on 4K-40K cached tokens among chunks on short contexts and decode sequences: the planner
    # cuts the long chunks' tiles into parts by their own number of steps (parts first in its list, whole tiles after)
    rng = np.random.default_rng(54000 + case)
    Hq, Hkv, hd = [(32, 8, 128), (28, 4, 128), (64, 8, 128), (8, 1, 128), (16, 2, 64)][case % 5]
    n_long, n_short, n_dec = int(rng.integers(1, 4)), int(rng.integers(0, 12)), int(rng.choice([0, 0, 3, 40]))
    ql = np.r_[rng.integers(8, 200, size=n_long), rng.integers(2, 400, size=n_short), np.ones(n_dec, np.int64)]
    cx = np.r_[(2.0 ** rng.uniform(12, 15.3, size=n_long)).astype(np.int64), rng.integers(0, 600, size=n_short),
               rng.integers(1, 3000, size=n_dec)]
    perm = rng.permutation(len(ql))
    ql, cx = ql[perm].astype(np.int32), cx[perm].astype(np.int32)
    nblk = int(((cx + ql + 15) // 16).sum()) + 32
    opts = [{}, {}, {"overlap": 2}, {"prefill_waves": 8}, {}, {"mixed_lean": 2}, {"prefill_sorted": 0}, {}, {"prefill_split": 7}, {}][case % 10]
    if hd != 128:
        opts = {k: v for k, v in opts.items() if k not in ("prefill_waves", "mixed_lean")}
    b = W.build_batch(Hq=Hq, Hkv=Hkv, hd=hd, q_lens=ql, ctx_lens=cx, num_blocks=nblk, seed=7200 + case, poison=True)
    plan = B.ooco_plan_dry_run(Hq, Hkv, hd, 16, b.max_blocks_per_seq, 256, 128 << 20, b.seq_lens, b.query_start_loc, b.ctx_lens,
                               prefill_split=opts.get("prefill_split", 0))
    say(f"case: long and short contexts {case}: {Hq}/{Hkv}/{hd} q_lens={ql.tolist()} ctx={cx.tolist()} options={opts}; "
        f"parts per tile {sorted(set(plan['prefill_tiles'][:, 4].tolist()))}")
    ref = ref_c.attn_mixed(b.q, b.k_cache, b.v_cache, b.block_tables, b.seq_lens, b.query_start_loc, b.ctx_lens)
    with B.Context(b.Hq, b.Hkv, b.hd, b.BS, b.num_blocks, b.max_blocks_per_seq) as ctx:
        first = run_gpu(b, ctx=ctx, options=opts)
        again = run_gpu(b, ctx=ctx)                 # (the arrival counters are back at zero)
    assert_parity(first, ref, f"long and short contexts {case}")
    assert np.array_equal(first, again)


@pytest.mark.parametrize("case", range(FIRST, FIRST + N_CASES))
def test_random_batch_append_and_copy(case):
    rng, b, _ = draw(case)
    say(f"case: random {case} append + copy: {b.Hq}/{b.Hkv}/{b.hd} q_lens={b.q_lens.tolist()} ctx={b.ctx_lens.tolist()}")
    T, nblk = b.total_q, b.num_blocks
    k_new = rng.integers(0, 65536, size=(T, b.Hkv, b.hd)).astype(np.uint16)      # any bit pattern: the copy is bit-exact
    v_new = rng.integers(0, 65536, size=(T, b.Hkv, b.hd)).astype(np.uint16)
    k_ref, v_ref = b.k_cache.copy(), b.v_cache.copy()
    ref_numpy.kv_append(k_new, v_new, k_ref, v_ref, b.block_tables, b.query_start_loc, b.ctx_lens)
    d = W.to_device(b)
    bt, sl, qsl, cl = device_meta(b)
    to_dev = lambda a: torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    with B.Context(b.Hq, b.Hkv, b.hd, b.BS, nblk, b.max_blocks_per_seq) as ctx:
        if rng.random() < 0.4:
            ctx.set_option("append_parts", int(rng.choice([1, 2, 4, 8])))
        ctx.kv_append(to_dev(k_new), to_dev(v_new), d.k_cache, d.v_cache, bt, qsl, cl)
        torch.cuda.synchronize()
        assert (bits(d.k_cache) == k_ref).all() and (bits(d.v_cache) == v_ref).all(), "append differs from the oracle"
        m = int(rng.integers(1, nblk + 1))
        src = rng.permutation(nblk)[:m].astype(np.int64)
        dst = rng.permutation(nblk)[:m].astype(np.int64)
        k2, v2 = torch.zeros_like(d.k_cache), torch.zeros_like(d.v_cache)
        if rng.random() < 0.5:
            ctx.set_option("copy_sort", int(rng.choice([0, 2])))
        ctx.kv_block_copy(d.k_cache, d.v_cache, k2, v2, torch.from_numpy(src).cuda(), torch.from_numpy(dst).cuda())
        torch.cuda.synchronize()
        kh, vh = np.zeros_like(k_ref), np.zeros_like(v_ref)
        ref_numpy.block_copy(k_ref, v_ref, kh, vh, src, dst)
        assert (bits(k2) == kh).all() and (bits(v2) == vh).all(), "block copy differs from the oracle"

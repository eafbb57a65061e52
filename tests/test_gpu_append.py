"""GPU parity of ooco_kv_append (through the C ABI) against the oracle: bit-exact pools."""
import numpy as np
import pytest
import torch

from oracle import ref_numpy
from paper_2511_21862_amd import binding as B
from paper_2511_21862_amd import workloads as W

from gpu_util import device_meta, run_gpu, say

pytestmark = pytest.mark.gpu

CASES = [
    # Hq, Hkv, hd, q_lens, ctx_lens
    (4, 1, 64, [1, 1, 5, 0, 40], [36, 15, 16, 7, 3]),          # decode rows, short chunk, chunk over 3 blocks
    (8, 2, 128, [33, 1, 2], [0, 31, 47]),                       # chunk from an empty cache, block-boundary decode
    (32, 8, 128, [1] * 9 + [128, 16], [5, 511, 512, 513, 15, 16, 17, 2047, 77, 333, 32]),
    (28, 4, 128, [17, 1, 16], [15, 64, 16]),                    # group of 7; chunk starting on the last slot
    (16, 1, 64, [0, 0, 3], [4, 0, 0]),                          # empty sequences first
]


def bits(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("case", range(len(CASES)))
def test_append_matches_oracle_bit_for_bit(case):
    Hq, Hkv, hd, ql, cx = CASES[case]
    need = int(sum((q + c + 15) // 16 for q, c in zip(ql, cx)))
    b = W.build_batch(Hq=Hq, Hkv=Hkv, hd=hd, q_lens=ql, ctx_lens=cx, num_blocks=need + 7, seed=60 + case)
    say(f"case: append {case}: Hkv={Hkv} hd={hd} q_lens={ql} ctx={cx}")
    rng = np.random.default_rng(case)
    T = b.total_q
    k_new = rng.integers(0, 65536, size=(T, Hkv, hd)).astype(np.uint16)
    v_new = rng.integers(0, 65536, size=(T, Hkv, hd)).astype(np.uint16)
    # oracle on host copies
    k_ref, v_ref = b.k_cache.copy(), b.v_cache.copy()
    ref_numpy.kv_append(k_new, v_new, k_ref, v_ref, b.block_tables, b.query_start_loc, b.ctx_lens)
    # GPU
    d = W.to_device(b)
    bt, sl, qsl, cl = device_meta(b)
    to_dev = lambda a: torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    with B.Context(Hq, Hkv, hd, b.BS, b.num_blocks, b.max_blocks_per_seq) as ctx:
        ctx.kv_append(to_dev(k_new), to_dev(v_new), d.k_cache, d.v_cache, bt, qsl, cl)
        torch.cuda.synchronize()
    assert (bits(d.k_cache) == k_ref).all(), "K pool differs"
    assert (bits(d.v_cache) == v_ref).all(), "V pool differs"
    changed = int((k_ref != b.k_cache).sum())
    say(f"  pools equal; {changed} K elements changed")


def test_append_then_attention_equals_attention_on_the_filled_cache():
    # the step as a serving loop runs it: the cache holds everything but this step's tokens (their slots
    # poisoned), append writes them, attention then sees the complete cache
    b = W.build_batch(Hq=32, Hkv=8, hd=128, q_lens=[1, 96, 1, 40, 1], ctx_lens=[700, 333, 64, 0, 15], num_blocks=120,
                      seed=66)
    say("case: append + attention")
    want = run_gpu(b)
    k_new = np.zeros((b.total_q, b.Hkv, b.hd), np.uint16)
    v_new = np.zeros_like(k_new)
    from dataclasses import replace
    hole = replace(b, k_cache=b.k_cache.copy(), v_cache=b.v_cache.copy())
    for i in range(b.num_seqs):
        k, v = W.gather_logical(b, i)
        q0, n, c = int(b.query_start_loc[i]), int(b.q_lens[i]), int(b.ctx_lens[i])
        k_new[q0:q0 + n], v_new[q0:q0 + n] = k[c:c + n], v[c:c + n]
        for t in range(n):
            blk, s = int(b.block_tables[i, (c + t) // 16]), (c + t) % 16
            hole.k_cache[blk, :, :, s, :] = 0x7FC0      # NaN
            hole.v_cache[blk, :, :, s] = 0x7FC0
    d = W.to_device(hole)
    bt, sl, qsl, cl = device_meta(b)
    to_dev = lambda a: torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    out = torch.empty((b.total_q, b.Hq, b.hd), dtype=torch.bfloat16, device="cuda")
    with B.Context(b.Hq, b.Hkv, b.hd, b.BS, b.num_blocks, b.max_blocks_per_seq) as ctx:
        ctx.plan(b.seq_lens, b.query_start_loc, b.ctx_lens)
        ctx.kv_append(to_dev(k_new), to_dev(v_new), d.k_cache, d.v_cache, bt, qsl, cl)
        ctx.attn_mixed(d.q, d.k_cache, d.v_cache, bt, sl, qsl, cl, out)
        torch.cuda.synchronize()
    assert (bits(out) == want).all()


def test_append_skips_rows_it_cannot_place():
    # a block id outside the pool and an empty batch: nothing is written, no error
    b = W.build_batch(Hq=4, Hkv=1, hd=64, q_lens=[1, 1], ctx_lens=[3, 20], num_blocks=6, seed=67)
    bt_bad = b.block_tables.copy()
    bt_bad[1, 1] = 10 ** 6
    d = W.to_device(b)
    k0 = bits(d.k_cache).copy()
    new = torch.ones((2, 1, 64), dtype=torch.bfloat16, device="cuda")
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    with B.Context(4, 1, 64, 16, b.num_blocks, b.max_blocks_per_seq) as ctx:
        ctx.kv_append(new, new, d.k_cache, d.v_cache, t(bt_bad), t(b.query_start_loc), t(b.ctx_lens))
        torch.cuda.synchronize()
        k1 = bits(d.k_cache)
        blk0 = int(b.block_tables[0, 0])
        assert (k1[blk0, :, :, 3, :] == 0x3F80).all()                      # sequence 0 was written
        mask = np.ones_like(k1, bool)
        mask[blk0, :, :, 3, :] = False
        assert (k1[mask] == k0[mask]).all()                                # nothing else changed
        B.ooco_kv_append(ctx.h, new, new, d.k_cache, d.v_cache, t(bt_bad), t(b.query_start_loc), t(b.ctx_lens), 0, 0)

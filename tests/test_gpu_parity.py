"""GPU parity: libooco (through the C ABI) against the float64 CPU oracle, element by element,
on seeded inputs.  Gates: max-abs <= 2e-2, mean-abs <= 2e-3, relative L2 <= 1e-2; block copy and
run-to-run determinism bit-exact."""
import os

import numpy as np
import pytest
import torch

from oracle import ref_c, ref_numpy
from paper_2511_21862_amd import binding as B
from paper_2511_21862_amd import workloads as W

from gpu_util import assert_parity, device_meta, run_gpu, say

pytestmark = pytest.mark.gpu


def oracle(b, fn=ref_c.attn_mixed, **kw):
    return fn(b.q, b.k_cache, b.v_cache, b.block_tables, b.seq_lens, b.query_start_loc, b.ctx_lens, **kw)


def test_config1_tiny_mixed_poisoned():
    b = W.config1(poison=True)
    say("case: config1 poisoned, numpy oracle")
    ref = oracle(b, ref_numpy.attn_mixed)
    assert_parity(run_gpu(b), ref, "config1")
    say("case: config1 without host plan")
    assert_parity(run_gpu(b, plan=False), ref, "config1 plan-less")


RAGGED = [
    # Hq, Hkv, hd, q_lens, ctx_lens
    (4, 1, 64, [1, 1, 1, 1], [0, 15, 16, 300]),
    (8, 2, 128, [1, 1, 1], [31, 32, 1000]),
    (32, 8, 128, [1] * 6, [5, 511, 512, 513, 2047, 77]),
    (64, 8, 128, [1, 1], [1500, 33]),
    (28, 4, 128, [1, 1, 7], [700, 64, 20]),                       # group of 7 (non power of two)
    (16, 1, 64, [1, 40], [129, 3]),                                # group of 16
    (4, 4, 64, [1, 33], [200, 0]),                                 # MHA
    (8, 2, 128, [2, 31, 32, 33, 65], [0, 5, 16, 100, 47]),         # ragged chunks, tiles with tails
    (32, 8, 128, [128, 1, 96, 1], [0, 400, 333, 64]),              # mixed
    (4, 1, 64, [0, 1, 0, 5], [4, 4, 0, 0]),                        # empty sequences inside the batch
]


@pytest.mark.parametrize("case", range(len(RAGGED)))
def test_ragged_cases(case):
    Hq, Hkv, hd, ql, ctx = RAGGED[case]
    nblk = int(sum((c + q + 15) // 16 for c, q in zip(ctx, ql))) + 7
    b = W.build_batch(Hq=Hq, Hkv=Hkv, hd=hd, q_lens=ql, ctx_lens=ctx, num_blocks=nblk, seed=1000 + case, poison=True)
    say(f"case: ragged {case}: Hq={Hq} Hkv={Hkv} hd={hd} q_lens={ql} ctx={ctx}")
    assert_parity(run_gpu(b), oracle(b), f"ragged {case}")


@pytest.mark.parametrize("segments,tail_pct,tail_blocks", [(1, 0, 8), (2, 0, 8), (7, 15, 2), (40, 0, 8), (10 ** 6, 0, 8),
                                                           (1, 50, 1), (3, 90, 4), (2, 30, 8)])
def test_forced_decode_run_layouts_agree(segments, tail_pct, tail_blocks):
    # (1, 0): no sequence split; 10**6: one wave per KV block; tail_pct > 0: part of the KV line is
    # fetched dynamically in runs of tail_blocks blocks
    b = W.build_batch(Hq=32, Hkv=8, hd=128, q_lens=[1, 1, 0, 1, 5], ctx_lens=[2000, 130, 7, 15, 40], num_blocks=170,
                      seed=77, poison=True)
    say(f"case: decode_segments {segments} tail {tail_pct}% x {tail_blocks}")
    ref = oracle(b)
    opts = {"decode_segments": segments, "decode_tail_pct": tail_pct, "decode_tail_blocks": tail_blocks}
    assert_parity(run_gpu(b, options=opts), ref, f"segments={segments} tail={tail_pct}%x{tail_blocks}")


@pytest.mark.parametrize("pad,segments,tail_pct", [(0, 0, 0), (1, 5, 0), (7, 40, 0), (64, 3, 0), (64, 10 ** 6, 0), (5, 6, 40)])
def test_piece_pad_values_agree(pad, segments, tail_pct):
    # the run cuts charge `pad` blocks for every piece a run starts; with 64 some runs hold no block at all
    b = W.build_batch(Hq=32, Hkv=8, hd=128, q_lens=[1, 1, 0, 1, 5, 1, 1], ctx_lens=[2000, 130, 7, 15, 40, 0, 300],
                      num_blocks=200, seed=78, poison=True)
    say(f"case: decode_piece_pad {pad}, decode_segments {segments}, tail {tail_pct}%")
    opts = {"decode_piece_pad": pad, "decode_segments": segments, "decode_tail_pct": tail_pct, "decode_tail_blocks": 2}
    assert_parity(run_gpu(b, options=opts), oracle(b), f"piece pad {pad} segments {segments}")


@pytest.mark.parametrize("Hkv,segments,tail_pct", [(8, 8, 0), (2, 16, 0), (4, 24, 10), (8, 0, 0), (8, 10 ** 6, 0)])
def test_xcd_weighted_decode_runs_agree(Hkv, segments, tail_pct):
    # static runs sized per XCD (run v on XCD v % 8, all kv heads of a run on one XCD)
    # (8, 16 and 24 runs are long enough for the weights to apply; the last two fall back to equal runs)
    b = W.build_batch(Hq=4 * Hkv, Hkv=Hkv, hd=128, q_lens=[1, 1, 0, 1, 5, 1], ctx_lens=[6000, 130, 7, 15, 40, 900],
                      num_blocks=520, seed=79, poison=True)
    weights = [100, 60, 140, 95, 105, 85, 115, 100]
    packed = sum(w << (8 * k) for k, w in enumerate(weights))
    say(f"case: xcd weights Hkv={Hkv} decode_segments {segments} tail {tail_pct}%")
    opts = {"decode_segments": segments, "decode_tail_pct": tail_pct, "decode_tail_blocks": 2, "xcd_weights": packed}
    assert_parity(run_gpu(b, options=opts), oracle(b), f"xcd weights Hkv={Hkv} segments={segments}")


@pytest.mark.parametrize("split", [0, 2, 3, 8, 16])
def test_prefill_tiles_split_along_the_context_agree(split):
    # each (tile, kv head) cut into `split` parts along its keys, partial results merged by the last part
    # (0 = the planner's own choice, which splits here: few tiles, long context)
    say(f"case: prefill_split {split}")
    b = W.build_batch(Hq=8, Hkv=2, hd=128, q_lens=[2, 31, 33, 65, 1, 200], ctx_lens=[0, 5, 100, 47, 300, 1500],
                      num_blocks=200, seed=83, poison=True)
    assert_parity(run_gpu(b, options={"prefill_split": split}), oracle(b), f"split {split}, ragged chunks")
    # MHA, small head dim: the 32 columns of a wave are 32 different rows, so a part can start beyond what
    # some of them see
    b = W.build_batch(Hq=4, Hkv=4, hd=64, q_lens=[100, 40], ctx_lens=[700, 3], num_blocks=80, seed=84, poison=True)
    assert_parity(run_gpu(b, options={"prefill_split": split}), oracle(b), f"split {split}, MHA hd 64")
    # twice on one context (counters are back at zero), bit-identical
    with B.Context(b.Hq, b.Hkv, b.hd, b.BS, b.num_blocks, b.max_blocks_per_seq) as ctx:
        first = run_gpu(b, ctx=ctx, options={"prefill_split": split})
        again = run_gpu(b, ctx=ctx)
        assert np.array_equal(first, again)


@pytest.mark.parametrize("opts", [{}, {"prefill_sorted": 0}, {"prefill_waves": 8}, {"prefill_sorted": 0, "prefill_split": 5},
                                  {"mixed_fused": 1, "mixed_dec_cus": 16}])
def test_chunks_on_long_and_short_contexts_split_by_their_own_steps(opts):
    # one chunk on a long context among chunks on short ones (and a few decode sequences): by default the long chunk's
    # tiles are cut into parts and the others stay whole; without the tile list every tile gets the same parts
    b = W.build_batch(Hq=32, Hkv=8, hd=128, q_lens=[96, 1, 128, 40, 1, 64], ctx_lens=[300, 900, 9000, 0, 64, 2500],
                      num_blocks=900, seed=87, poison=True)
    say(f"case: chunks on 0 .. 9000 cached tokens, {opts}")
    if not opts:
        plan = B.ooco_plan_dry_run(32, 8, 128, 16, b.max_blocks_per_seq, 256, 128 << 20, b.seq_lens, b.query_start_loc, b.ctx_lens)
        parts = dict(zip(plan["prefill_tiles"][:, 1].tolist(), plan["prefill_tiles"][:, 4].tolist()))
        assert max(parts.values()) > 2 and min(parts.values()) == 1
    ref = oracle(b)
    assert_parity(run_gpu(b, options=opts), ref, f"long and short contexts {opts}")
    # prefill chunks only, twice on one context: the counters are back at zero, the bits the same
    c = W.build_batch(Hq=28, Hkv=4, hd=128, q_lens=[96, 130, 40], ctx_lens=[300, 7000, 0], num_blocks=600, seed=88, poison=True)
    with B.Context(c.Hq, c.Hkv, c.hd, c.BS, c.num_blocks, c.max_blocks_per_seq) as ctx:
        first = run_gpu(c, ctx=ctx, options={k: v for k, v in opts.items() if not k.startswith("mixed")})
        again = run_gpu(c, ctx=ctx)
        assert np.array_equal(first, again)
    assert_parity(first, oracle(c), f"prefill-only, long and short contexts {opts}")


def test_binding_imported_before_torch_finds_the_gpu():
    # a fresh process that imports the binding first and torch after it: the binding brings torch's HIP runtime in
    # before the library's, so that the process holds one runtime and the context finds the device
    import subprocess
    import sys
    code = ("import paper_2511_21862_amd.binding as B, torch; ctx = B.Context(32, 8, 128, 16, 64, 8); ctx.close(); "
            "x = torch.zeros(4, device='cuda'); torch.cuda.synchronize(); print('context ok')")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    say("case: binding imported before torch, fresh process")
    res = subprocess.run([sys.executable, "-c", code], cwd=root, capture_output=True, text=True, timeout=300)
    assert res.returncode == 0 and "context ok" in res.stdout, res.stderr[-2000:]


def test_many_tiles_in_forced_parts_without_the_tile_list():
    # 66 tiles forced into 16 parts each: 1,056 (tile, part) entries do not fit the tile list, so every tile gets its
    # parts chunk by chunk -- 8,448 partial results (more than there are arrival counters, which count per tile here)
    # in a workspace of 1 GiB
    b = W.build_batch(Hq=32, Hkv=8, hd=128, q_lens=[1056, 1056], ctx_lens=[1100, 1100], num_blocks=300, seed=89, poison=True)
    plan = B.ooco_plan_dry_run(32, 8, 128, 16, b.max_blocks_per_seq, 256, 1 << 30, b.seq_lens, b.query_start_loc, b.ctx_lens,
                               prefill_split=16)
    assert len(plan["prefill_tiles"]) == 66 and plan["prefill_parts"] == 16
    say("case: 66 tiles in 16 forced parts each, no tile list")
    assert_parity(run_gpu(b, options={"prefill_split": 16}, workspace_bytes=1 << 30), oracle(b), "66 tiles x 16 parts")


@pytest.mark.parametrize("opts", [{}, {"prefill_sorted": 0}, {"prefill_sorted": 2}, {"prefill_split": 3}, {"prefill_waves": 8}, {"mixed_lean": 2},
                                  {"mixed_fused": 1}, {"overlap": 0}, {"overlap": 2}, {"overlap": 2, "mixed_lean": 2}],
                         ids=lambda o: "-".join(f"{k}{v}" for k, v in o.items()) or "default")
def test_tiles_of_several_chunks_interleave(opts):
    # few tiles: the plan lists them one by one, longest first across chunks (the tiles of the chunk on the long
    # context, then alternately the others'); same results whatever the order and the kernel
    say(f"case: several chunks, tile list, {opts}")
    b = W.build_batch(Hq=32, Hkv=8, hd=128, q_lens=[100, 1, 257, 1, 64, 33, 1, 2], ctx_lens=[900, 700, 10, 64, 411, 0, 2000, 77],
                      num_blocks=420, seed=85, poison=True)
    assert_parity(run_gpu(b, options=opts), oracle(b), f"several chunks {opts}")
    b = W.build_batch(Hq=8, Hkv=2, hd=64, q_lens=[70, 90, 1, 200], ctx_lens=[300, 0, 100, 150], num_blocks=90, seed=86, poison=True)
    assert_parity(run_gpu(b, options=opts), oracle(b), f"several chunks {opts}, head_dim 64")


def test_repeated_calls_reuse_counters_and_workspace():
    b = W.build_batch(Hq=8, Hkv=2, hd=128, q_lens=[1, 1, 1], ctx_lens=[700, 90, 300], num_blocks=80, seed=78)
    ref = oracle(b)
    say("case: repeated calls on one context")
    with B.Context(b.Hq, b.Hkv, b.hd, b.BS, b.num_blocks, b.max_blocks_per_seq) as ctx:
        first = run_gpu(b, ctx=ctx, options={"decode_segments": 9, "decode_tail_pct": 40, "decode_tail_blocks": 1})
        for seg in (9, 4, 9, 17):
            out = run_gpu(b, ctx=ctx, options={"decode_segments": seg})
            assert_parity(out, ref, f"repeat segments={seg}")
            if seg == 9:
                assert np.array_equal(out, first)


def test_batch_above_inline_plan_limit_uses_device_plan():
    n = 1100                                  # more sequences than fit the kernel-argument plan
    rng = np.random.default_rng(5)
    ql = np.where(np.arange(n) % 97 == 0, 3, 1).astype(np.int32)
    ctx_l = rng.integers(0, 40, size=n).astype(np.int32)
    b = W.build_batch(Hq=4, Hkv=1, hd=64, q_lens=ql, ctx_lens=ctx_l, num_blocks=3600, seed=79)
    say("case: 1100 sequences")
    assert_parity(run_gpu(b), oracle(b), "1100 sequences")


def test_extreme_shapes():
    # one sequence at the maximum table length (every decode run holds a piece of it: 96-part merge), next to
    # the smallest possible pieces of work
    b = W.build_batch(Hq=8, Hkv=1, hd=128, q_lens=[1, 1, 2, 1], ctx_lens=[131071, 0, 0, 15], num_blocks=8200, seed=80,
                      max_blocks_per_seq=8192)
    say("case: 131072-token decode sequence + one-token sequences + two-row chunk")
    assert_parity(run_gpu(b), oracle(b), "131072-token sequence")
    # widest GQA group with the small head dim, chunks that start and end inside blocks, long prior context
    b = W.build_batch(Hq=16, Hkv=1, hd=64, q_lens=[300, 1, 45], ctx_lens=[1003, 2500, 2], num_blocks=260, seed=81,
                      poison=True)
    say("case: group of 16, hd 64, ragged chunks on long context")
    assert_parity(run_gpu(b), oracle(b), "g16 hd64 chunks")
    # several thousand tiny sequences (device plan path, many waves with many pieces)
    n = 3000
    rng = np.random.default_rng(6)
    ql = np.where(np.arange(n) % 211 == 0, 2, 1).astype(np.int32)
    b = W.build_batch(Hq=8, Hkv=2, hd=128, q_lens=ql, ctx_lens=rng.integers(0, 33, size=n).astype(np.int32),
                      num_blocks=9100, seed=82)
    say("case: 3000 tiny sequences")
    assert_parity(run_gpu(b), oracle(b), "3000 tiny sequences")


def test_peaky_scores_give_order_one_outputs():
    # scores x8: softmax concentrates on few keys, outputs are O(1) and the relative gate bites
    b = W.build_batch(Hq=32, Hkv=8, hd=128, q_lens=[1, 1, 64], ctx_lens=[900, 3000, 500], num_blocks=300, seed=5,
                      poison=True)
    scale = 8.0 / np.sqrt(128.0)
    say("case: peaky scale")
    ref = oracle(b, scale=scale)
    e = assert_parity(run_gpu(b, scale=scale), ref, "peaky")
    assert np.abs(ref).mean() > 0.2


def test_small_value_data_passes_relative_gate():
    # N(0,1)/sqrt(128) data: outputs ~2e-3, an all-zero answer would pass the absolute gates
    b = W.build_batch(Hq=32, Hkv=8, hd=128, q_lens=[1, 1], ctx_lens=[2047, 700], num_blocks=200, seed=6,
                      value_std=1 / np.sqrt(128.0))
    say("case: small values")
    assert_parity(run_gpu(b), oracle(b), "small values")


def test_run_to_run_and_block_permutation_determinism():
    b = W.build_batch(Hq=32, Hkv=8, hd=128, q_lens=[1, 1, 48], ctx_lens=[3000, 100, 70], num_blocks=256, seed=8)
    say("case: determinism")
    o1 = run_gpu(b, options={"decode_segments": 12})
    o2 = run_gpu(b, options={"decode_segments": 12})
    assert np.array_equal(o1, o2)
    o3 = run_gpu(W.permute_blocks(b, 3), options={"decode_segments": 12})
    assert np.array_equal(o1, o3)


def test_block_copy_bit_exact_round_trip():
    b = W.build_batch(Hq=32, Hkv=8, hd=128, q_lens=[1, 1, 1], ctx_lens=[500, 90, 1300], num_blocks=300, seed=9)
    say("case: block copy")
    d = W.to_device(b)
    victims = [0, 2]
    src = W.victim_block_ids(b, victims)
    rng = np.random.default_rng(0)
    n = len(src)
    stage_blocks = n + 5
    dst = rng.permutation(stage_blocks)[:n].astype(np.int64)
    ks = torch.full((stage_blocks,) + tuple(d.k_cache.shape[1:]), -7.0, dtype=torch.bfloat16, device="cuda")
    vs = torch.full((stage_blocks,) + tuple(d.v_cache.shape[1:]), -7.0, dtype=torch.bfloat16, device="cuda")
    with B.Context(b.Hq, b.Hkv, b.hd, b.BS, b.num_blocks, b.max_blocks_per_seq) as ctx:
        ctx.kv_block_copy(d.k_cache, d.v_cache, ks, vs, torch.from_numpy(src).cuda(), torch.from_numpy(dst).cuda())
        torch.cuda.synchronize()
        # oracle copy on the host
        kh = np.full(ks.shape, W.f32_to_bf16_bits(np.float32([-7.0]))[0], np.uint16)
        vh = kh.reshape(-1)[: vs.numel()].reshape(vs.shape).copy()
        ref_c.block_copy(b.k_cache, b.v_cache, kh, vh, src, dst)
        assert np.array_equal(ks.view(torch.int16).cpu().numpy().view(np.uint16), kh)
        assert np.array_equal(vs.view(torch.int16).cpu().numpy().view(np.uint16), vh)
        # restore into fresh ids of the main pool and check attention is unchanged bit for bit
        before = run_gpu(b, ctx=ctx)
        used = set(int(x) for x in b.block_tables[b.block_tables >= 0])
        fresh = np.array([i for i in range(b.num_blocks) if i not in used][:n], np.int64)
        assert len(fresh) == n
        ctx.kv_block_copy(ks, vs, d.k_cache, d.v_cache, torch.from_numpy(dst).cuda(), torch.from_numpy(fresh).cuda())
        torch.cuda.synchronize()
        b2 = W.to_host(d)
        bt = b.block_tables.copy()
        pos = 0
        for s in victims:
            nb = (int(b.seq_lens[s]) + 15) // 16
            bt[s, :nb] = fresh[pos:pos + nb]
            pos += nb
        b2.block_tables = bt
        after = run_gpu(b2, ctx=ctx)
        assert np.array_equal(before, after)
        # zero pairs: no launch, no error
        ctx.kv_block_copy(ks, vs, d.k_cache, d.v_cache, torch.zeros(0, dtype=torch.int64, device="cuda"),
                          torch.zeros(0, dtype=torch.int64, device="cuda"))


@pytest.mark.parametrize("variant", [10, 11, 20, 21, 40, 41, 80, 81, 1041])
def test_block_copy_variants_are_bit_exact(variant):
    # option "copy_variant": 16-byte vectors per thread x 10 + (1 = non-temporal accesses); +1000 here = with the
    # pairs ordered by destination id on the device first (option "copy_sort", which large copies use by themselves)
    sort, variant = variant >= 1000, variant % 1000
    b = W.build_batch(Hq=32, Hkv=8, hd=128, q_lens=[1, 1], ctx_lens=[700, 45], num_blocks=80, seed=19)
    say(f"case: block copy variant {variant}, sorted {sort}")
    d = W.to_device(b)
    src = W.victim_block_ids(b, [0, 1])
    n = len(src)
    dst = np.random.default_rng(variant).permutation(n + 3)[:n].astype(np.int64)
    ks = torch.full((n + 3,) + tuple(d.k_cache.shape[1:]), 3.0, dtype=torch.bfloat16, device="cuda")
    vs = torch.full((n + 3,) + tuple(d.v_cache.shape[1:]), 3.0, dtype=torch.bfloat16, device="cuda")
    with B.Context(b.Hq, b.Hkv, b.hd, b.BS, b.num_blocks, b.max_blocks_per_seq) as ctx:
        ctx.set_option("copy_variant", variant)
        ctx.set_option("copy_sort", 2 if sort else 0)
        src_d, dst_d = torch.from_numpy(src).cuda(), torch.from_numpy(dst).cuda()
        ctx.kv_block_copy(d.k_cache, d.v_cache, ks, vs, src_d, dst_d)
        if sort:   # again with fewer pairs (the context's sort buffer is reused), same blocks, same result
            ctx.kv_block_copy(d.k_cache, d.v_cache, ks, vs, src_d[: n // 2], dst_d[: n // 2])
        torch.cuda.synchronize()
        assert torch.equal(src_d.cpu(), torch.from_numpy(src)) and torch.equal(dst_d.cpu(), torch.from_numpy(dst))   # the caller's lists are not touched
    kh = np.full(ks.shape, W.f32_to_bf16_bits(np.float32([3.0]))[0], np.uint16)
    vh = kh.reshape(-1)[: vs.numel()].reshape(vs.shape).copy()
    ref_c.block_copy(b.k_cache, b.v_cache, kh, vh, src, dst)
    assert np.array_equal(ks.view(torch.int16).cpu().numpy().view(np.uint16), kh)
    assert np.array_equal(vs.view(torch.int16).cpu().numpy().view(np.uint16), vh)


@pytest.mark.parametrize("opts", [{"decode_nbi": 1}, {"decode_nbi": 2}, {"decode_nbi": 4}, {"rotate_heads": 0}, {"decode_first": 0}, {"prefill_sorted": 0}, {"prefill_sorted": 2},
                                  {"overlap": 0}, {"overlap": 2}, {"overlap": 2, "decode_first": 0}, {"overlap": 2, "mixed_lean": 2}, {"mixed_lean": 2}, {"mixed_lean": 2, "prefill_split": 2}, {"mixed_lean": 2, "decode_segments": 5}, {"mixed_lean": 0}, {"prefill_waves": 8}, {"prefill_waves": 8, "prefill_split": 3}, {"prefill_waves": 4}, {"mixed_fused": 1}, {"mixed_fused": 1, "mixed_dec_cus": 1},
                                  {"mixed_fused": 1, "mixed_dec_cus": 31}, {"mixed_fused": 1, "mixed_dec_cus": 16, "prefill_split": 3}, {"decode_nbi": 2, "decode_segments": 9, "decode_tail_pct": 20,
                                                   "decode_tail_blocks": 3}],
                         ids=lambda o: "-".join(f"{k}{v}" for k, v in o.items()))
def test_tuning_knobs_agree(opts):
    # the knobs kept for experiments select other kernel instantiations or launch orders: same results
    b = W.build_batch(Hq=32, Hkv=8, hd=128, q_lens=[1, 1, 70, 1, 1, 0, 1], ctx_lens=[1500, 31, 200, 0, 16, 9, 333],
                      num_blocks=160, seed=91, poison=True)
    say(f"case: knobs {opts}")
    assert_parity(run_gpu(b, options=opts), oracle(b), f"knobs {opts}")
    b64 = W.build_batch(Hq=8, Hkv=2, hd=64, q_lens=[1, 1, 1], ctx_lens=[900, 17, 64], num_blocks=70, seed=92, poison=True)
    assert_parity(run_gpu(b64, options=opts), oracle(b64), f"knobs {opts}, head_dim 64")


def test_errors_surface_through_the_abi():
    b = W.config1()
    d = W.to_device(b)
    bt, sl, qsl, cl = device_meta(b)
    out = torch.empty((b.total_q, b.Hq, b.hd), dtype=torch.bfloat16, device="cuda")
    with B.Context(b.Hq, b.Hkv, b.hd, b.BS, b.num_blocks, b.max_blocks_per_seq) as ctx:
        with pytest.raises(B.OocoError) as e:
            B.ooco_attn_mixed(ctx.h, None, d.k_cache, d.v_cache, bt, sl, qsl, cl, out, b.num_seqs, b.total_q)
        assert e.value.status == B.OOCO_EINVAL
        ctx.plan(b.seq_lens, b.query_start_loc, b.ctx_lens)
        with pytest.raises(B.OocoError) as e:
            B.ooco_attn_mixed(ctx.h, d.q, d.k_cache, d.v_cache, bt, sl, qsl, cl, out, b.num_seqs - 1, b.total_q)
        assert e.value.status == B.OOCO_ESHAPE
        with pytest.raises(B.OocoError):
            ctx.set_option("no_such_option", 1)
        for bad in (5, 42, 90):   # block-copy variants that no kernel instantiation stands behind
            with pytest.raises(B.OocoError) as e:
                ctx.set_option("copy_variant", bad)
            assert e.value.status == B.OOCO_EINVAL
        B.ooco_attn_mixed(ctx.h, d.q, d.k_cache, d.v_cache, bt, sl, qsl, cl, out, 0, 0)     # empty: OK


def test_profiled_calls_keep_the_overlap_and_the_results():
    # option "profile" brackets every kernel with events on the stream it runs on: same launch order, same
    # streams, same output bits; the whole-call time covers both kernels
    b = W.build_batch(Hq=32, Hkv=8, hd=128, q_lens=[1, 300, 1, 1, 1], ctx_lens=[2500, 900, 64, 4000, 700],
                      num_blocks=700, seed=93, poison=True)
    say("case: profiled mixed calls")
    d = W.to_device(b)
    bt, sl, qsl, cl = device_meta(b)
    out = torch.empty((b.total_q, b.Hq, b.hd), dtype=torch.bfloat16, device="cuda")
    with B.Context(b.Hq, b.Hkv, b.hd, b.BS, b.num_blocks, b.max_blocks_per_seq) as ctx:
        ctx.set_option("plan_persistent", 1)
        ctx.set_option("overlap", 2)             # (a batch this short would otherwise run its kernels in sequence)
        ctx.plan(b.seq_lens, b.query_start_loc, b.ctx_lens)
        ctx.attn_mixed(d.q, d.k_cache, d.v_cache, bt, sl, qsl, cl, out)
        torch.cuda.synchronize()
        plain = out.clone()
        ctx.set_option("profile", 1)
        for _ in range(5):
            out.zero_()
            ctx.attn_mixed(d.q, d.k_cache, d.v_cache, bt, sl, qsl, cl, out)
        r = ctx.profile_read_calls()
        ctx.set_option("profile", 0)
        torch.cuda.synchronize()
    assert r["calls"] == 5 and r["per_call"].shape == (5, 3)
    pc = r["per_call"]
    say(f"  per call (prefill, decode, whole call) ms: {pc.tolist()}")
    assert (pc > 0).all()
    # the two kernels lie inside the call; they overlap, so the call is shorter than their sum would need
    assert (pc[:, 2] >= pc[:, :2].max(axis=1) * 0.9).all()
    assert torch.equal(out.view(torch.int16), plain.view(torch.int16))
    assert_parity(out.view(torch.int16).cpu().numpy().view(np.uint16), oracle(b), "profiled mixed call")


def test_a_plan_serves_one_call_only():
    # decode loop: the caller plans once and then advances the lengths on the device only.  The plan is used up by
    # its call, so the later calls plan by themselves from the device arrays and see every new token, also when a
    # sequence crosses a block boundary.
    base = np.array([15, 31, 700, 1024], np.int32)
    say("case: plan used up by its call, lengths advance on the device")
    with B.Context(32, 8, 128, 16, 200, 80) as ctx:
        full = W.build_batch(Hq=32, Hkv=8, hd=128, q_lens=[1, 1, 1, 1], ctx_lens=base + 2, num_blocks=200, seed=95,
                             max_blocks_per_seq=80)
        for step in range(3):
            # the same pools and tables, lengths one token longer every step
            b = W.Batch(Hq=32, Hkv=8, hd=128, BS=16, num_blocks=200, block_tables=full.block_tables,
                        seq_lens=base + 1 + step, ctx_lens=base + step, query_start_loc=full.query_start_loc, q=full.q,
                        k_cache=full.k_cache, v_cache=full.v_cache)
            if step == 0:
                ctx.plan(b.seq_lens, b.query_start_loc, b.ctx_lens)
            got = run_gpu(b, plan=False, ctx=ctx)
            assert_parity(got, oracle(b), f"decode step {step}")

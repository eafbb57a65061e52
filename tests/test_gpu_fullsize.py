"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration
bench.py times (default plan, default options, device-resident pools): EVERY query row of
configurations 2-5 is checked against the float64 C oracle (the sequences travel to the host in
groups), plus properties that hold at any size."""
import numpy as np
import pytest
import torch

from oracle import ref_c
from paper_2511_21862_amd import binding as B
from paper_2511_21862_amd import workloads as W

from gpu_util import assert_parity, device_meta, say

pytestmark = pytest.mark.gpu


def run_device_batch(b, options=None):
    """One ooco_plan + ooco_attn_mixed on a batch whose pools already live on the GPU."""
    bt, sl, qsl, cl = device_meta(b)
    out = torch.full((b.total_q, b.Hq, b.hd), float("nan"), dtype=torch.bfloat16, device="cuda")
    with B.Context(b.Hq, b.Hkv, b.hd, b.BS, b.num_blocks, b.max_blocks_per_seq) as ctx:
        for k, v in (options or {}).items():
            ctx.set_option(k, v)
        ctx.plan(b.seq_lens, b.query_start_loc, b.ctx_lens)
        info = ctx.plan_info()
        ctx.attn_mixed(b.q, b.k_cache, b.v_cache, bt, sl, qsl, cl, out)
        torch.cuda.synchronize()
    return out, info


def oracle_all_rows(b, kv_tokens_per_batch=600_000):
    """The float64 C oracle on EVERY query row of a device-resident batch: the sequences go to the host in groups
    (workloads.subset: a compact copy of their blocks) of at most `kv_tokens_per_batch` KV tokens, so that host
    memory stays bounded; returns float64 [total_q, Hq, hd]."""
    ref = np.full((b.total_q, b.Hq, b.hd), np.nan, dtype=np.float64)
    order = [int(i) for i in np.flatnonzero(b.q_lens > 0)]
    group, tokens, n_groups = [], 0, 0
    def flush():
        nonlocal group, tokens, n_groups
        if not group:
            return
        s = W.subset(b, group)
        r = ref_c.attn_mixed(s.q, s.k_cache, s.v_cache, s.block_tables, s.seq_lens, s.query_start_loc, s.ctx_lens)
        ref[s.extra["rows"]] = r
        n_groups += 1
        group, tokens = [], 0
    for i in order:
        if group and tokens + int(b.seq_lens[i]) > kv_tokens_per_batch:
            flush()
        group.append(i)
        tokens += int(b.seq_lens[i])
    flush()
    assert not np.isnan(ref).any()
    return ref, n_groups


def worst_rows(got_bits, ref, b):
    """(row, sequence, max-abs error) of the worst query row, and the worst per-row relative L2 error."""
    g = W.bf16_bits_to_f32(got_bits).astype(np.float64)
    d = np.abs(g - ref).reshape(ref.shape[0], -1)
    row_max = d.max(axis=1)
    row_rel = np.sqrt((d ** 2).sum(axis=1)) / np.maximum(np.sqrt((ref.reshape(ref.shape[0], -1) ** 2).sum(axis=1)), 1e-30)
    r = int(row_max.argmax())
    seq = int(np.searchsorted(b.query_start_loc, r, side="right") - 1)
    return dict(row=r, seq=seq, seq_len=int(b.seq_lens[seq]), max_abs=float(row_max[r]), worst_row_rel_l2=float(row_rel.max()),
                worst_rel_row=int(row_rel.argmax()))


CASES = ["config2", "config3", "config4", "config5"]


@pytest.mark.parametrize("name", CASES)
def test_full_size_every_row(name):
    b = getattr(W, name)(device="cuda")
    say(f"case: {name} full size: {b.num_seqs} sequences, {b.total_q} query tokens, pool {b.num_blocks} blocks")
    out, info = run_device_batch(b)
    say(f"  plan: {info}")
    assert bool(torch.isfinite(out.float()).all()), f"{name}: non-finite or unwritten output"
    ref, n_groups = oracle_all_rows(b)
    say(f"  oracle on all {b.total_q} rows ({int(b.seq_lens[b.q_lens > 0].sum())} KV tokens) in {n_groups} groups")
    got = out.view(torch.int16).cpu().numpy().view(np.uint16)
    assert_parity(got, ref, f"{name}, every row")
    w = worst_rows(got, ref, b)
    say(f"  worst row: {w}")
    # no single row hides behind the batch-wide averages: each row alone is within the absolute gate, and within a
    # relative error that bf16 rounding of output and weights explains
    assert w["max_abs"] <= 2e-2 and w["worst_row_rel_l2"] <= 2.5e-2
    # a second call with the dynamic tail and other run counts changes nothing beyond rounding: every row again
    out2, _ = run_device_batch(b, options={"decode_segments": 64, "decode_tail_pct": 10})
    got2 = out2.view(torch.int16).cpu().numpy().view(np.uint16)
    assert_parity(got2, ref, f"{name}, every row, other run layout")
    say(f"  worst row, other run layout: {worst_rows(got2, ref, b)}")


def test_config4_preemption_sequence():
    """Config 4 with its one preemption: attention over 512 sequences; the KV blocks of the 64 victims are
    copied to a staging pool; attention over the remaining 448; the victims come back into fresh physical
    blocks; attention over all 512 again.  The first and last step see the same logical batch under the
    same plan, so their outputs must agree bit for bit (paging invariance through the block copy)."""
    b = W.config4(device="cuda")
    victims = np.asarray(b.extra["victims"])
    keep = np.setdiff1d(np.arange(b.num_seqs), victims)
    src = W.victim_block_ids(b, victims)
    n = len(src)
    say(f"case: config4 preemption: {len(victims)} victims, {n} blocks")
    free, pos = b.extra["free_list"], int(b.extra["free_pos"])
    assert pos + n <= len(free)
    fresh = free[pos:pos + n].astype(np.int64)
    k_st = torch.empty((n,) + tuple(b.k_cache.shape[1:]), dtype=torch.bfloat16, device="cuda")
    v_st = torch.empty((n,) + tuple(b.v_cache.shape[1:]), dtype=torch.bfloat16, device="cuda")
    src_d, stage_d, fresh_d = (torch.from_numpy(x).cuda() for x in (src, np.arange(n, dtype=np.int64), fresh))

    out1, _ = run_device_batch(b)
    with B.Context(b.Hq, b.Hkv, b.hd, b.BS, b.num_blocks, b.max_blocks_per_seq) as ctx:
        ctx.kv_block_copy(b.k_cache, b.v_cache, k_st, v_st, src_d, stage_d)           # eviction
        torch.cuda.synchronize()
        assert torch.equal(k_st, b.k_cache.index_select(0, src_d)) and torch.equal(v_st, b.v_cache.index_select(0, src_d))
        # the victims' old blocks are now free: overwrite them, nothing that remains may depend on them
        b.k_cache.index_fill_(0, src_d, float("nan"))
        b.v_cache.index_fill_(0, src_d, float("nan"))
        # step on the remaining sequences
        ql = b.q_lens[keep]
        qsl = np.zeros(len(keep) + 1, np.int32)
        qsl[1:] = np.cumsum(ql)
        rest = W.Batch(Hq=b.Hq, Hkv=b.Hkv, hd=b.hd, BS=b.BS, num_blocks=b.num_blocks,
                       block_tables=b.block_tables[keep], seq_lens=b.seq_lens[keep], ctx_lens=b.ctx_lens[keep],
                       query_start_loc=qsl, q=b.q.index_select(0, torch.from_numpy(b.query_start_loc[keep].astype(np.int64)).cuda()),
                       k_cache=b.k_cache, v_cache=b.v_cache, name="cfg4 minus victims")
        out2, _ = run_device_batch(rest)
        ref_rows = out1.index_select(0, torch.from_numpy(b.query_start_loc[keep].astype(np.int64)).cuda())
        d = (out2.float() - ref_rows.float()).abs()
        say(f"  remaining 448 vs first step: max diff {float(d.max()):.3g}")
        assert bool(torch.isfinite(out2.float()).all()) and float(d.max()) <= 2e-2
        # restore into fresh blocks, tables updated
        ctx.kv_block_copy(k_st, v_st, b.k_cache, b.v_cache, stage_d, fresh_d)
        torch.cuda.synchronize()
    bt = b.block_tables.copy()
    nb = (b.seq_lens + b.BS - 1) // b.BS
    p = 0
    for s in victims:
        bt[s, : nb[s]] = fresh[p:p + nb[s]]
        p += int(nb[s])
    from dataclasses import replace
    out3, _ = run_device_batch(replace(b, block_tables=bt))
    same = torch.equal(out3.view(torch.int16), out1.view(torch.int16))
    say(f"  after restore: bit-identical to the first step: {same}")
    assert same

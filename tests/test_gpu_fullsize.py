"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration
bench.py times (default plan, default options, device-resident pools): sampled query rows are
checked one by one against the float64 C oracle (a chunk row is a single-query decode over its
visible keys, see workloads.row_sample), plus properties that hold at any size."""
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


def sampled_pairs(b, rng, n_decode, rows_per_chunk):
    """(sequence, row) pairs: the longest and shortest decode sequences plus random ones; for every
    chunk its first and last rows, the rows around the query-tile boundaries and random rows."""
    ql = b.q_lens
    dec = np.flatnonzero(ql == 1)
    pairs = []
    if len(dec):
        order = dec[np.argsort(b.seq_lens[dec], kind="stable")]
        pick = {int(order[0]), int(order[-1])}
        pick.update(int(x) for x in rng.choice(dec, size=min(n_decode, len(dec)), replace=False))
        pairs += [(s, 0) for s in sorted(pick)]
    tile_rows = max(1, 128 // (b.Hq // b.Hkv))
    for s in np.flatnonzero(ql > 1):
        n = int(ql[s])
        rows = {0, 1, n - 1, n - 2}
        for t in (tile_rows, (n // tile_rows // 2) * tile_rows, ((n - 1) // tile_rows) * tile_rows):
            rows.update((t - 1, t, t + 1))
        rows.update(int(x) for x in rng.integers(0, n, size=rows_per_chunk))
        pairs += [(int(s), t) for t in sorted(r for r in rows if 0 <= r < n)]
    return pairs


CASES = [
    # name, n_decode samples, random rows per chunk
    ("config2", 64, 0),
    ("config3", 24, 24),
    ("config4", 24, 0),
    ("config5", 4, 16),
]


@pytest.mark.parametrize("name,n_decode,rows_per_chunk", CASES)
def test_full_size_sampled_rows(name, n_decode, rows_per_chunk):
    b = getattr(W, name)(device="cuda")
    say(f"case: {name} full size: {b.num_seqs} sequences, {b.total_q} query tokens, pool {b.num_blocks} blocks")
    out, info = run_device_batch(b)
    say(f"  plan: {info}")
    # property at any size: every output element was written and is finite
    assert bool(torch.isfinite(out.float()).all()), f"{name}: non-finite or unwritten output"
    pairs = sampled_pairs(b, np.random.default_rng(1234), n_decode, rows_per_chunk)
    s = W.row_sample(b, pairs)
    say(f"  oracle on {len(pairs)} sampled rows ({int(s.seq_lens.sum())} keys)")
    ref = ref_c.attn_mixed(s.q, s.k_cache, s.v_cache, s.block_tables, s.seq_lens, s.query_start_loc, s.ctx_lens)
    rows = torch.from_numpy(s.extra["rows"]).cuda()
    got = out.index_select(0, rows).view(torch.int16).cpu().numpy().view(np.uint16)
    assert_parity(got, ref, f"{name} sampled")
    # property at any size: a second call with the dynamic tail and other run counts changes nothing
    # beyond rounding (the same rows still pass the gate)
    out2, _ = run_device_batch(b, options={"decode_segments": 64, "decode_tail_pct": 10})
    got2 = out2.index_select(0, rows).view(torch.int16).cpu().numpy().view(np.uint16)
    assert_parity(got2, ref, f"{name} sampled, other run layout")


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

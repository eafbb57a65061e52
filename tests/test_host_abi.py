"""Host-side checks that need no GPU: the library loads, exports every declared symbol, and the
planner validates lengths and covers every KV block / query row exactly once."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2511_21862_amd import binding as B
from paper_2511_21862_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "ooco.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ooco_[a-z_]+)\s*\(", text)))


# The comparisons of the host functions with their oracles need no GPU; they run in the CPU suite and, under the
# second parameter, once more in the GPU suite, so that the record of the GPU run shows them against the library
# that runs there.
BOTH_RECORDS = pytest.mark.parametrize("record", ["cpu", pytest.param("gpu-box", marks=pytest.mark.gpu)])


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(B.LIB_PATH)
    names = declared_symbols()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_ctx_create_rejects_bad_geometry_before_touching_a_device():
    bad = [
        dict(num_q_heads=32, num_kv_heads=7), dict(num_q_heads=0), dict(num_q_heads=64, num_kv_heads=2),
        dict(head_dim=96), dict(block_size=32), dict(num_blocks=0), dict(max_blocks_per_seq=0),
    ]
    base = dict(num_q_heads=32, num_kv_heads=8, head_dim=128, block_size=16, num_blocks=64, max_blocks_per_seq=8)
    for kw in bad:
        with pytest.raises(B.OocoError) as e:
            B.ooco_ctx_create(**{**base, **kw})
        assert e.value.status in (B.OOCO_ESHAPE, B.OOCO_EINVAL)
        assert "ooco_ctx_create" in e.value.message


def dry(seq, qsl, ctx, **kw):
    args = dict(num_q_heads=32, num_kv_heads=8, head_dim=128, block_size=16, max_blocks_per_seq=8192, num_cus=256,
                workspace_bytes=128 << 20)
    args.update(kw)
    return B.ooco_plan_dry_run(h_seq_lens=seq, h_query_start_loc=qsl, h_ctx_lens=ctx, **args)


@pytest.mark.parametrize("seq,qsl,ctx,frag", [
    ([10, 5], [1, 2, 3], [9, 4], "query_start_loc[0]"),
    ([10, 5], [0, 2, 1], [8, 6], "decreases"),
    ([10, 5], [0, 1, 2], [9, 3], "!= seq_len"),
    ([10, -1], [0, 1, 1], [9, -1], "negative"),
    ([10, 16 * 8192 + 1], [0, 1, 2], [9, 16 * 8192], "max_blocks_per_seq"),
])
def test_plan_rejects_inconsistent_lengths(seq, qsl, ctx, frag):
    with pytest.raises(B.OocoError) as e:
        dry(seq, qsl, ctx)
    assert e.value.status == B.OOCO_ESHAPE and frag in e.value.message


def check_cover(b, plan):
    """Every KV block of every decode sequence is in exactly one piece, every query row of every
    chunk in exactly one tile; pieces needing a merge have distinct slots."""
    d, p = plan["decode_pieces"], plan["prefill_tiles"]
    nb = (b.seq_lens.astype(np.int64) + 15) // 16
    ql = b.q_lens
    for i in range(b.num_seqs):
        rows = d[d[:, 0] == i]
        if ql[i] == 1:
            rows = rows[np.argsort(rows[:, 1])]
            assert rows[0, 1] == 0 and rows[-1, 2] == nb[i]
            assert (rows[1:, 1] == rows[:-1, 2]).all() and (rows[:, 2] > rows[:, 1]).all()
            if len(rows) > 1:
                assert (rows[:, 3] == rows[:, 4] + i).all()          # slot = run + seq
                assert (np.diff(rows[:, 4]) == 1).all()              # consecutive runs
            else:
                assert rows[0, 3] == -1
        else:
            assert len(rows) == 0
        t = p[p[:, 0] == i]
        if ql[i] > 1:
            t = t[np.argsort(t[:, 1])]
            assert t[0, 1] == b.query_start_loc[i] and (t[:, 2].sum() == ql[i])
            assert (t[1:, 1] == t[:-1, 1] + t[:-1, 2]).all()
            assert (t[:, 3] == b.ctx_lens[i] + (t[:, 1] - b.query_start_loc[i])).all()
        else:
            assert len(t) == 0
    slots = d[d[:, 3] >= 0][:, 3]
    assert len(np.unique(slots)) == len(slots)
    assert len(slots) == 0 or slots.max() < plan["slots"]


def meta_only(fn, **kw):
    """Lengths of a configuration without materialising its multi-GiB pools."""
    import unittest.mock as m

    def fake(**a):
        ql = np.asarray(a["q_lens"], np.int32)
        cx = np.asarray(a["ctx_lens"], np.int32)
        qsl = np.zeros(len(ql) + 1, np.int32)
        qsl[1:] = np.cumsum(ql)
        return W.Batch(Hq=a["Hq"], Hkv=a["Hkv"], hd=a["hd"], BS=16, num_blocks=a["num_blocks"],
                       block_tables=np.zeros((len(ql), 1), np.int32), seq_lens=cx + ql, ctx_lens=cx,
                       query_start_loc=qsl, q=None, k_cache=None, v_cache=None)

    with m.patch.object(W, "build_batch", side_effect=fake):
        return fn(**kw)


@pytest.mark.parametrize("cfg", ["config1", "config2", "config3", "config4", "config5"])
def test_plan_covers_every_block_and_row_once(cfg):
    b = meta_only(getattr(W, cfg))
    for seg, pct, blk in ((0, 15, 8), (1, 15, 8), (3, 50, 1), (7, 0, 8), (500, 15, 3), (10 ** 9, 15, 8), (2, 90, 5)):
        plan = dry(b.seq_lens, b.query_start_loc, b.ctx_lens, num_q_heads=b.Hq, num_kv_heads=b.Hkv, head_dim=b.hd,
                   workspace_bytes=1 << 30, decode_segments=seg, decode_tail_pct=pct, decode_tail_blocks=blk)
        check_cover(b, plan)


def check_workspace(plan, Hq, Hkv, hd, workspace_bytes):
    """What the kernels will write of partial results lies inside the workspace: the decode slots (fp32 accumulator,
    maximum and sum per slot and query head), then, 256-byte aligned, one part per (part entry, kv head) of the split
    prefill tiles (fp32, per query column of the tile)."""
    dec = (plan["slots"] * Hq * (hd + 2) * 4 + 255) // 256 * 256
    t = plan["prefill_tiles"]
    entries = int(t[t[:, 4] > 1][:, 4].sum()) if len(t) else 0
    cols = 256 if len(t) and int(t[:, 2].max()) * (Hq // Hkv) > 128 else 128
    assert min(entries, len(t)) * Hkv <= 8192      # arrival counters: per part-0 slot with the tile list, per tile without
    assert entries == 0 or dec + entries * Hkv * cols * (hd + 2) * 4 <= workspace_bytes
    assert plan["slots"] * Hq * (hd + 2) * 4 <= workspace_bytes
    assert plan["prefill_parts"] == (int(t[:, 4].max()) if len(t) else 1)


def test_plans_of_random_batches_cover_every_block_and_row_once():
    # 300 seeded batches: 1-400 sequences, a random mix of empty / decode / chunk sequences, lengths over four orders of
    # magnitude, head shapes, compute-unit counts, workspace sizes and every planner option that shapes the work lists
    rng = np.random.default_rng(20251)
    for case in range(300):
        n = int(rng.choice([1, 2, 5, 30, 120, 400]))
        kinds = rng.choice(3, size=n, p=[0.1, 0.6, 0.3])
        ql = np.where(kinds == 0, 0, np.where(kinds == 1, 1, rng.integers(2, 3000, size=n))).astype(np.int32)
        cx = np.where(rng.random(n) < 0.15, 0, (2.0 ** rng.uniform(0, 16, size=n)).astype(np.int64)).astype(np.int32)
        qsl = np.zeros(n + 1, np.int32)
        qsl[1:] = np.cumsum(ql)
        Hq, Hkv, hd = [(32, 8, 128), (28, 4, 128), (64, 8, 128), (8, 1, 128), (16, 16, 64), (4, 1, 64)][rng.integers(6)]
        kw = dict(num_q_heads=Hq, num_kv_heads=Hkv, head_dim=hd, num_cus=int(rng.choice([256, 304, 64, 8])),
                  workspace_bytes=int(rng.choice([1 << 20, 64 << 20, 1 << 30])),
                  decode_segments=int(rng.choice([0, 0, 1, 5, 77, 10 ** 9])), decode_tail_pct=int(rng.choice([0, 0, 15, 60])),
                  decode_tail_blocks=int(rng.choice([1, 3, 8])), prefill_split=int(rng.choice([0, 0, 1, 2, 7])),
                  decode_piece_pad=int(rng.choice([-1, -1, 0, 3, 64])))
        if rng.random() < 0.2:
            kw["xcd_weights"] = rng.integers(60, 140, size=8).astype(np.int32)
        b = W.Batch(Hq=Hq, Hkv=Hkv, hd=hd, BS=16, num_blocks=1, block_tables=np.zeros((n, 1), np.int32), seq_lens=cx + ql,
                    ctx_lens=cx, query_start_loc=qsl, q=None, k_cache=None, v_cache=None)
        try:
            plan = dry(b.seq_lens, b.query_start_loc, b.ctx_lens, **kw)
            check_cover(b, plan)
            check_workspace(plan, Hq, Hkv, hd, kw["workspace_bytes"])
        except Exception as e:
            raise AssertionError(f"case {case}: q_lens {ql.tolist()} ctx {cx.tolist()} {kw}") from e


def test_default_plan_is_equal_static_runs_plus_short_tail_runs():
    for cfg in (W.config2, W.config4, W.config5):
        b = meta_only(cfg)
        plan = dry(b.seq_lens, b.query_start_loc, b.ctx_lens, num_q_heads=b.Hq, num_kv_heads=b.Hkv,
                   workspace_bytes=1 << 30, decode_tail_pct=15, decode_piece_pad=0)
        d = plan["decode_pieces"]
        R, T = plan["decode_runs"], plan["tail_runs"]
        per_run = np.bincount(d[:, 4], weights=d[:, 2] - d[:, 1], minlength=R + T)
        assert per_run[:R].max() - per_run[:R].min() <= 1 and per_run[:R].min() >= 1
        assert T > 0 and per_run[R:].max() - per_run[R:].min() <= 1 and 1 <= per_run[R:].max() <= 8
        total = per_run.sum()
        assert 0.10 * total <= per_run[R:].sum() <= 0.16 * total           # 15 % handed out dynamically
        assert R * b.Hkv <= 256 * 8
        assert (np.diff(d[:, 4]) >= 0).all()
    # no tail when asked for none, or when runs are short anyway
    b = meta_only(W.config2)
    assert dry(b.seq_lens, b.query_start_loc, b.ctx_lens, decode_tail_pct=0)["tail_runs"] == 0
    assert dry(b.seq_lens, b.query_start_loc, b.ctx_lens, decode_segments=2000)["tail_runs"] == 0


def test_runs_that_start_more_pieces_stream_fewer_blocks():
    for cfg in (W.config2, W.config3, W.config4):
        b = meta_only(cfg)
        for pad in (3, 6, 1):
            plan = dry(b.seq_lens, b.query_start_loc, b.ctx_lens, num_q_heads=b.Hq, num_kv_heads=b.Hkv,
                       workspace_bytes=1 << 30, decode_piece_pad=pad)
            check_cover(b, plan)
            d = plan["decode_pieces"]
            R = plan["decode_runs"]
            blocks = np.bincount(d[:, 4], weights=d[:, 2] - d[:, 1], minlength=R)
            starts = np.bincount(d[:, 4], weights=(d[:, 1] == 0), minlength=R)
            cost = blocks + pad * starts
            # equal up to the rounding of the cuts and a piece start that a cut may split between two runs
            assert cost.max() - cost.min() <= 2 * pad + 1, (pad, cost.min(), cost.max())
            assert np.percentile(cost, 90) - np.percentile(cost, 10) <= 1
            assert blocks.max() - blocks.min() >= pad                       # and the block counts do differ
        default = dry(b.seq_lens, b.query_start_loc, b.ctx_lens, num_q_heads=b.Hq, num_kv_heads=b.Hkv, workspace_bytes=1 << 30)
        three = dry(b.seq_lens, b.query_start_loc, b.ctx_lens, num_q_heads=b.Hq, num_kv_heads=b.Hkv, workspace_bytes=1 << 30,
                    decode_piece_pad=3)
        assert (default["decode_pieces"] == three["decode_pieces"]).all()   # head_dim 128: three blocks


def test_xcd_weights_shape_the_static_runs():
    w = [100, 90, 110, 95, 105, 85, 115, 100]
    for cfg in (W.config1, W.config2, W.config3, W.config4, W.config5):
        b = meta_only(cfg)
        for seg, pct, trial_pad in ((0, 0, 0), (96, 0, 0), (100, 15, 0), (8, 0, 0), (17, 30, 0), (0, 0, 3), (100, 15, 5)):
            plan = dry(b.seq_lens, b.query_start_loc, b.ctx_lens, num_q_heads=b.Hq, num_kv_heads=b.Hkv, head_dim=b.hd,
                       workspace_bytes=1 << 30, decode_segments=seg, decode_tail_pct=pct, xcd_weights=w,
                       decode_piece_pad=trial_pad)
            check_cover(b, plan)
            R = plan["decode_runs"]
            if R < 8 or trial_pad:
                continue                      # too few runs for one per XCD: equal runs
            assert R % 8 == 0
            d = plan["decode_pieces"]
            per_run = np.bincount(d[:, 4], weights=d[:, 2] - d[:, 1], minlength=R)[:R]
            per_xcd = per_run.reshape(-1, 8).sum(0)
            share = per_xcd / per_xcd.sum()
            assert np.abs(share - np.array(w) / sum(w)).max() < 0.01 + 8.0 / per_xcd.sum()
    # fewer than 8 runs, or no weights: equal runs
    b = meta_only(W.config2)
    plan = dry(b.seq_lens, b.query_start_loc, b.ctx_lens, decode_segments=5, xcd_weights=w, decode_piece_pad=0)
    d = plan["decode_pieces"]
    per_run = np.bincount(d[:, 4], weights=d[:, 2] - d[:, 1])
    assert plan["decode_runs"] == 5 and per_run.max() - per_run.min() <= 1
    with pytest.raises(B.OocoError):
        dry(b.seq_lens, b.query_start_loc, b.ctx_lens, xcd_weights=[1, 2, 3, 0, 5, 6, 7, 8])


def test_small_workspace_reduces_the_number_of_runs():
    b = meta_only(W.config4)
    big = dry(b.seq_lens, b.query_start_loc, b.ctx_lens, workspace_bytes=1 << 30)
    small = dry(b.seq_lens, b.query_start_loc, b.ctx_lens, workspace_bytes=9 << 20)
    assert small["slots"] * 32 * 130 * 4 <= 9 << 20 < big["slots"] * 32 * 130 * 4
    assert small["decode_runs"] < big["decode_runs"]
    check_cover(b, small)
    tiny = dry(b.seq_lens, b.query_start_loc, b.ctx_lens, workspace_bytes=1024)
    assert tiny["decode_runs"] == 1 and tiny["tail_runs"] == 0 and tiny["slots"] == 0
    assert (tiny["decode_pieces"][:, 3] == -1).all()


def prefill_parts(n, c, prior, **kw):
    return dry([prior + c] * n, [i * c for i in range(n + 1)], [prior] * n, **kw)["prefill_parts"]


def test_prefill_tiles_are_split_only_when_the_batch_cannot_occupy_the_gpu():
    # the benchmark configurations' prefill parts and other batches with a workgroup or more per CU stay whole
    for n, c, prior in ((2, 2048, 4096), (8, 512, 1024), (1, 2048, 8192), (4, 512, 2048), (1, 2048, 0)):
        assert prefill_parts(n, c, prior) == 1, (n, c, prior)
    # a few tiles walking a long context alone are cut up; fewer parts the more tiles there are
    p1, p4, p8 = (prefill_parts(n, 128, 8192) for n in (1, 4, 8))
    assert 16 >= p1 > p4 >= p8 >= 1 and p4 >= 2
    # no context to cut: one 64-key step per part at least
    assert prefill_parts(1, 128, 0) == 1
    assert prefill_parts(1, 32, 100, prefill_split=8) <= 3
    # forced values are honoured up to 16; the workspace bounds the parts (66,560 bytes each here)
    assert prefill_parts(1, 128, 8192, prefill_split=3) == 3
    assert prefill_parts(1, 128, 8192, prefill_split=50) == 16
    assert prefill_parts(1, 128, 8192, prefill_split=8, workspace_bytes=32 * 5 * 66560) == 5
    assert prefill_parts(1, 128, 8192, workspace_bytes=0) == 1
    # decode-only batches report 1
    assert dry([100, 200], [0, 1, 2], [99, 199])["prefill_parts"] == 1


def test_tiles_get_parts_by_their_own_number_of_steps():
    # a chunk on a long context among chunks on short ones: its tiles are cut up, the others stay whole, and no part is
    # longer than the longest tile's parts; forced values give every tile the same number of parts
    ql = np.array([128, 128, 128, 128, 1], np.int32)
    cx = np.array([256, 16384, 300, 256, 77], np.int32)
    qsl = np.zeros(len(ql) + 1, np.int32)
    qsl[1:] = np.cumsum(ql)
    plan = dry(cx + ql, qsl, cx)
    t = plan["prefill_tiles"]
    steps = (t[:, 3] + t[:, 2] + 63) // 64
    k = plan["prefill_parts"]
    assert 4 <= k <= 16 and (t[t[:, 0] == 1, 4] == k).all() and (t[t[:, 0] != 1, 4] == 1).all()
    longest = -(-steps.max() // k)
    assert (-(-steps // t[:, 4]) <= longest).all()
    check_cover(W.Batch(Hq=32, Hkv=8, hd=128, BS=16, num_blocks=1, block_tables=np.zeros((5, 1), np.int32), seq_lens=cx + ql,
                        ctx_lens=cx, query_start_loc=qsl, q=None, k_cache=None, v_cache=None), plan)
    # the first parts go out by decreasing length of a part
    per = -(-steps // t[:, 4])
    assert (np.diff(per) <= 0).all()
    forced = dry(cx + ql, qsl, cx, prefill_split=4)["prefill_tiles"]
    assert (forced[:, 4] == np.minimum(4, (forced[:, 3] + forced[:, 2] + 63) // 64)).all()
    # a batch of equal chunks gets equal parts
    eq = dry([8192 + 128] * 2, [0, 128, 256], [8192] * 2)
    assert len(set(eq["prefill_tiles"][:, 4].tolist())) == 1 and eq["prefill_parts"] > 1


def test_decode_runs_of_short_sequence_batches():
    # profiles/decode_short_sequences_rule.md: sequences of 24 blocks or fewer on average get four waves per compute
    # unit (128 runs for 8 kv heads) and as many runs as sequences; longer ones three waves and runs of 16 blocks at least
    def runs(n, tokens):
        return dry([tokens] * n, list(range(n + 1)), [tokens - 1] * n)["decode_runs"]
    assert runs(512, 128) == 128 and runs(2048, 256) == 128 and runs(1024, 384) == 128
    assert runs(32, 128) == 32 and runs(32, 64) == 32 and runs(64, 256) == 64 and runs(8, 128) == 8
    assert runs(4096, 512) == 96 and runs(256, 8192) == 96 and runs(64, 32768) == 96
    assert runs(1, 8192) == 32                    # a small batch of one long sequence: 16 blocks per run


def test_planned_parts_match_the_measured_best_on_the_profiled_batches():
    # the choices that profiles/prefill_split_rule.md and profiles/mixed_lean_rule.md measure as best or within a few
    # per cent of the best (256 compute units, 32/8 heads): a change of the cost model that moves one of them needs a new
    # measurement
    def parts(ql, cx):
        ql, cx = np.asarray(ql, np.int32), np.asarray(cx, np.int32)
        qsl = np.zeros(len(ql) + 1, np.int32)
        qsl[1:] = np.cumsum(ql)
        t = dry(cx + ql, qsl, cx)["prefill_tiles"]
        return {int(i): sorted(set(t[t[:, 0] == i][:, 4].tolist())) for i in np.flatnonzero(ql > 1)}, int(t[:, 2].max())
    for (n, c, pc), want in (((1, 128, 8192), 8), ((1, 128, 32768), 16), ((4, 128, 8192), 4), ((1, 512, 8192), 4),
                             ((2, 512, 4096), 2), ((2, 512, 1000), 1), ((8, 128, 2048), 1), ((10, 128, 8192), 1),
                             ((3, 512, 8192), 1), ((1, 2048, 8192), 1), ((16, 128, 1000), 1)):
        got, _ = parts([c] * n, [pc] * n)
        assert all(v == [want] for v in got.values()), ((n, c, pc), got)
    # chunks on unequal contexts: the long chunk's tiles are cut up, the others stay whole
    got, _ = parts([256] * 9, [32768] + [512] * 8)
    assert got[0] == [7] and all(got[i] == [1] for i in range(1, 9))
    got, _ = parts([2048, 128], [0, 30000])
    assert got[0] == [1] and 8 <= got[1][0] <= 12
    # an online chunk on a long prefix beside 128 decode sequences: the lean pair (64-row tiles), one round of workgroups
    got, rows = parts([512] + [1] * 128, [30000] + [2048] * 128)
    assert rows == 64 and got[0] == [4]
    got, rows = parts([512] + [1] * 32, [30000] + [2048] * 32)          # a short decode part: planned as a prefill batch
    assert rows == 32 and got[0] == [4]


def test_few_prefill_tiles_are_dispatched_longest_first_across_chunks():
    # up to 896 tiles: one list entry per tile, by decreasing number of 64-key steps whatever the chunk; ties keep
    # the chunk order (longest sequence first) and the later tile of a chunk first
    ql = np.array([512, 1, 300, 512, 33, 1, 512, 64, 2], np.int32)
    cx = np.array([1662, 4000, 0, 175, 90, 17, 1781, 700, 5], np.int32)
    qsl = np.zeros(len(ql) + 1, np.int32)
    qsl[1:] = np.cumsum(ql)
    t = dry(cx + ql, qsl, cx)["prefill_tiles"]
    want = sum(-(-int(q) // 32) for q in ql if q > 1)
    assert len(t) == want and len({(int(r[0]), int(r[1])) for r in t}) == want          # every tile once
    steps = (t[:, 3] + t[:, 2] + 63) // 64
    # 63 tiles on 256 compute units and 8 kv heads: one round of at most two workgroups per unit, workgroups w and
    # w + 256 (tile positions p and p + 32) share a unit -- the first 32 positions descend, the others ASCEND, so that
    # the longest tile is paired with the shortest
    assert steps[0] == (1781 + 512 + 63) // 64 and (np.diff(steps[:32]) <= 0).all() and (np.diff(steps[32:]) >= 0).all()
    assert steps[32:].max() <= steps[:32].min()
    assert len(np.unique(t[:32, 0])) > 1                                                   # chunks interleave
    order = np.r_[np.arange(32), np.arange(len(t) - 1, 31, -1)]                             # back to descending order
    td, sd = t[order], steps[order]
    for a, b2, sa, sb in zip(td[:-1], td[1:], sd[:-1], sd[1:]):
        if sa == sb and a[0] != b2[0]:
            assert (cx + ql)[a[0]] >= (cx + ql)[b2[0]]
        if sa == sb and a[0] == b2[0]:
            assert a[1] > b2[1]
    # a batch of two rounds keeps the plain descending order
    ql3 = np.full(8, 512, np.int32)
    cx3 = np.array([1662, 175, 367, 485, 371, 1641, 1781, 1192], np.int32)
    qsl3 = np.zeros(9, np.int32)
    qsl3[1:] = np.cumsum(ql3)
    t3 = dry(cx3 + ql3, qsl3, cx3)["prefill_tiles"]
    assert len(t3) == 128 and (np.diff((t3[:, 3] + t3[:, 2] + 63) // 64) <= 0).all()
    # 528 tiles still have a list; the 16 tiles of the chunk on 70,000 cached tokens are cut up and come first
    ql2, cx2 = np.array([8192, 8192, 512], np.int32), np.array([100, 100, 70000], np.int32)
    qsl2 = np.zeros(4, np.int32)
    qsl2[1:] = np.cumsum(ql2)
    t2 = dry(cx2 + ql2, qsl2, cx2)["prefill_tiles"]
    assert len(t2) == 256 + 256 + 16
    assert (t2[:16, 0] == 2).all() and (t2[:16, 4] > 1).all() and (t2[16:, 4] == 1).all()
    assert (np.diff((t2[16:, 3] + t2[16:, 2] + 63) // 64) <= 0).all()
    # more than 896 tiles: chunk by chunk, longest sequence first, later tiles first
    ql4, cx4 = np.array([16384, 16384, 512], np.int32), np.array([100, 5000, 70000], np.int32)
    qsl4 = np.zeros(4, np.int32)
    qsl4[1:] = np.cumsum(ql4)
    t4 = dry(cx4 + ql4, qsl4, cx4)["prefill_tiles"]
    assert len(t4) == 512 + 512 + 16
    assert (t4[:16, 0] == 2).all() and (t4[16:528, 0] == 1).all() and (t4[528:, 0] == 0).all()
    for i in (0, 1, 2):
        assert (np.diff(t4[t4[:, 0] == i][:, 1]) < 0).all()


def test_lean_pair_is_planned_only_where_the_prefill_part_weighs_enough():
    # the eight-wave prefill workgroups of the register-lean pair show in the dry run as tiles of 256 / g query rows
    # (g = 4: 64) instead of 128 / g; the pair is planned when every compute unit gets such a workgroup and the prefill
    # part's estimated time is 0.30 .. 4 times the decode part's
    rng = np.random.default_rng(3)
    dec = rng.integers(1500, 4000, size=128).astype(np.int32)          # about 1.4 GB of K/V

    def tile_rows(n_chunks, chunk, n_dec):
        ql = np.r_[np.full(n_chunks, chunk), np.ones(n_dec, int)].astype(np.int32)
        cx = np.r_[np.full(n_chunks, 1000), dec[:n_dec] - 1].astype(np.int32)
        qsl = np.zeros(len(ql) + 1, np.int32)
        qsl[1:] = np.cumsum(ql)
        return int(dry(cx + ql, qsl, cx)["prefill_tiles"][:, 2].max())

    assert tile_rows(8, 512, 128) == 64            # config 3's proportions
    assert tile_rows(2, 2048, 128) == 64
    assert tile_rows(4, 512, 128) == 32            # too little prefill work beside this much decode
    assert tile_rows(16, 128, 128) == 32
    assert tile_rows(8, 2048, 16) == 32            # prefill-dominated: the stand-alone kernels
    assert tile_rows(8, 512, 0) == 32 and tile_rows(1, 512, 128) == 32


def test_empty_batch_plans_to_nothing():
    plan = dry(np.zeros(0, np.int32), np.zeros(1, np.int32), np.zeros(0, np.int32), num_seqs=0)
    assert len(plan["decode_pieces"]) == 0 and len(plan["prefill_tiles"]) == 0


# ----------------------------------------------------------------------------- latency model (host function)
@BOTH_RECORDS
def test_predict_latency_equals_the_model_oracle(record):
    from oracle import perf_model
    rng = np.random.default_rng(3)
    for trial in range(40):
        Hkv = int(rng.choice([1, 2, 4, 8]))
        Hq = Hkv * int(rng.choice([1, 4, 7, 8]))
        hd = int(rng.choice([64, 128]))
        n = int(rng.integers(1, 40))
        ql = rng.choice([0, 1, 1, 1, 2, 17, 512, 2048], size=n)
        cx = rng.integers(0, 100000, size=n)
        qsl = np.concatenate([[0], np.cumsum(ql)])
        p = dict(F_ap=10 ** rng.uniform(13, 15.5), F_ad=10 ** rng.uniform(12, 15), M_a=10 ** rng.uniform(11.5, 13),
                 O_p=rng.uniform(0, 1e-4), O_d=rng.uniform(0, 1e-4))
        causal = bool(trial % 2)
        got = B.ooco_predict_latency(p, Hq, Hkv, hd, qsl, cx, causal_flops=causal)
        want = perf_model.predict(p, Hq, Hkv, hd, ql, cx, causal=causal)
        for k in want:
            assert got[k] == pytest.approx(want[k], rel=1e-12, abs=1e-300), (trial, k)
    assert B.ooco_predict_latency(p, 32, 8, 128, [0], [])["latency"] == 0.0
    for bad in (dict(p, M_a=0.0), dict(p, F_ap=-1.0)):
        with pytest.raises(B.OocoError):
            B.ooco_predict_latency(bad, 32, 8, 128, [0, 1], [5])
    with pytest.raises(B.OocoError):
        B.ooco_predict_latency(p, 32, 7, 128, [0, 1], [5])


# ----------------------------------------------------------------------------- Mix Decoding Selection (host function)
@BOTH_RECORDS
def test_mix_decoding_select_equals_the_oracle(record):
    from oracle import mix_select
    rng = np.random.default_rng(12)
    p = dict(F_ap=9e14, F_ad=2e14, M_a=6e12, O_p=1e-5, O_d=9e-6)
    for trial in range(80):
        Hkv = int(rng.choice([2, 4, 8]))
        Hq = Hkv * int(rng.choice([1, 4, 7, 8]))
        on = rng.integers(16, 6000, size=rng.integers(0, 6))
        off = rng.integers(16, 40000, size=rng.integers(0, 40))
        if trial % 5 == 0 and len(off):
            off[:] = off[0]                                            # ties in the sort
        order = rng.integers(-1, len(off) + 1, size=rng.integers(0, 12))
        base = mix_select.latency(p, Hq, Hkv, 128, list(on) + list(off[: len(off) // 2]))
        S = float(rng.uniform(0.3, 2.5)) * max(base, 5e-6)
        want = mix_select.mix_decoding_select(p, Hq, Hkv, 128, S, on, off, order)
        got = B.ooco_mix_decoding_select(p, Hq, Hkv, 128, S, on, off, order)
        assert list(got["selected"]) == want["selected"], trial
        assert got["latency"] == pytest.approx(want["latency"], rel=1e-12)
    # the hand-worked example of tests/golden/mix_selection.txt through the library
    mp = dict(F_ap=1e18, F_ad=1e18, M_a=4.096e9, O_p=0.0, O_d=10e-6)
    got = B.ooco_mix_decoding_select(mp, 32, 8, 128, 700e-6, [100, 200], [50, 400, 30, 120, 60, 500], [1, 5, 1])
    assert list(got["selected"]) == [True, False, True, True, True, False] and got["latency"] == pytest.approx(594e-6, rel=1e-12)
    with pytest.raises(B.OocoError):
        B.ooco_mix_decoding_select(mp, 32, 8, 128, 1e-3, [0], [5], [])
    # the bound is inclusive in both phases (Algorithm 2 admits on L <= S): bounds that equal a predicted latency
    on, off = [700, 1500], [900, 300, 5000, 1200, 650]
    S = B.ooco_predict_latency(p, 32, 8, 128, np.arange(4), np.array(on + [off[2]]) - 1)["latency"]
    assert S == mix_select.latency(p, 32, 8, 128, on + [off[2]])
    assert list(B.ooco_mix_decoding_select(p, 32, 8, 128, S, on, off, [2])["selected"]) == [False, False, True, False, False]
    S = mix_select.latency(p, 32, 8, 128, on + [300, 650, 900])
    assert list(B.ooco_mix_decoding_select(p, 32, 8, 128, S, on, off, [])["selected"]) == [True, True, False, False, True]


# ----------------------------------------------------------------------------- migration decision, eviction rule
@BOTH_RECORDS
def test_migration_and_eviction_equal_the_oracle(record):
    from oracle import migration, mix_select
    rng = np.random.default_rng(31)
    branches = set()
    for trial in range(120):
        p = dict(F_ap=9e14, F_ad=float(rng.choice([3e12, 2e14])), M_a=6e12, O_p=1e-5, O_d=9e-6)
        Hkv = int(rng.choice([2, 4, 8]))
        Hq = Hkv * int(rng.choice([1, 4, 7]))
        Bl = [int(x) for x in rng.integers(1, 3000, size=rng.integers(0, 8))]
        sat = int(rng.integers(1, 16))
        S = max(mix_select.latency(p, Hq, Hkv, 128, Bl), 5e-6) * float(rng.uniform(0.9, 1.6) if trial % 2 else rng.uniform(1.0, 3.0))
        cap = int(rng.integers(20, 1500))
        lo = int(rng.choice([1, 16, 1200]))
        hi = lo + int(rng.integers(0, 1500))
        inc = bool(trial % 7)
        want = migration.migration_preference(p, Hq, Hkv, 128, S, Bl, inc, sat, 16, cap, lo, hi)
        got = B.ooco_migration_preference(p, Hq, Hkv, 128, S, Bl, inc, sat, 16, cap, lo, hi)
        assert got == want, (trial, got, want)
        branches.add(got["branch"])
        rel = [int(x) for x in rng.integers(1, 4000, size=rng.integers(0, 20))]
        if trial % 4 == 0 and rel:
            rel = [rel[0]] * len(rel)                                  # ties in the order
        pref = got["pref"] or int(rng.integers(1, 3000))
        mm = int(rng.integers(0, 8))
        assert (B.ooco_migration_select(p, Hq, Hkv, 128, S, Bl, rel, pref, 16, cap, mm)
                == migration.migration_select(p, Hq, Hkv, 128, S, Bl, rel, pref, 16, cap, mm)), trial
        need = int(rng.integers(0, 300))
        bs = int(rng.integers(0, 20))
        w = migration.eviction_victims(rel, need, 16, bs, sat)
        g = B.ooco_eviction_victims(rel, need, 16, bs, sat)
        assert g["victims"] == w["victims"] and g["enough"] == w["enough"], trial
    assert branches == {"none", "saturated", "reach", "shortest"}


@BOTH_RECORDS
def test_migration_golden_cases_through_the_library(record):
    mp = dict(F_ap=1e18, F_ad=1e18, M_a=4.096e9, O_p=0.0, O_d=10e-6)
    path = os.path.join(ROOT, "tests", "golden", "migration.txt")
    rows = [l.split() for l in open(path) if l[:1].isalpha()]
    assert len(rows) == 15
    for c in rows:
        if c[0] == "pref":
            r = B.ooco_migration_preference(mp, 32, 8, 128, float(c[1]) * 1e-6, [100, 200], int(c[2]), int(c[3]), 16,
                                            int(c[4]), int(c[5]), int(c[6]))
            assert (r["branch"], -1 if r["pref"] is None else r["pref"]) == (c[8], int(c[9])), c
            continue
        lens = [int(x) for x in c[c.index(":") + 1:c.index("->")]]
        want = [int(x) for x in c[c.index("->") + 1:]]
        if c[0] == "select":
            assert B.ooco_migration_select(mp, 32, 8, 128, float(c[1]) * 1e-6, [100, 200], lens, int(c[2]), 16, 10 ** 6,
                                           int(c[3])) == want, c
        else:
            r = B.ooco_eviction_victims(lens, int(c[1]), 16, int(c[2]), int(c[3]))
            assert [int(r["enough"])] + r["victims"] == want, c


def test_migration_functions_reject_bad_arguments():
    mp = dict(F_ap=1e18, F_ad=1e18, M_a=4.096e9, O_p=0.0, O_d=10e-6)
    for kw in (dict(len_min=0), dict(len_min=10, len_max=9), dict(bs_sat=0), dict(block_size=0), dict(batch_lens=[5, 0])):
        args = dict(batch_lens=[100], all_included=True, bs_sat=2, block_size=16, capacity_blocks=100, len_min=1, len_max=100)
        args.update(kw)
        with pytest.raises(B.OocoError) as e:
            B.ooco_migration_preference(mp, 32, 8, 128, 1e-3, **args)
        assert "ooco_migration_preference" in e.value.message
    with pytest.raises(B.OocoError):
        B.ooco_migration_select(mp, 32, 8, 128, 1e-3, [100], [50, -3], 60, 16, 100, 4)
    with pytest.raises(B.OocoError):
        B.ooco_eviction_victims([10, 0], 5, 16, 3, 8)
    assert B.ooco_eviction_victims([], 5, 16, 3, 8) == dict(victims=[], enough=False)
    assert B.ooco_eviction_victims([40], 0, 16, 3, 8) == dict(victims=[], enough=True)

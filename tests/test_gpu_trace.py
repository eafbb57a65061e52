"""Option "trace" on the GPU: the decode waves' and the prefill workgroups' own time stamps (ooco_trace_read) are
complete and ordered, and tracing changes no output bit."""
import numpy as np
import pytest
import torch

from paper_2511_21862_amd import binding as B
from paper_2511_21862_amd import workloads as W

from gpu_util import device_meta, run_gpu, say

pytestmark = pytest.mark.gpu


def traced(b, options=None):
    """(output bits of a traced call, stamps, plan info) of one batch."""
    d = W.to_device(b)
    bt, sl, qsl, cl = device_meta(b)
    out = torch.full((b.total_q, b.Hq, b.hd), float("nan"), dtype=torch.bfloat16, device="cuda")
    with B.Context(b.Hq, b.Hkv, b.hd, b.BS, b.num_blocks, b.max_blocks_per_seq) as ctx:
        for k, v in (options or {}).items():
            ctx.set_option(k, v)
        ctx.set_option("trace", 1)
        ctx.plan(b.seq_lens, b.query_start_loc, b.ctx_lens)
        info = ctx.plan_info()
        ctx.attn_mixed(d.q, d.k_cache, d.v_cache, bt, sl, qsl, cl, out)
        stamps = ctx.trace_read()
    return out.view(torch.int16).cpu().numpy().view(np.uint16), stamps, info


def test_decode_waves_leave_ordered_stamps_and_the_output_is_unchanged():
    rng = np.random.default_rng(11)
    lens = rng.integers(200, 6000, size=24).astype(np.int32)
    b = W.build_batch(Hq=32, Hkv=8, hd=128, q_lens=np.ones(24, np.int32), ctx_lens=lens - 1,
                      num_blocks=int(((lens + 15) // 16).sum()) + 9, seed=11, poison=True)
    say("case: trace of a decode batch")
    got, t, info = traced(b)
    assert np.array_equal(got, run_gpu(b))
    assert len(t) == info["decode_waves"] * b.Hkv and len(t) > 0
    t = t.astype(np.int64)
    # wave start <= first tiles arrived <= end of streaming <= wave end, all within a few milliseconds (100 MHz clock)
    assert (t[:, 0] > 0).all()
    assert (t[:, 0] <= t[:, 1]).all() and (t[:, 1] <= t[:, 2]).all() and (t[:, 2] <= t[:, 3]).all()
    assert t[:, 3].max() - t[:, 0].min() < 100 * 5000
    say(f"  {len(t)} waves, kernel span {(t[:, 3].max() - t[:, 0].min()) / 100:.1f} us")


@pytest.mark.parametrize("opts", [{}, {"prefill_split": 2}, {"prefill_waves": 8}], ids=["default", "split2", "8waves"])
def test_prefill_workgroups_leave_stamps_and_the_output_is_unchanged(opts):
    b = W.build_batch(Hq=32, Hkv=8, hd=128, q_lens=[300, 64, 513], ctx_lens=[900, 0, 2000], num_blocks=260, seed=12,
                      poison=True)
    say(f"case: trace of a prefill-only batch, {opts}")
    got, t, info = traced(b, opts)
    assert np.array_equal(got, run_gpu(b, options=opts))
    # one workgroup per (tile, part, kv head); a tile never has more parts than 64-key steps
    assert info["prefill_tiles"] * b.Hkv <= len(t) <= info["prefill_tiles"] * b.Hkv * info["prefill_parts"]
    if "prefill_split" in opts:
        assert len(t) > info["prefill_tiles"] * b.Hkv
    t = t.astype(np.int64)
    assert (t[:, 0] > 0).all() and (t[:, 0] <= t[:, 3]).all()
    assert t[:, 3].max() - t[:, 0].min() < 100 * 5000
    xcd, cu = t[:, 1] >> 8, t[:, 1] & 255
    assert ((xcd >= 0) & (xcd < 8)).all()
    # four phases of a workgroup, 16 bits each, in 10 ns since its start: tile looked up, first loads sent off, first
    # tiles arrived, last step done (0: a part of a split tile that found no step left for it)
    ph = np.stack([(t[:, 2] >> (16 * k)) & 0xFFFF for k in range(4)], axis=1)
    ran = t[:, 2] != 0
    assert ran.sum() >= len(t) // 2
    assert (np.diff(ph[ran], axis=1) >= 0).all() and (ph[ran, 0] > 0).all()
    assert (ph[ran, 3] <= np.minimum(t[ran, 3] - t[ran, 0], 0xFFFF)).all()
    # the hardware deals a launch's workgroups to the XCDs in turn (starting wherever the last launch stopped), so
    # with eight kv heads all tiles of a kv head meet in one L2
    assert len(np.unique((xcd - np.arange(len(t))) % 8)) == 1
    say(f"  {len(t)} workgroups on {len(np.unique(t[:, 1]))} compute units, span {(t[:, 3].max() - t[:, 0].min()) / 100:.1f} us; "
        f"median phases {np.median(ph[ran], axis=0) / 100} us")

"""The entry point that allocates nothing (ooco_attn_mixed_static) against ooco_attn_mixed, through the C ABI:
two calls in a row on one GPU, the second on a smaller batch, so that the second call finds the first one's
contents in the shared device array."""
import numpy as np
import pytest
import torch

from oracle import ref_c
from paper_2511_21862_amd import binding as B
from paper_2511_21862_amd import workloads as W

from gpu_util import MAX_ABS, MEAN_ABS, assert_parity, device_meta, run_gpu, say

pytestmark = pytest.mark.gpu


def run_static(b):
    d = W.to_device(b)
    bt, sl, qsl, cl = device_meta(b)
    out = torch.full((b.total_q, b.Hq, b.hd), float("nan"), dtype=torch.bfloat16, device="cuda")
    B.ooco_attn_mixed_static(b.Hq, b.Hkv, b.hd, b.BS, b.max_blocks_per_seq, 0.0, b.seq_lens, b.query_start_loc, b.ctx_lens,
                             d.q, d.k_cache, d.v_cache, bt, sl, qsl, cl, out, b.num_seqs, b.total_q)
    torch.cuda.synchronize()
    return out.view(torch.int16).cpu().numpy().view(np.uint16)


def check(b, what):
    got = run_static(b)
    # the existing entry point with the same planning choices (prefill tiles not split, the stand-alone pair of
    # kernels): same run layout, same bits
    want = run_gpu(b, options={"prefill_split": 1, "mixed_lean": 0})
    g, w = W.bf16_bits_to_f32(got).astype(np.float64), W.bf16_bits_to_f32(want).astype(np.float64)
    d = np.abs(g - w)
    say(f"  {what}: vs ooco_attn_mixed max-abs {d.max():.3g} mean-abs {d.mean():.3g}, bit-identical {np.array_equal(got, want)}")
    assert np.isfinite(g).all() and d.max() <= MAX_ABS and d.mean() <= MEAN_ABS
    assert np.array_equal(got, want)
    # ... and with its defaults (tiles of a small batch may be split there): same values within the float gate
    want2 = W.bf16_bits_to_f32(run_gpu(b)).astype(np.float64)
    d2 = np.abs(g - want2)
    assert d2.max() <= MAX_ABS and d2.mean() <= MEAN_ABS
    ref = ref_c.attn_mixed(b.q, b.k_cache, b.v_cache, b.block_tables, b.seq_lens, b.query_start_loc, b.ctx_lens)
    assert_parity(got, ref, what)


def test_static_entry_point_matches_attn_mixed_on_two_calls_in_a_row():
    say("case: ooco_attn_mixed_static, large then small batch")
    rng = np.random.default_rng(71)
    # first call: 40 decode sequences (many of them cut into partial results) and three ragged chunks
    dl = np.concatenate([rng.integers(900, 9000, size=36), [1, 17, 16, 4097]]).astype(np.int32)
    ql = np.concatenate([np.ones(len(dl), np.int32), [300, 70, 129]]).astype(np.int32)
    cx = np.concatenate([dl - 1, [1000, 0, 37]]).astype(np.int32)
    big = W.build_batch(Hq=32, Hkv=8, hd=128, q_lens=ql, ctx_lens=cx, num_blocks=int((cx + ql + 15).sum() // 16 + 64),
                        seed=71, poison=True)
    check(big, "first call (43 sequences)")
    # second call, smaller, other head shape: finds the first call's partial results and counters in the array
    small = W.build_batch(Hq=28, Hkv=4, hd=128, q_lens=[1, 1, 40, 1, 0, 1], ctx_lens=[3000, 15, 100, 5000, 7, 640],
                          num_blocks=700, seed=72, poison=True)
    check(small, "second call (6 sequences, 28/4 heads)")
    tiny = W.config1(poison=True)
    check(tiny, "third call (config 1)")


def test_static_entry_point_rejects_what_it_cannot_hold():
    b = W.config1()
    d = W.to_device(b)
    bt, sl, qsl, cl = device_meta(b)
    out = torch.empty((b.total_q, b.Hq, b.hd), dtype=torch.bfloat16, device="cuda")
    n = 961
    with pytest.raises(B.OocoError) as e:
        B.ooco_attn_mixed_static(b.Hq, b.Hkv, b.hd, b.BS, b.max_blocks_per_seq, 0.0, np.ones(n, np.int32),
                                 np.arange(n + 1, dtype=np.int32), np.zeros(n, np.int32), d.q, d.k_cache, d.v_cache, bt, sl,
                                 qsl, cl, out, n, n)
    assert e.value.status == B.OOCO_ENOMEM and "960" in e.value.message
    with pytest.raises(B.OocoError) as e:
        B.ooco_attn_mixed_static(b.Hq, b.Hkv, 96, b.BS, b.max_blocks_per_seq, 0.0, b.seq_lens, b.query_start_loc, b.ctx_lens,
                                 d.q, d.k_cache, d.v_cache, bt, sl, qsl, cl, out, b.num_seqs, b.total_q)
    assert e.value.status == B.OOCO_ESHAPE
    with pytest.raises(B.OocoError) as e:
        B.ooco_attn_mixed_static(b.Hq, b.Hkv, b.hd, b.BS, b.max_blocks_per_seq, 0.0, b.seq_lens, b.query_start_loc, b.ctx_lens,
                                 None, d.k_cache, d.v_cache, bt, sl, qsl, cl, out, b.num_seqs, b.total_q)
    assert e.value.status == B.OOCO_EINVAL
    # nothing to do: no launch, no error
    B.ooco_attn_mixed_static(b.Hq, b.Hkv, b.hd, b.BS, b.max_blocks_per_seq, 0.0, b.seq_lens, b.query_start_loc, b.ctx_lens,
                             d.q, d.k_cache, d.v_cache, bt, sl, qsl, cl, out, 0, 0)

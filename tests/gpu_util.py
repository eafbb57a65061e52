"""Helpers shared by the GPU parity tests: run a batch through libooco, compare with the oracle."""
import sys

import numpy as np
import torch

from paper_2511_21862_amd import binding as B
from paper_2511_21862_amd import workloads as W

MAX_ABS, MEAN_ABS, REL_L2 = 2e-2, 2e-3, 1e-2     # parity gates (bf16 in, fp32 accumulate, vs float64)


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def device_meta(b, device="cuda"):
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(device)
    return t(b.block_tables), t(b.seq_lens), t(b.query_start_loc), t(b.ctx_lens)


def run_gpu(b, *, plan=True, options=None, scale=0.0, ctx=None, workspace_bytes=0):
    """Runs one ooco_attn_mixed call; returns the bf16 output as uint16 bit patterns on the host."""
    d = W.to_device(b)
    bt, sl, qsl, cl = device_meta(b)
    out = torch.full((max(b.total_q, 1), b.Hq, b.hd), float("nan"), dtype=torch.bfloat16, device="cuda")[: b.total_q]
    own = ctx is None
    if own:
        ctx = B.Context(b.Hq, b.Hkv, b.hd, b.BS, b.num_blocks, b.max_blocks_per_seq, scale=scale,
                        workspace_bytes=workspace_bytes)
    try:
        for k, v in (options or {}).items():
            ctx.set_option(k, v)
        if plan:
            ctx.plan(b.seq_lens, b.query_start_loc, b.ctx_lens)
        ctx.attn_mixed(d.q, d.k_cache, d.v_cache, bt, sl, qsl, cl, out)
        torch.cuda.synchronize()
    finally:
        if own:
            ctx.close()
    return out.view(torch.int16).cpu().numpy().view(np.uint16)


def errors(gpu_bits, ref64):
    g = W.bf16_bits_to_f32(gpu_bits).astype(np.float64)
    diff = np.abs(g - ref64)
    denom = np.sqrt((ref64 ** 2).sum())
    return dict(max_abs=float(diff.max()) if diff.size else 0.0, mean_abs=float(diff.mean()) if diff.size else 0.0,
                rel_l2=float(np.sqrt((diff ** 2).sum()) / denom) if denom > 0 else 0.0,
                finite=bool(np.isfinite(g).all()))


def assert_parity(gpu_bits, ref64, what=""):
    e = errors(gpu_bits, ref64)
    say(f"  parity {what}: {e}")
    assert e["finite"], f"{what}: non-finite output"
    assert e["max_abs"] <= MAX_ABS, f"{what}: max-abs {e['max_abs']}"
    assert e["mean_abs"] <= MEAN_ABS, f"{what}: mean-abs {e['mean_abs']}"
    assert e["rel_l2"] <= REL_L2, f"{what}: relative L2 {e['rel_l2']}"
    return e

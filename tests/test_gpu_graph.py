"""ooco_attn_mixed under HIP graph capture: a planned call enqueues kernels and event fork/join only, so a
serving loop can capture a run of layers once and replay it.  Every replay is checked against the eager
result, with eager work and synchronisations between the replays."""
import pytest
import torch

from paper_2511_21862_amd import binding as B
from paper_2511_21862_amd import workloads as W

from gpu_util import device_meta, say

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("mixed", [False, True, "split", "lean"])
def test_captured_calls_replay_to_the_eager_result(mixed):
    # "split": the chunk sits on a long prefix, so its tiles are cut along the context and merged through the
    # workspace and the arrival counters, which every replay must find reset
    ql = [1, 1, 96, 1, 1] if mixed else [1, 1, 1, 1, 1]
    ctx_lens = [3000, 129, 4000 if mixed == "split" else 400, 64, 900]
    b = W.build_batch(Hq=32, Hkv=8, hd=128, q_lens=ql, ctx_lens=ctx_lens, num_blocks=560, seed=91)
    d = W.to_device(b)
    bt, sl, qsl, cl = device_meta(b)
    say(f"case: graph capture, {'mixed' if mixed else 'decode-only'} batch")
    eager = torch.empty((b.total_q, b.Hq, b.hd), dtype=torch.bfloat16, device="cuda")
    out = torch.zeros_like(eager)
    with B.Context(b.Hq, b.Hkv, b.hd, b.BS, b.num_blocks, b.max_blocks_per_seq) as ctx:
        ctx.set_option("plan_persistent", 1)     # one plan serves the eager calls, the capture and nothing changes in between
        if mixed == "lean":                      # the register-lean pair of kernels of large mixed batches, forced here
            ctx.set_option("mixed_lean", 2)
        ctx.plan(b.seq_lens, b.query_start_loc, b.ctx_lens)
        if mixed != "lean":
            assert (ctx.plan_info()["prefill_parts"] > 1) == (mixed == "split")
        ctx.attn_mixed(d.q, d.k_cache, d.v_cache, bt, sl, qsl, cl, eager)
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            ctx.attn_mixed(d.q, d.k_cache, d.v_cache, bt, sl, qsl, cl, out, side)     # warm-up on the capture stream
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                for _ in range(3):                                                    # three "layers"
                    ctx.attn_mixed(d.q, d.k_cache, d.v_cache, bt, sl, qsl, cl, out, torch.cuda.current_stream())
        for rep in range(4):
            out.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(out.view(torch.int16), eager.view(torch.int16)), f"replay {rep} differs from the eager result"
            # eager work of the same context between replays
            ctx.attn_mixed(d.q, d.k_cache, d.v_cache, bt, sl, qsl, cl, out)
            torch.cuda.synchronize()
            assert torch.equal(out.view(torch.int16), eager.view(torch.int16))


@pytest.mark.filterwarnings("ignore:The CUDA Graph is empty")
def test_a_plan_with_a_dynamic_tail_is_refused_on_a_capturing_stream():
    # the tail's ticket base is fixed at enqueue time, so a replay would leave the tail runs undone: the call says so
    b = W.build_batch(Hq=32, Hkv=8, hd=128, q_lens=[1, 1, 1], ctx_lens=[3000, 129, 900], num_blocks=300, seed=93)
    d = W.to_device(b)
    bt, sl, qsl, cl = device_meta(b)
    say("case: graph capture of a plan with a dynamic tail")
    out = torch.zeros((b.total_q, b.Hq, b.hd), dtype=torch.bfloat16, device="cuda")
    with B.Context(b.Hq, b.Hkv, b.hd, b.BS, b.num_blocks, b.max_blocks_per_seq) as ctx:
        ctx.set_option("plan_persistent", 1)
        ctx.set_option("decode_segments", 4)
        ctx.set_option("decode_tail_pct", 20)
        ctx.set_option("decode_tail_blocks", 4)
        ctx.plan(b.seq_lens, b.query_start_loc, b.ctx_lens)
        assert B.ooco_plan_dry_run(32, 8, 128, 16, b.max_blocks_per_seq, 256, 128 << 20, b.seq_lens, b.query_start_loc,
                                   b.ctx_lens, decode_segments=4, decode_tail_pct=20, decode_tail_blocks=4)["tail_runs"] > 0
        ctx.attn_mixed(d.q, d.k_cache, d.v_cache, bt, sl, qsl, cl, out)            # eager: fine
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                with pytest.raises(B.OocoError):
                    ctx.attn_mixed(d.q, d.k_cache, d.v_cache, bt, sl, qsl, cl, out, torch.cuda.current_stream())
        torch.cuda.synchronize()
        ctx.attn_mixed(d.q, d.k_cache, d.v_cache, bt, sl, qsl, cl, out)            # and eager calls go on working
        torch.cuda.synchronize()
        assert bool(torch.isfinite(out.float()).all())

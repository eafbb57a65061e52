"""ooco_attn_mixed under HIP graph capture: a planned call enqueues kernels and event fork/join only, so a
serving loop can capture a run of layers once and replay it.  Every replay is checked against the eager
result, with eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

from paper_2511_21862_amd import binding as B
from paper_2511_21862_amd import workloads as W

from gpu_util import device_meta, say

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("mixed", [False, True, "split", "lean", "in sequence"])
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
        # a batch this short runs its two kernels one after the other by default ("in sequence"); the other mixed
        # variants force the fork onto the context's second stream and the join, which is what a capture must record
        if mixed and mixed != "in sequence":
            ctx.set_option("overlap", 2)
        if mixed == "lean":                      # the register-lean pair of kernels of large mixed batches, forced here
            ctx.set_option("mixed_lean", 2)
        if mixed and mixed != "split":           # (the planner would cut even this short chunk's tiles in three)
            ctx.set_option("prefill_split", 1)
        ctx.plan(b.seq_lens, b.query_start_loc, b.ctx_lens)
        if mixed not in ("lean", "in sequence"):
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


def test_a_whole_step_replays_to_the_eager_result():
    # what a serving loop captures: the step's K/V appended, attention over the grown cache (through the context and
    # through the entry point that allocates nothing), the blocks of one sequence copied out to a staging pool
    b = W.build_batch(Hq=32, Hkv=8, hd=128, q_lens=[1, 80, 1, 1, 33], ctx_lens=[2000, 300, 15, 700, 0], num_blocks=260,
                      seed=94)
    d = W.to_device(b)
    bt, sl, qsl, cl = device_meta(b)
    say("case: graph capture of append + attention + block copy")
    g = torch.Generator(device="cuda").manual_seed(94)
    k_new = torch.empty((b.total_q, b.Hkv, b.hd), dtype=torch.bfloat16, device="cuda").normal_(0.0, 1.0, generator=g)
    v_new = torch.empty_like(k_new).normal_(0.0, 1.0, generator=g)
    nb0 = (int(b.seq_lens[0]) + 15) // 16
    src = torch.from_numpy(b.block_tables[0, :nb0].astype(np.int64)).cuda()
    dst = torch.arange(nb0, dtype=torch.int64, device="cuda")

    def pools():
        return (d.k_cache.clone(), d.v_cache.clone(), torch.zeros((nb0,) + tuple(d.k_cache.shape[1:]), dtype=torch.bfloat16, device="cuda"),
                torch.zeros((nb0,) + tuple(d.v_cache.shape[1:]), dtype=torch.bfloat16, device="cuda"))

    def step(ctx, kc, vc, ks, vs, out, out2, stream):
        ctx.kv_append(k_new, v_new, kc, vc, bt, qsl, cl, stream)
        ctx.attn_mixed(d.q, kc, vc, bt, sl, qsl, cl, out, stream)
        B.ooco_attn_mixed_static(b.Hq, b.Hkv, b.hd, b.BS, b.max_blocks_per_seq, 0.0, b.seq_lens, b.query_start_loc,
                                 b.ctx_lens, d.q, kc, vc, bt, sl, qsl, cl, out2, b.num_seqs, b.total_q, stream)
        ctx.kv_block_copy(kc, vc, ks, vs, src, dst, stream)

    bits = lambda t: t.view(torch.int16)
    with B.Context(b.Hq, b.Hkv, b.hd, b.BS, b.num_blocks, b.max_blocks_per_seq) as ctx:
        ctx.set_option("plan_persistent", 1)
        ctx.plan(b.seq_lens, b.query_start_loc, b.ctx_lens)
        kc_e, vc_e, ks_e, vs_e = pools()
        out_e = torch.empty((b.total_q, b.Hq, b.hd), dtype=torch.bfloat16, device="cuda")
        out2_e = torch.empty_like(out_e)
        step(ctx, kc_e, vc_e, ks_e, vs_e, out_e, out2_e, torch.cuda.current_stream())
        torch.cuda.synchronize()
        kc, vc, ks, vs = pools()
        out, out2 = torch.zeros_like(out_e), torch.zeros_like(out_e)
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            step(ctx, kc, vc, ks, vs, out, out2, side)                       # warm-up on the capture stream
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                step(ctx, kc, vc, ks, vs, out, out2, torch.cuda.current_stream())
        for rep in range(3):
            for t, t0 in ((kc, d.k_cache), (vc, d.v_cache)):
                t.copy_(t0)                                                  # the cache as it was before the step
            for t in (ks, vs, out, out2):
                t.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for got, want, what in ((kc, kc_e, "K pool"), (vc, vc_e, "V pool"), (out, out_e, "attention"),
                                    (out2, out2_e, "attention, no-alloc entry"), (ks, ks_e, "staged K"), (vs, vs_e, "staged V")):
                assert torch.equal(bits(got), bits(want)), f"replay {rep}: {what} differs from the eager step"


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

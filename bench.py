#!/usr/bin/env python3
"""Benchmark of the mixed-batch paged-attention step on ONE MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg5|cfg3|cfg2|cfg4|cfg3-prefill|cfg5-prefill|cfg3-decode|cfg5-decode|cfg4-copy|cfg4-copy-seq|cfg3-append|cfg5-append|cfg4-preempt|shape-<Hq>-<Hkv>-<hd>|mix-<c>x<r>+<d>[:<Hq>-<Hkv>]|pf-<c>x<r>@<ctx>[:<Hq>-<Hkv>]|pfx-[<n>x]<r>@<ctx>+...]

The default workload is the largest mixed configuration (cfg5: 2 online prefill chunks of 2048 tokens + 32 offline
decode sequences of 32K-131K tokens, 64/8 heads).

A step = one pass of the whole path over one synthetic batch already resident in HBM: host
planning (ooco_plan) + ooco_attn_mixed (prefill kernel, decode kernel with its in-kernel merge).  Steps
rotate over copies of the batch placed in disjoint physical blocks so that no step finds its KV
in the 256 MB last-level cache.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published


def read_traffic(kernel, workload):
    """HBM bytes per launch from the committed rocprofv3 counter summary of this kernel and workload
    (profiles/<kernel>_<workload>.md, line `traffic_hbm_bytes_per_launch = N`), or None."""
    import re

    path = os.path.join(ROOT, "profiles", f"{kernel}_{workload}.md")
    if not os.path.exists(path):
        return None
    m = re.search(r"^traffic_hbm_bytes_per_launch\s*=\s*(\d+)", open(path).read(), flags=re.M)
    return int(m.group(1)) if m else None


def make_workload(name):
    from paper_2511_21862_amd import workloads as W

    if name == "cfg2":
        return W.config2(device="cuda"), "decode"
    if name == "cfg2-n01":          # same shape, N(0,1) values (outputs O(0.05) instead of O(0.002))
        return W.config2(device="cuda", value_std=1.0), "decode"
    if name == "cfg3":
        return W.config3(device="cuda"), "decode"
    if name == "cfg3-prefill":
        return W.config3(device="cuda", n_decode=0), "prefill"
    if name == "cfg3-decode":       # the decode sequences of config 3 without its chunks
        return W.config3(device="cuda", decode_only=True), "decode"
    if name == "cfg5-decode":       # the decode sequences of config 5 without its chunks
        return W.config5(device="cuda", n_prefill=0), "decode"
    if name == "cfg4":
        return W.config4(device="cuda"), "decode"
    if name == "cfg5":
        return W.config5(device="cuda"), "decode"
    if name == "cfg5-prefill":
        return W.config5(device="cuda", n_decode=0, num_blocks=4096), "prefill"
    heads = (32, 8)
    if name.startswith(("mix-", "pf-")) and ":" in name:   # ...:<Hq>-<Hkv>: the same batch with other head counts
        name, shape = name.split(":")
        heads = tuple(int(x) for x in shape.split("-"))
        full = f"{name}:{shape}"
    else:
        full = name
    if name.startswith("mix-"):     # mix-<chunks>x<rows>+<decodes>: config 3's recipe with other proportions
        chunks, rest = name[4:].split("x")
        rows, ndec = rest.split("+")
        b = W.config3(device="cuda", n_prefill=int(chunks), chunk=int(rows), n_decode=int(ndec), Hq=heads[0], Hkv=heads[1])
        b.name = full
        return b, ("decode" if int(ndec) else "prefill")
    if name.startswith("pf-"):      # pf-<chunks>x<rows>@<ctx>: prefill chunks of equal length on equal prior context
        chunks, rest = name[3:].split("x")
        rows, ctx = rest.split("@")
        n, c, pc = int(chunks), int(rows), int(ctx)
        need = n * ((c + pc + 15) // 16)
        b = W.build_batch(Hq=heads[0], Hkv=heads[1], hd=128, q_lens=[c] * n, ctx_lens=[pc] * n, num_blocks=max(4096, 5 * need),
                          seed=3, device="cuda", name=full)
        return b, "prefill"
    if name.startswith("pfx-"):     # pfx-[<n>x]<rows>@<ctx>+[<n>x]<rows>@<ctx>+...: prefill chunks of several lengths and prior contexts
        ql, cx = [], []
        for item in name[4:].split("+"):
            n, rest = item.split("x") if "x" in item else ("1", item)
            rows, ctx = rest.split("@")
            ql += [int(rows)] * int(n)
            cx += [int(ctx)] * int(n)
        need = sum((c + q + 15) // 16 for q, c in zip(ql, cx))
        b = W.build_batch(Hq=32, Hkv=8, hd=128, q_lens=ql, ctx_lens=cx, num_blocks=max(4096, 5 * need), seed=3, device="cuda",
                          name=name)
        return b, ("decode" if 1 in ql else "prefill")     # (items of one row are decode sequences)
    if name.startswith("shape-"):   # shape-<Hq>-<Hkv>-<hd>: 256 decode sequences of 512-4096 tokens with another head shape
        Hq, Hkv, hd = (int(x) for x in name.split("-")[1:4])
        rng = np.random.default_rng(77)
        seq = W.uniform_lengths(rng, 256, 512, 4096)
        return W.build_batch(Hq=Hq, Hkv=Hkv, hd=hd, q_lens=np.ones(256, np.int32), ctx_lens=seq - 1, num_blocks=98304,
                             seed=77, device="cuda", rng=rng, name=f"decode256-{Hq}-{Hkv}-{hd}"), "decode"
    raise SystemExit(f"unknown workload {name}")


def cpu_baseline(b, budget_units=45.0e6):
    """The oracle as it stands, timed on this machine's host cores on a bounded sample of the same batch: every
    prefill chunk (while they fit the budget) plus every k-th decode sequence, k the smallest stride that keeps
    the sample within the budget.  One unit = one (query row, key) pair over 32 query heads; the C oracle does
    about two million of them per second on 16 cores, so the default budget is 20-25 s of CPU work."""
    from oracle import ref_c
    from paper_2511_21862_amd import workloads as W

    ql, ctx = b.q_lens.astype(np.float64), b.ctx_lens.astype(np.float64)
    units = (ql * ctx + ql * (ql + 1) / 2.0) * (b.Hq / 32.0)
    chunks = [int(i) for i in np.flatnonzero(b.q_lens > 1)]
    dec = [int(i) for i in np.flatnonzero(b.q_lens == 1)]
    keep, acc = [], 0.0
    for i in chunks:
        if acc + units[i] <= budget_units or not keep:
            keep.append(i)
            acc += units[i]
    n_chunks = len(keep)
    stride = 0
    if dec:
        stride = 1
        while units[dec[::stride]].sum() > max(budget_units - acc, 0.0) and stride < len(dec):
            stride += 1
        if units[dec[::stride]].sum() <= max(budget_units - acc, 0.0) or not keep:
            keep += dec[::stride]
            acc += float(units[dec[::stride]].sum())
        else:
            stride = 0
    sub = W.subset(b, keep)
    args = (sub.q, sub.k_cache, sub.v_cache, sub.block_tables, sub.seq_lens, sub.query_start_loc, sub.ctx_lens)
    times = []
    threads = 0
    for _ in range(3 if acc < 8.0e6 else 1):
        t0 = time.perf_counter()
        _, threads = ref_c.attn_mixed(*args, return_threads=True)
        times.append(time.perf_counter() - t0)
    t = float(np.median(times))
    what = f"{n_chunks} of {len(chunks)} prefill chunks"
    what += f" + every {stride}. decode sequence ({len(keep) - n_chunks} of {len(dec)})" if stride else " + no decode sequence"
    return {
        "value": sub.total_q / t, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
        "sample": f"{what}: {sub.total_q} of {b.total_q} query tokens, {int(sub.seq_lens.sum())} KV tokens, "
                  f"float64 C/OpenMP oracle, {'median of 3 runs' if len(times) > 1 else 'one run'}, {t:.3f} s",
    }


def bench_block_copy(a):
    """Row B1: ooco_kv_block_copy of the blocks of config 4's 64 evicted sequences into a staging
    pool (one kernel per step; steps alternate between two staging pools)."""
    import torch

    from oracle import ref_c
    from paper_2511_21862_amd import accounting
    from paper_2511_21862_amd import binding as B
    from paper_2511_21862_amd import workloads as W

    b = W.config4(device="cuda")
    src = W.victim_block_ids(b, b.extra["victims"])
    n = len(src)
    rng = np.random.default_rng(44)
    stage_blocks = n + 64
    # destination ids: a random subset of the staging pool (default: a staging pool whose free list is in
    # no particular order), or 0..n-1 ("cfg4-copy-seq": a freshly set up staging pool)
    if a.workload == "cfg4-copy-seq":
        dsts = [torch.arange(n, dtype=torch.int64, device="cuda") for _ in range(2)]
    else:
        dsts = [torch.from_numpy(rng.permutation(stage_blocks)[:n].astype(np.int64)).cuda() for _ in range(2)]
    stages = [(torch.empty((stage_blocks,) + tuple(b.k_cache.shape[1:]), dtype=torch.bfloat16, device="cuda"),
               torch.empty((stage_blocks,) + tuple(b.v_cache.shape[1:]), dtype=torch.bfloat16, device="cuda"))
              for _ in range(2)]
    src_d = torch.from_numpy(src).cuda()
    ctx = B.Context(b.Hq, b.Hkv, b.hd, b.BS, b.num_blocks, b.max_blocks_per_seq)
    for o in a.opt:
        k, v = o.split("=")
        ctx.set_option(k, int(v))
    stream = torch.cuda.current_stream()

    def step(i):
        ks, vs = stages[i % 2]
        ctx.kv_block_copy(b.k_cache, b.v_cache, ks, vs, src_d, dsts[i % 2], stream)

    for i in range(a.warmup):
        step(i)
    torch.cuda.synchronize()
    # one kernel per step, launched back to back: the timed region is bracketed by one pair of HIP events on the
    # launch stream (torch's current stream here), region time / steps = the kernel's average launch duration
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record(stream)
    for i in range(a.steps):
        step(i)
    ev1.record(stream)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / a.steps
    kms = ev0.elapsed_time(ev1) / a.steps
    nbytes = accounting.block_copy_bytes(n, b.Hkv, b.hd, b.BS)
    tokens = int(b.seq_lens[b.extra["victims"]].sum())
    line = {
        "metric": "KV block copy (preemption eviction) tokens/s + achieved HBM GB/s (% of peak), 1 MI355X",
        "value": tokens / dt, "unit": "tokens/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": dt * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8", "data": "synthetic",
        "config": {"workload": "cfg4-eviction-copy", "bench_name": a.workload, "victim_seqs": len(b.extra["victims"]),
                   "blocks": n, "kv_tokens": tokens, "Hkv": b.Hkv, "head_dim": b.hd, "block_size": b.BS},
        "roofline": {"bound": "hbm", "kernel": "block_copy_kernel", "achieved": nbytes / (kms * 1e-3) / 1e9,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": nbytes / (kms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "traffic": None, "algorithmic_bytes_per_launch": nbytes, "kernel_ms": kms},
    }
    line["roofline"]["traffic"] = read_traffic("block_copy_kernel", a.workload)
    if not a.no_cpu_baseline:
        # host memcpy of a bounded sample of the same id lists (the C oracle's block copy)
        m = min(n, 2048)
        kh = np.zeros((m,) + tuple(b.k_cache.shape[1:]), np.uint16)
        vh = np.zeros((m,) + tuple(b.v_cache.shape[1:]), np.uint16)
        ksrc, vsrc = np.ones_like(kh), np.ones_like(vh)
        ids = np.arange(m, dtype=np.int64)
        perm = rng.permutation(m).astype(np.int64)
        ts = []
        for _ in range(3):
            t1 = time.perf_counter()
            ref_c.block_copy(ksrc, vsrc, kh, vh, ids, perm)
            ts.append(time.perf_counter() - t1)
        t = float(np.median(ts))
        line["cpu_baseline"] = {"value": m * b.BS / t, "unit": "tokens/s", "cores": 1, "kind": "oracle",
                                "sample": f"{m} of {n} blocks, host memcpy per block pair (C oracle), median of 3, "
                                          f"{t:.4f} s each, {accounting.block_copy_bytes(m, b.Hkv, b.hd, b.BS) / t / 1e9:.1f} GB/s"}
    ctx.close()
    print(json.dumps(line), flush=True)


def bench_append(a):
    """ooco_kv_append of one step's tokens of config 3 or 5 (the step that precedes the attention call);
    steps rotate over copies of the batch dealt from disjoint physical blocks."""
    import torch

    from oracle import ref_numpy
    from paper_2511_21862_amd import accounting
    from paper_2511_21862_amd import binding as B
    from paper_2511_21862_amd import workloads as W

    b = (W.config3 if a.workload.startswith("cfg3") else W.config5)(device="cuda")
    dev = lambda x: torch.from_numpy(np.ascontiguousarray(x)).cuda()
    bts = [dev(t) for t in W.replica_tables(b, 4)]
    qsl, cl = dev(b.query_start_loc), dev(b.ctx_lens)
    g = torch.Generator(device="cuda").manual_seed(11)
    k_new = torch.randn((b.total_q, b.Hkv, b.hd), generator=g, device="cuda").to(torch.bfloat16)
    v_new = torch.randn((b.total_q, b.Hkv, b.hd), generator=g, device="cuda").to(torch.bfloat16)
    ctx = B.Context(b.Hq, b.Hkv, b.hd, b.BS, b.num_blocks, b.max_blocks_per_seq)
    for o in a.opt:
        k, v = o.split("=")
        ctx.set_option(k, int(v))
    stream = torch.cuda.current_stream()

    def step(i):
        ctx.kv_append(k_new, v_new, b.k_cache, b.v_cache, bts[i % len(bts)], qsl, cl, stream)

    for i in range(a.warmup):
        step(i)
    torch.cuda.synchronize()
    # one kernel per step, launched back to back: the timed region is bracketed by one pair of HIP events on the
    # launch stream (torch's current stream here), region time / steps = the kernel's average launch duration
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record(stream)
    for i in range(a.steps):
        step(i)
    ev1.record(stream)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / a.steps
    kms = ev0.elapsed_time(ev1) / a.steps
    nbytes = 2 * b.total_q * accounting.per_token_kv_bytes(b.Hkv, b.hd)      # new vectors read + slots written
    line = {
        "metric": "KV append tokens/s + achieved HBM GB/s (% of peak), 1 MI355X",
        "value": b.total_q / dt, "unit": "tokens/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": dt * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8", "data": "synthetic",
        "config": {"workload": b.name + "-append", "bench_name": a.workload, "q_tokens": b.total_q, "num_seqs": b.num_seqs,
                   "Hkv": b.Hkv, "head_dim": b.hd, "block_size": b.BS},
        "roofline": {"bound": "hbm", "kernel": "kv_append_kernel", "achieved": nbytes / (kms * 1e-3) / 1e9,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": nbytes / (kms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "traffic": read_traffic("kv_append_kernel", a.workload), "algorithmic_bytes_per_launch": nbytes,
                     "kernel_ms": kms},
    }
    if not a.no_cpu_baseline:
        # the numpy oracle on a bounded sample: the first sequences up to about 64 tokens
        n = int(np.searchsorted(b.query_start_loc, 64, side="right"))
        n = max(1, min(n, b.num_seqs))
        s = W.subset(b, list(range(n)))
        kn = np.zeros((s.total_q, b.Hkv, b.hd), np.uint16)
        t1 = time.perf_counter()
        ref_numpy.kv_append(kn, kn, s.k_cache, s.v_cache, s.block_tables, s.query_start_loc, s.ctx_lens)
        t = time.perf_counter() - t1
        line["cpu_baseline"] = {"value": s.total_q / t, "unit": "tokens/s", "cores": 1, "kind": "oracle",
                                "sample": f"first {n} sequences ({s.total_q} tokens), numpy definition, {t:.2f} s"}
    ctx.close()
    print(json.dumps(line), flush=True)


def bench_preempt(a):
    """Layer-level preemption of an offline decode iteration by an online prefill chunk (paper Section 3.4.1),
    attention layers only, through the package's preemption driver (paper_2511_21862_amd/preempt.py): config 4's
    512 offline decode sequences run a 32-layer iteration, one ooco_attn_mixed per layer, enqueued with a run-ahead
    of at most two layers; a timer thread raises the preemption flag somewhere inside the iteration and the loop
    sees it before its next enqueue.  The online request (2048 new tokens on 4096 tokens of context = 384 KV
    blocks, none free) names its victims through ooco_eviction_victims, once on a compute-bound node (long
    requests first) and once on a memory-bound one (short first); their blocks go to a staging pool through
    ooco_kv_block_copy, the chunk runs its 32 attention layers in the freed blocks, the victims come back, and the
    iteration resumes at the layer it stopped at."""
    import threading

    import torch

    from paper_2511_21862_amd import binding as B
    from paper_2511_21862_amd import preempt as P
    from paper_2511_21862_amd import workloads as W

    L = 32
    b = W.config4(device="cuda")
    dev = lambda x: torch.from_numpy(np.ascontiguousarray(x)).cuda()
    bt, sl, qsl, cl = dev(b.block_tables), dev(b.seq_lens), dev(b.query_start_loc), dev(b.ctx_lens)
    out = torch.empty((b.total_q, b.Hq, b.hd), dtype=torch.bfloat16, device="cuda")
    c_len, c_ctx = 2048, 4096
    c_nb = (c_len + c_ctx + 15) // 16
    c_q = torch.randn((c_len, b.Hq, b.hd), device="cuda").to(torch.bfloat16)
    c_out = torch.empty_like(c_q)
    stream = torch.cuda.current_stream()
    dec = B.Context(b.Hq, b.Hkv, b.hd, b.BS, b.num_blocks, b.max_blocks_per_seq)
    onl = B.Context(b.Hq, b.Hkv, b.hd, b.BS, b.num_blocks, b.max_blocks_per_seq)
    dec.set_option("plan_persistent", 1)
    onl.set_option("plan_persistent", 1)
    dec.plan(b.seq_lens, b.query_start_loc, b.ctx_lens)
    c_seq, c_qsl, c_cx = np.array([c_len + c_ctx], np.int32), np.array([0, c_len], np.int32), np.array([c_ctx], np.int32)
    onl.plan(c_seq, c_qsl, c_cx)

    def layer(_l):
        dec.attn_mixed(b.q, b.k_cache, b.v_cache, bt, sl, qsl, cl, out, stream)

    def iteration(bs_sat=None, delay=None):
        """One iteration; with bs_sat a timer raises the flag `delay` seconds after the start."""
        torch.cuda.synchronize()
        flag = P.PreemptFlag() if bs_sat is not None else None
        timer = None

        def on_preempt(_next_layer):
            t0 = time.perf_counter()
            ev = P.Eviction(dec, b.seq_lens, b.block_tables, c_nb, bs_sat)
            k_st, v_st = P.staging_pools(b, ev.num_blocks)
            t1 = time.perf_counter()
            ev.evict(b.k_cache, b.v_cache, k_st, v_st, stream)
            stream.synchronize()
            t2 = time.perf_counter()
            c_bt = np.full((1, b.max_blocks_per_seq), -1, np.int32)
            c_bt[0, :c_nb] = ev.block_ids[:c_nb]
            meta = [dev(c_bt), dev(c_seq), dev(c_qsl), dev(c_cx)]
            for _ in range(L):
                onl.attn_mixed(c_q, b.k_cache, b.v_cache, *meta, c_out, stream)
            stream.synchronize()
            t3 = time.perf_counter()
            ev.restore(b.k_cache, b.v_cache, k_st, v_st, stream)
            stream.synchronize()
            t4 = time.perf_counter()
            return dict(victims=len(ev.victims), victim_blocks=ev.num_blocks, select_ms=(t1 - t0) * 1e3,
                        evict_ms=(t2 - t1) * 1e3, online_chunk_layers_ms=(t3 - t2) * 1e3, restore_ms=(t4 - t3) * 1e3)

        if flag is not None:
            timer = threading.Timer(delay, flag.raise_now)
            timer.start()
        t0 = time.perf_counter()
        rep = P.run_layers(L, layer, stream, flag=flag, on_preempt=on_preempt)
        dt = time.perf_counter() - t0
        if timer is not None:
            timer.join()
        return dt, rep

    for _ in range(max(1, a.warmup // 8)):
        iteration()
    n_it = max(3, a.steps // 20)
    plain = [iteration()[0] for _ in range(n_it)]
    t_plain = float(np.median(plain))
    want = out.clone()
    regimes = {}
    rng = np.random.default_rng(9)
    for name, bs_sat in (("compute_bound", 256), ("memory_bound", 4096)):
        runs = [iteration(bs_sat, float(rng.uniform(0.1, 0.8)) * t_plain) for _ in range(n_it)]
        runs = [(t, r) for t, r in runs if r is not None]
        keys = [k for k in runs[0][1] if k != "resumed_at_layer"]
        regimes[name] = {k: float(np.median([r[k] for _, r in runs])) for k in keys}
        regimes[name]["preempted_iteration_ms"] = float(np.median([t for t, _ in runs])) * 1e3
        regimes[name]["preemptions"] = len(runs)
        regimes[name]["bs_sat"] = bs_sat
    same = bool(torch.equal(want.view(torch.int16), out.view(torch.int16)))
    line = {
        "metric": "layer-level preemption of an offline decode iteration (attention layers only), 1 MI355X",
        "value": b.total_q * L / t_plain, "unit": "tokens/s", "n_gpus": 1, "steps": len(plain), "warmup": a.warmup,
        "ms_per_step": t_plain * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "cfg4-preempt", "layers": L, "decode_seqs": b.num_seqs, "online_chunk": [c_len, c_ctx],
                   "online_chunk_blocks": c_nb, "run_ahead_layers": 2},
        "iteration_ms": t_plain * 1e3, "layer_ms": t_plain * 1e3 / L,
        "preempt_latency_ms": {k: v["preempt_latency_ms"] for k, v in regimes.items()},
        "preemption": regimes, "output_after_preemption_bit_identical": same,
    }
    dec.close()
    onl.close()
    print(json.dumps(line), flush=True)


def wg_timeline(ctx, b, run_step, torch, reps=5):
    """One traced launch of a prefill-only batch: when every workgroup started and ended (option "trace"; the
    kernel's own 100 MHz time stamps), summed up per eighth of the dispatch order and per compute unit.  Median
    over `reps` launches of every figure, in microseconds from the first workgroup's start."""
    from paper_2511_21862_amd import binding as B

    tiles = B.ooco_plan_dry_run(b.Hq, b.Hkv, b.hd, b.BS, b.max_blocks_per_seq, torch.cuda.get_device_properties(0).multi_processor_count,
                                512 << 20, h_seq_lens=b.seq_lens, h_query_start_loc=b.query_start_loc,
                                h_ctx_lens=b.ctx_lens)["prefill_tiles"]
    steps_tile = (tiles[:, 3] + tiles[:, 2] + 63) // 64
    ctx.set_option("trace", 1)
    rows = []
    for _ in range(reps):
        run_step()
        torch.cuda.synchronize()
        raw = ctx.trace_read()
        t0 = raw[:, 0].astype(np.float64) / 100.0
        t1 = raw[:, 3].astype(np.float64) / 100.0
        cu = raw[:, 1].astype(np.int64)
        base = t0.min()
        t0, t1 = t0 - base, t1 - base
        n = len(t0)
        # (with split tiles the list holds (tile, part) entries in an order of its own: no per-workgroup steps then, -1)
        steps = np.repeat(steps_tile, n // len(steps_tile)) if n == len(steps_tile) * b.Hkv else np.full(n, -1.0)
        r = {"workgroups": n, "compute_units": int(len(np.unique(cu))), "span_us": float(t1.max()),
             "all_first_round_started_by_us": float(np.sort(t0)[min(n, 2 * len(np.unique(cu))) - 1]),
             "slot_busy_us_mean": float((t1 - t0).sum() / (2 * len(np.unique(cu)))),
             "steps_total": int(steps_tile.sum()) * b.Hkv}
        ends = np.array([t1[cu == c].max() for c in np.unique(cu)])
        r["cu_last_end_us_min_mean_max"] = [float(ends.min()), float(ends.mean()), float(ends.max())]
        eighth = []
        for k in range(8):
            sel = slice(k * n // 8, (k + 1) * n // 8)
            eighth.append([float(steps[sel].mean()), float(t0[sel].min()), float(t0[sel].max()), float(t1[sel].min()),
                           float(t1[sel].max()), float((t1 - t0)[sel].mean())])
        r["eighths_steps_start_min_max_end_min_max_duration_mean"] = eighth
        # phases of a workgroup (16 bits each in the third stamp, 10 ns since its start): tile looked up, first loads
        # sent off, first tiles arrived, last step done; the epilogue is what remains until its end.  Medians over
        # the first round (the workgroups that start on an idle GPU) and over the later ones.
        x = raw[:, 2].astype(np.uint64)
        ph = np.stack([((x >> np.uint64(16 * k)) & np.uint64(0xFFFF)).astype(np.float64) / 100.0 for k in range(4)], axis=1)
        order = np.argsort(t0, kind="stable")
        first = order[: min(n, 2 * len(np.unique(cu)))]
        later = order[min(n, 2 * len(np.unique(cu))):]
        for name, idx in (("first_round", first), ("later_rounds", later)):
            idx = idx[x[idx] != 0]
            if len(idx):
                r[f"phases_us_{name}_lookup_issued_landed_loopend_epilogue"] = (
                    np.median(ph[idx], axis=0).tolist() + [float(np.median((t1 - t0)[idx] - ph[idx, 3]))])
        rows.append(r)
    ctx.set_option("trace", 0)
    med = lambda key: np.median(np.array([r[key] for r in rows], dtype=np.float64), axis=0)
    outd = {k: (med(k).tolist() if isinstance(rows[0][k], list) else float(med(k))) for k in rows[0]}
    outd["launches"] = reps
    return outd


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg5")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--replan-every-step", type=int, default=1)
    ap.add_argument("--opt", action="append", default=[], help="name=value passed to ooco_set_option")
    ap.add_argument("--wg-timeline", action="store_true",
                    help="prefill-only workloads: add the workgroups' start and end times of one traced launch to the line")
    a = ap.parse_args()
    if a.gpus != 1:
        raise SystemExit("bench.py: this build measures one GPU only (no collectives, no sharding); run with --gpus 1")

    import torch

    from paper_2511_21862_amd import accounting
    from paper_2511_21862_amd import binding as B
    from paper_2511_21862_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if a.workload in ("cfg4-copy", "cfg4-copy-seq"):
        return bench_block_copy(a)
    if a.workload in ("cfg3-append", "cfg5-append"):
        return bench_append(a)
    if a.workload == "cfg4-preempt":
        return bench_preempt(a)
    b, dominant = make_workload(a.workload)
    work = accounting.batch_work(b.Hq, b.Hkv, b.hd, b.BS, b.seq_lens, b.q_lens)
    mixed = work["prefill_chunks"] > 0 and work["decode_seqs"] > 0
    tables = W.replica_tables(b, 4)
    dev = lambda x: torch.from_numpy(np.ascontiguousarray(x)).cuda()
    bts = [dev(t) for t in tables]
    sl, qsl, cl = dev(b.seq_lens), dev(b.query_start_loc), dev(b.ctx_lens)
    out = torch.empty((b.total_q, b.Hq, b.hd), dtype=torch.bfloat16, device="cuda")
    ctx = B.Context(b.Hq, b.Hkv, b.hd, b.BS, b.num_blocks, b.max_blocks_per_seq, workspace_bytes=512 << 20)
    for o in a.opt:
        k, v = o.split("=")
        ctx.set_option(k, int(v))
    if not a.replan_every_step:
        ctx.set_option("plan_persistent", 1)
    stream = torch.cuda.current_stream()
    host_us = {"plan": 0.0, "launch": 0.0}

    def step(i, clock=False):
        t0 = time.perf_counter() if clock else 0.0
        if a.replan_every_step or i == 0:
            ctx.plan(b.seq_lens, b.query_start_loc, b.ctx_lens)
        t1 = time.perf_counter() if clock else 0.0
        ctx.attn_mixed(b.q, b.k_cache, b.v_cache, bts[i % len(bts)], sl, qsl, cl, out, stream)
        if clock:
            host_us["plan"] += (t1 - t0) * 1e6
            host_us["launch"] += (time.perf_counter() - t1) * 1e6

    step(0)
    info = ctx.plan_info()
    kernels = ctx.plan_kernels()            # as rocprofv3 names them, decode first
    for i in range(a.warmup):
        step(i)
    torch.cuda.synchronize()
    # The timed region is also bracketed by one pair of HIP events on the launch stream (every kernel of a step
    # is ordered inside it: the side stream is forked from and joined into this stream), so region time / steps
    # is the GPU time of one step with its kernels running exactly as in the product path; for a batch with one
    # kind of work it is that one kernel's average launch duration.
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record(stream)
    for i in range(a.steps):
        step(i)
    ev1.record(stream)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / a.steps * 1e3
    region_ms_per_step = ev0.elapsed_time(ev1) / a.steps
    # host cost of planning and of enqueueing, one step at a time with the GPU idle in between
    n_host = min(a.steps, 50)
    for i in range(n_host):
        step(i, clock=True)
        torch.cuda.synchronize()
    host_us = {k: v / n_host for k, v in host_us.items()}

    # per-kernel durations: the same K steps again with HIP events recorded inside the library around each kernel
    # on the stream it runs on (launch order and overlap unchanged), so that the event records stay out of `value`
    ctx.set_option("profile", 1)
    prof = {"prefill_ms": 0.0, "decode_ms": 0.0, "call_ms": 0.0, "calls": 0}
    per_call = []
    done = 0
    while done < a.steps:
        n = min(512, a.steps - done)
        for i in range(n):
            step(done + i)
        r = ctx.profile_read_calls()
        for k in prof:
            prof[k] += r[k]
        per_call.append(r["per_call"])
        done += n
    ctx.set_option("profile", 0)
    kern = {k: prof[k] / max(prof["calls"], 1) for k in ("prefill_ms", "decode_ms", "call_ms")}
    kern["per_launch_events"] = dict(kern)
    pc = np.concatenate(per_call) if per_call else np.zeros((0, 3))
    if len(pc):      # spread of the per-launch event times: p10 / median / p90
        kern["prefill_ms_p10_p50_p90"] = [float(x) for x in np.percentile(pc[:, 0], [10, 50, 90])]
        kern["decode_ms_p10_p50_p90"] = [float(x) for x in np.percentile(pc[:, 1], [10, 50, 90])]
        kern["call_ms_p10_p50_p90"] = [float(x) for x in np.percentile(pc[:, 2], [10, 50, 90])]
    if work["prefill_chunks"] == 0:
        kern["decode_ms"] = min(kern["decode_ms"], region_ms_per_step)
    elif work["decode_seqs"] == 0:
        kern["prefill_ms"] = min(kern["prefill_ms"], region_ms_per_step)
    kern["region_ms_per_step"] = region_ms_per_step
    kern["overlapped"] = bool(mixed)

    whole_step_frac = work["bytes_total"] / (region_ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS
    if dominant == "decode":
        # the dominant kernel as it runs in the step (beside the prefill kernel when the batch holds both kinds)
        alg = work["bytes_decode"]
        dur = kern["decode_ms"] * 1e-3
        achieved = alg / dur / 1e9 if dur > 0 else 0.0
        roofline = {"bound": "hbm", "kernel": kernels[0], "achieved": achieved, "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                    "algorithmic_bytes_per_launch": alg, "kernel_ms": kern["decode_ms"],
                    "whole_step_frac": whole_step_frac, "whole_step_bytes": work["bytes_total"],
                    "whole_step_ms": region_ms_per_step}
    else:
        alg = work["flops_causal_prefill"]
        dur = kern["prefill_ms"] * 1e-3
        achieved = alg / dur / 1e12 if dur > 0 else 0.0
        roofline = {"bound": "mfma", "kernel": kernels[-1], "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                    "algorithmic_flops_per_launch": alg, "kernel_ms": kern["prefill_ms"]}
    roofline["traffic"] = read_traffic(roofline["kernel"].split("<")[0], a.workload)

    line = {
        "metric": "mixed-batch attention tokens/s + achieved HBM GB/s (% of peak), 1 MI355X",
        "value": b.total_q / (dt / a.steps),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": b.name, "bench_name": a.workload, "num_seqs": b.num_seqs, "decode_seqs": work["decode_seqs"],
                   "prefill_chunks": work["prefill_chunks"], "q_tokens": work["q_tokens"], "kv_tokens": work["kv_tokens"],
                   "Hq": b.Hq, "Hkv": b.Hkv, "head_dim": b.hd, "block_size": b.BS, "replicas": len(bts),
                   "plan": info, "kernels": kernels, "replan_every_step": bool(a.replan_every_step)},
        "hbm_gbs_whole_step": work["bytes_total"] / (dt / a.steps) / 1e9,
        "hbm_frac_whole_step": work["bytes_total"] / (dt / a.steps) / 1e9 / HBM_PEAK_GBS,
        "kv_tokens_per_s": work["kv_tokens"] / (dt / a.steps),
        "tflops_causal_whole_step": work["flops_causal"] / (dt / a.steps) / 1e12,
        "plan_host_us": host_us["plan"], "launch_host_us": host_us["launch"],
        "kernel_ms": kern,
        "roofline": roofline,
    }
    if a.wg_timeline and work["decode_seqs"] == 0:
        line["wg_timeline"] = wg_timeline(ctx, b, lambda: step(0), torch)
    if not a.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(b)
    ctx.close()
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()

"""Fits the environment parameters of the attention latency model (ooco_predict_latency: F_ap, F_ad, M_a,
O_p, O_d) to this library's own measured call times on the GPU it runs on, and reports the model's error.

    python -m paper_2511_21862_amd.fit_model [--out-json FILE] [--out-md FILE] [--reps 15]

The paper obtains these parameters "through a small amount of profiling data" and reports an average absolute
error of about 5 % for whole model iterations (Section 3.3.2).  Here the sweep covers decode-only batches
(batch size x context length) and prefill-only batches (chunks x chunk length x prior context); mixed batches
are held out for validation.  Times are HIP-event times around one ooco_attn_mixed call on its stream (plan
made once, outside) over bursts of 8 calls enqueued back to back, median over the repetitions, KV pool far larger
than the caches.  Only batches that can occupy the whole GPU enter the fit; the others are reported beside it.
Predictions are made by the library (ooco_predict_latency); this script only searches the five parameters."""
from __future__ import annotations

import argparse
import json

import numpy as np


def _measure(torch, B, ctx, pool, Hq, Hkv, hd, q_lens, ctx_lens, perm, reps, overlap=1):
    """Median event time (s) of one call on a batch dealt from the pool's block permutation."""
    ql = np.asarray(q_lens, np.int32)
    cx = np.asarray(ctx_lens, np.int32)
    seq = ql + cx
    nb = (seq + 15) // 16
    assert int(nb.sum()) <= len(perm), "sweep point larger than the pool"
    maxb = ctx.max_blocks
    bt = np.full((len(ql), maxb), -1, np.int32)
    pos = 0
    for i, n in enumerate(nb):
        bt[i, :n] = perm[pos:pos + n]
        pos += int(n)
    qsl = np.zeros(len(ql) + 1, np.int32)
    qsl[1:] = np.cumsum(ql)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    bt_d, sl_d, qsl_d, cl_d = dev(bt), dev(seq), dev(qsl), dev(cx)
    T = int(ql.sum())
    q = torch.randn((T, Hq, hd), device="cuda").to(torch.bfloat16)
    out = torch.empty_like(q)
    ctx.set_option("overlap", overlap)
    ctx.set_option("plan_persistent", 1)
    ctx.plan(seq, qsl, cx)
    stream = torch.cuda.current_stream()
    ts = []
    burst = 8      # calls are enqueued back to back, as a layer loop does; time per call = burst time / burst
    for r in range(reps + 2):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(burst):
            ctx.attn_mixed(q, pool[0], pool[1], bt_d, sl_d, qsl_d, cl_d, out, stream)
        e1.record(stream)
        torch.cuda.synchronize()
        if r >= 2:
            ts.append(e0.elapsed_time(e1) * 1e-3 / burst)
    return float(np.median(ts)), qsl, cx


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--out-json", default=None)
    ap.add_argument("--out-md", default=None)
    ap.add_argument("--reps", type=int, default=15)
    ap.add_argument("--pool-blocks", type=int, default=196608)
    a = ap.parse_args()
    import torch
    from scipy.optimize import least_squares

    from . import binding as B

    Hq, Hkv, hd, BS = 32, 8, 128, 16
    NB, maxb = a.pool_blocks, 8192
    g = torch.Generator(device="cuda").manual_seed(1)
    pool = (torch.randn((NB, Hkv, hd // 8, BS, 8), generator=g, device="cuda").to(torch.bfloat16),
            torch.randn((NB, Hkv, hd, BS), generator=g, device="cuda").to(torch.bfloat16))
    perm = np.random.default_rng(1).permutation(NB).astype(np.int32)
    ctx = B.Context(Hq, Hkv, hd, BS, NB, maxb)
    ctx.max_blocks = maxb
    rng = np.random.default_rng(2)

    points = []   # (kind, description, q_lens, ctx_lens)
    for bs in (1, 8, 32, 128, 512):
        for L in (256, 1024, 4096, 16384, 65536):
            if bs * L <= 2_600_000 and L <= maxb * BS:
                lens = np.maximum(1, rng.integers(L // 2, L + L // 2 + 1, size=bs))       # ragged around L
                points.append(("decode", f"{bs} x ~{L}", np.ones(bs, np.int32), lens - 1))
    for n in (1, 4, 8):
        for c in (128, 512, 2048):
            for pc in (0, 2048, 8192):
                points.append(("prefill", f"{n} x {c} on {pc}", np.full(n, c, np.int32), np.full(n, pc, np.int32)))
    held = [
        ("mixed", "8 x 512 on ~1K + 128 x ~2.7K", np.r_[np.full(8, 512), np.ones(128, int)],
         np.r_[rng.integers(0, 2048, 8), rng.integers(500, 5000, 128)]),
        ("mixed", "2 x 2048 on 4096 + 32 x ~64K", np.r_[np.full(2, 2048), np.ones(32, int)],
         np.r_[np.full(2, 4096), rng.integers(32768, 100000, 32)]),
        ("mixed", "1 x 256 on 0 + 256 x ~1K", np.r_[np.full(1, 256), np.ones(256, int)],
         np.r_[np.zeros(1, int), rng.integers(512, 1536, 256)]),
    ]
    rows = []
    for kind, desc, ql, cx in points:
        t, qsl, cxa = _measure(torch, B, ctx, pool, Hq, Hkv, hd, ql, cx, perm, a.reps)
        # the model's regime: enough work to occupy the whole GPU (a roofline has no notion of idle CUs)
        full = (int((ql + cx).sum()) >= 32768 and len(ql) >= 8) if kind == "decode" else int(ql.sum()) >= 1024
        rows.append(dict(kind=kind, desc=desc, t=t, qsl=qsl, cx=cxa, full=full))
        print(f"measured {kind:8s} {desc:28s} {t * 1e6:10.1f} us", flush=True)
    val = []
    for kind, desc, ql, cx in held:
        for ov in (0, 1):
            t, qsl, cxa = _measure(torch, B, ctx, pool, Hq, Hkv, hd, ql, cx, perm, a.reps, overlap=ov)
            val.append(dict(kind=kind, desc=desc + (" (kernels overlapped)" if ov else " (kernels in sequence)"), t=t, qsl=qsl,
                            cx=cxa))
            print(f"measured {kind:8s} {val[-1]['desc']:58s} {t * 1e6:10.1f} us", flush=True)

    names = ("F_ap", "F_ad", "M_a", "O_p", "O_d")
    fit_rows = [r for r in rows if r["full"]]
    small = [r for r in rows if not r["full"]]
    results = {}
    lines = ["# Attention latency model fitted on MI355X (`ooco_predict_latency`)\n",
             "Command: `python -m paper_2511_21862_amd.fit_model` (32 query heads, 8 KV heads, head_dim 128, bf16; "
             f"pool of {NB} blocks; median of {a.reps} HIP-event-timed bursts of 8 calls per point).  {len(fit_rows)} batches "
             f"that can occupy the whole GPU enter the fit; {len(small)} smaller ones (decode below 8 sequences or 32K KV "
             "tokens, prefill below 1024 query rows) are reported beside it: they leave compute units idle (one workgroup "
             "walks a long context alone), which a roofline with one constant overhead cannot express.\n"]
    for causal in (False, True):
        def pred(theta, r):
            p = dict(zip(names, np.exp(theta)))
            return B.ooco_predict_latency(p, Hq, Hkv, hd, r["qsl"], r["cx"], causal_flops=causal)["latency"]

        def resid(theta, which=None):
            return np.array([pred(theta, r) / r["t"] - 1.0 for r in (fit_rows if which is None else which)])

        x0 = np.log([1.0e15, 2.0e14, 5.0e12, 1.0e-5, 1.0e-5])
        theta = least_squares(resid, x0, method="trf", x_scale=1.0, diff_step=1e-3).x
        params = dict(zip(names, (float(v) for v in np.exp(theta))))
        err, err_small = np.abs(resid(theta)), np.abs(resid(theta, small))
        verr = np.array([abs(pred(theta, r) / r["t"] - 1.0) for r in val])
        key = "causal_flops" if causal else "table2_flops"
        results[key] = dict(params=params, mean_abs_err=float(err.mean()), small_batches_mean_abs_err=float(err_small.mean()),
                            heldout_mean_abs_err=float(verr.mean()))
        lines += [f"## {'Visible-pair (causal) FLOP count' if causal else 'FLOP count of Table 2 as printed (no causality)'}\n",
                  f"- F_ap = {params['F_ap'] / 1e12:.1f} TFLOP/s, F_ad = {params['F_ad'] / 1e12:.1f} TFLOP/s (decode operators are "
                  f"memory-bound: F_ad is not identified by the data), M_a = {params['M_a'] / 1e9:.0f} GB/s, "
                  f"O_p = {params['O_p'] * 1e6:.1f} us, O_d = {params['O_d'] * 1e6:.1f} us",
                  f"- fitted points: mean absolute error {err.mean() * 100:.1f} %, median {np.median(err) * 100:.1f} %, worst "
                  f"{err.max() * 100:.1f} % (the paper reports about 5 % for whole model iterations)",
                  f"- small batches outside the fit: mean {err_small.mean() * 100:.1f} %, worst {err_small.max() * 100:.1f} %",
                  f"- held-out mixed batches: mean {verr.mean() * 100:.1f} % (the model adds prefill and decode times; with the two "
                  "kernels overlapped on two streams a call is faster than the sum)\n",
                  "| kind | batch | in fit | measured us | predicted us | error % |", "|---|---|---|---|---|---|"]
        for r, e in zip(rows, resid(theta, rows)):
            lines.append(f"| {r['kind']} | {r['desc']} | {'yes' if r['full'] else 'no'} | {r['t'] * 1e6:.1f} | "
                         f"{pred(theta, r) * 1e6:.1f} | {e * 100:+.1f} |")
        for r in val:
            p = pred(theta, r)
            lines.append(f"| mixed (held out) | {r['desc']} | no | {r['t'] * 1e6:.1f} | {p * 1e6:.1f} | {(p / r['t'] - 1) * 100:+.1f} |")
        lines.append("")
    text = "\n".join(lines) + "\n"
    print(text)
    if a.out_md:
        open(a.out_md, "w").write(text)
    if a.out_json:
        json.dump(dict(geometry=dict(Hq=Hq, Hkv=Hkv, hd=hd), **results), open(a.out_json, "w"), indent=1)
    ctx.close()


if __name__ == "__main__":
    main()

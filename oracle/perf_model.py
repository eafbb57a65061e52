"""Definition-level oracle of the paper's roofline latency model, restricted to the attention operator.

TEST INFRASTRUCTURE ONLY -- the product path never imports this file.

What is computed (Section 3.3: operator model of Table 2 with the symbols of Table 1, environment
parameters of Table 3, operator latency of Equation 1, and the rule that an iteration's latency is the
sum of its operators' latencies plus a static overhead):

    attention operator of one request with S_q query rows over S_kv keys, D_h = H_q * head_dim:
        FLOPs  = 4 * D_h * S_q * S_kv
        bytes  = 2 * d * (S_q * D_h + S_kv * D_h * H_kv / H_q)
        time   = max(FLOPs / F_a, bytes / M_a),   F_a = F_ap for a prefill operator (S_q > 1),
                                                   F_a = F_ad for a decode operator (S_q == 1)
    iteration = sum over the requests of the batch + O_p if the batch holds prefill work
                                                   + O_d if it holds decode work

Readings (the paper is silent or garbled here; the build's design notes list them too):
  * the memory term's head ratio is H_kv / H_q (printed inverted: grouped-query attention must shrink
    the KV bytes, Section 2.3);
  * Table 2's FLOPs ignore causality; the model keeps the table's count by default; with causal=True the
    count is restricted to the visible (row, key) pairs, 4 * D_h * (S_q * ctx + S_q (S_q + 1) / 2), the
    work a causal kernel does (for a decode operator both counts coincide);
  * the paper's iterations are either prefill or decode; a mixed call is modelled as both kinds of
    work in one iteration: operator times add, and each kind present contributes its overhead once;
  * only the attention operator is modelled here (GEMM and communication operators are outside the
    path this repository builds).
Plain float64, one request at a time.  Pins: tests/test_oracle_pins.py (hand-evaluated Table 2 values,
the two regimes of Equation 1 and their crossing point, additivity, overhead rule).
"""
from __future__ import annotations

from typing import Dict, Sequence


def attention_flops(Hq: int, hd: int, S_q: int, S_kv: int) -> float:
    return 4.0 * (Hq * hd) * S_q * S_kv


def attention_bytes(Hq: int, Hkv: int, hd: int, S_q: int, S_kv: int, d: int = 2) -> float:
    D_h = Hq * hd
    return 2.0 * d * (S_q * D_h + S_kv * D_h * Hkv / Hq)


def op_latency(flops: float, nbytes: float, F: float, M: float) -> float:
    return max(flops / F, nbytes / M)


def attention_flops_causal(Hq: int, hd: int, S_q: int, ctx: int) -> float:
    pairs = 0
    for t in range(S_q):          # row t sees the ctx cached keys and rows 0..t of the chunk
        pairs += ctx + t + 1
    return 4.0 * (Hq * hd) * pairs


def predict(params: Dict[str, float], Hq: int, Hkv: int, hd: int, q_lens: Sequence[int], ctx_lens: Sequence[int],
            d: int = 2, causal: bool = False) -> Dict[str, float]:
    """params: F_ap, F_ad [FLOP/s], M_a [B/s], O_p, O_d [s].  Returns the iteration latency and its parts."""
    t_prefill = t_decode = flops = nbytes = t_compute = t_memory = 0.0
    any_p = any_d = False
    for ql, ctx in zip(q_lens, ctx_lens):
        ql, ctx = int(ql), int(ctx)
        if ql <= 0:
            continue
        f = attention_flops_causal(Hq, hd, ql, ctx) if causal else attention_flops(Hq, hd, ql, ctx + ql)
        b = attention_bytes(Hq, Hkv, hd, ql, ctx + ql, d)
        F = params["F_ap"] if ql > 1 else params["F_ad"]
        t = op_latency(f, b, F, params["M_a"])
        if f / F >= b / params["M_a"]:
            t_compute += t
        else:
            t_memory += t
        if ql > 1:
            t_prefill += t
            any_p = True
        else:
            t_decode += t
            any_d = True
        flops += f
        nbytes += b
    overhead = (params["O_p"] if any_p else 0.0) + (params["O_d"] if any_d else 0.0)
    return dict(latency=t_prefill + t_decode + overhead, prefill=t_prefill, decode=t_decode, overhead=overhead,
                flops=flops, bytes=nbytes, compute_bound=t_compute, memory_bound=t_memory)

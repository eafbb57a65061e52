"""Oracle of the paper's Mix Decoding Selection (Algorithm 2, Section 3.4.4).

TEST INFRASTRUCTURE ONLY -- the product path never imports this file.

Before every decode step the node picks the requests of the step: every online request, then as many
candidate offline requests as the TPOT bound S allows according to the latency predictor L (here the
attention latency model of oracle/perf_model.py applied to a decode-only batch, one operator per request
with S_q = 1 and S_kv = the request's length).  Steps, in the paper's order:
  1. B starts as the set of online requests.
  2. Up to K offline requests are looked at in random order; a request joins B if L(B + request) <= S,
     otherwise it is dropped for this step.
  3. If offline requests remain that were not looked at and L(B) < S, they are sorted by ascending length and
     the longest prefix of that order with L(B + prefix) <= S joins B (found by bisection; L grows with every
     request added, so the admissible prefixes are nested).
Readings (the listing leaves them open): the random order is an INPUT (a sequence of offline indices drawn by the
caller, so that both implementations see the same draws); an index that repeats or lies outside the candidates
counts as one of the K looks and changes nothing; ties in the sort are broken by index; if the online
requests alone exceed S they are all kept (best-effort mode) and no offline request can join.
Pins: tests/test_oracle_pins.py (a hand-worked example, closed forms for equal lengths, invariants checked by
exhaustive scan on small random cases)."""
from __future__ import annotations

from typing import Dict, List, Sequence

from . import perf_model


def latency(params: Dict[str, float], Hq: int, Hkv: int, hd: int, lens: Sequence[int]) -> float:
    """L(B) for a decode-only batch: requests of the given lengths (KV tokens including the new one)."""
    return perf_model.predict(params, Hq, Hkv, hd, [1] * len(lens), [int(n) - 1 for n in lens])["latency"]


def mix_decoding_select(params, Hq, Hkv, hd, S: float, online_lens: Sequence[int], offline_lens: Sequence[int],
                        random_order: Sequence[int]) -> Dict[str, object]:
    """Returns dict(selected=[bool per offline request], latency=L(B), looked=[bool per offline request])."""
    n = len(offline_lens)
    batch: List[int] = [int(x) for x in online_lens]
    selected = [False] * n
    looked = [False] * n
    for r in random_order:                       # K looks
        r = int(r)
        if r < 0 or r >= n or looked[r]:
            continue
        looked[r] = True
        if latency(params, Hq, Hkv, hd, batch + [int(offline_lens[r])]) <= S:
            batch.append(int(offline_lens[r]))
            selected[r] = True
    rest = sorted((i for i in range(n) if not looked[i]), key=lambda i: (int(offline_lens[i]), i))
    if rest and latency(params, Hq, Hkv, hd, batch) < S:
        lo, hi = 0, len(rest)                    # largest m with L(B + rest[:m]) <= S
        while lo < hi:
            mid = (lo + hi + 1) // 2
            if latency(params, Hq, Hkv, hd, batch + [int(offline_lens[i]) for i in rest[:mid]]) <= S:
                lo = mid
            else:
                hi = mid - 1
        for i in rest[:lo]:
            batch.append(int(offline_lens[i]))
            selected[i] = True
    return dict(selected=selected, latency=latency(params, Hq, Hkv, hd, batch), looked=looked)

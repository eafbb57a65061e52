"""Oracle of the paper's Offline Request Migration Decision (Algorithm 1, Section 3.4.3) and of the rule
for choosing which offline requests to evict from a latency-strict node (Section 3.4.1).

TEST INFRASTRUCTURE ONLY -- the product path never imports this file.

Migration decision.  A latency-strict node whose last decode step took every request it holds (B) and is
predicted to stay under the TPOT bound, L(B) < S, asks a latency-relaxed node for more offline requests and
names the request length it prefers, Pref.  bs(B) is the number of requests in B, bs_sat the batch size from
which the step is compute-saturated, U_mem the share of the KV cache in use.  In the paper's order:
  * L(B) >= S, or some request of the node was left out of B: no migration (Pref = none);
  * bs(B) >= bs_sat (a larger batch buys no efficiency, so fill the memory): Pref = the largest length l such
    that one more request of length l keeps L <= S and U_mem <= 1;
  * otherwise the aim is to reach bs_sat.  With n = bs_sat - bs(B) missing requests: if n requests of the
    shortest length keep L <= S, Pref = the largest l such that n requests of length l keep L <= S;
    else Pref = the shortest length (as many requests as possible).
Readings (the listing leaves them open):
  * L is the attention latency model of oracle/perf_model.py on a decode-only batch (oracle/mix_select.latency);
  * lengths range over [len_min, len_max], given by the caller (what the latency-relaxed node can offer);
  * in the saturated branch r is ONE request; in the unsaturated branch r is the GROUP that would reach bs_sat
    (the text speaks of adding a group of requests), taken as n requests of one common length, and the same
    group appears in the existence test (at the shortest length, the cheapest such group) and in the maximum;
  * the memory condition is written only in the saturated branch and is applied only there;
  * a maximum over an empty set (not even len_min fits) gives no migration;
  * U_mem counts KV blocks: sum of ceil(length / block_size) over capacity_blocks.
Selection on the latency-relaxed node ("most close to Pref"): its ongoing offline requests are visited by
ascending |length - Pref| (ties: shorter first, then lower index); a request is migrated if the strict node's
batch with it still has L <= S and U_mem <= 1, otherwise it is passed over; at most max_migrate requests go.

Eviction victims (Section 3.4.1).  An online request that finished its prefill needs need_blocks free KV
blocks on the strict node.  If the node is compute-bound (bs(B) >= bs_sat, as in Algorithm 1) long requests
go first, which keeps the decode batch large; otherwise short ones go first, which keeps the recomputation
small.  Requests are taken in that order (ties by index) until their blocks cover the need; then, in the order
taken, a victim whose blocks are not needed any more (the others still cover the need) is kept after all.
Readings: the paper gives only the direction of the preference; greedy order, the final pass and the
block-granular accounting are this build's.  If all requests together do not cover the need, all are returned
and `enough` is False.
Pins: tests/test_oracle_pins.py (closed forms in the memory-bound regime, hand-worked cases, exhaustive
subset search on small inputs)."""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

from . import mix_select


def blocks(length: int, block_size: int) -> int:
    return (int(length) + block_size - 1) // block_size


def u_mem(lens: Sequence[int], block_size: int, capacity_blocks: int) -> float:
    return sum(blocks(n, block_size) for n in lens) / capacity_blocks


def migration_preference(params, Hq, Hkv, hd, S: float, batch_lens: Sequence[int], all_included: bool, bs_sat: int,
                         block_size: int, capacity_blocks: int, len_min: int, len_max: int) -> Dict[str, object]:
    """Returns dict(pref=length or None, branch='none'|'saturated'|'reach'|'shortest')."""
    B = [int(n) for n in batch_lens]
    L = lambda lens: mix_select.latency(params, Hq, Hkv, hd, lens)
    if not (L(B) < S and all_included):
        return dict(pref=None, branch="none")
    if len(B) >= bs_sat:
        fits = [l for l in range(len_min, len_max + 1)
                if L(B + [l]) <= S and u_mem(B + [l], block_size, capacity_blocks) <= 1.0]
        return dict(pref=max(fits) if fits else None, branch="saturated" if fits else "none")
    n = bs_sat - len(B)
    if L(B + [len_min] * n) <= S:
        fits = [l for l in range(len_min, len_max + 1) if L(B + [l] * n) <= S]
        return dict(pref=max(fits), branch="reach")
    return dict(pref=len_min, branch="shortest")


def migration_select(params, Hq, Hkv, hd, S: float, batch_lens: Sequence[int], relaxed_lens: Sequence[int], pref: int,
                     block_size: int, capacity_blocks: int, max_migrate: int) -> List[int]:
    """Indices into relaxed_lens of the requests to migrate, in the order they are taken."""
    B = [int(n) for n in batch_lens]
    order = sorted(range(len(relaxed_lens)), key=lambda i: (abs(int(relaxed_lens[i]) - pref), int(relaxed_lens[i]), i))
    chosen: List[int] = []
    for i in order:
        if len(chosen) >= max_migrate:
            break
        cand = B + [int(relaxed_lens[i])]
        if mix_select.latency(params, Hq, Hkv, hd, cand) <= S and u_mem(cand, block_size, capacity_blocks) <= 1.0:
            B = cand
            chosen.append(i)
    return chosen


def eviction_victims(offline_lens: Sequence[int], need_blocks: int, block_size: int, batch_size: int,
                     bs_sat: int) -> Dict[str, object]:
    """Returns dict(victims=[indices in the order taken], enough=bool, compute_bound=bool)."""
    compute_bound = batch_size >= bs_sat
    key = (lambda i: (-int(offline_lens[i]), i)) if compute_bound else (lambda i: (int(offline_lens[i]), i))
    order = sorted(range(len(offline_lens)), key=key)
    taken: List[int] = []
    freed = 0
    for i in order:
        if freed >= need_blocks:
            break
        taken.append(i)
        freed += blocks(offline_lens[i], block_size)
    enough = freed >= need_blocks
    if enough:
        for i in list(taken):
            b = blocks(offline_lens[i], block_size)
            if freed - b >= need_blocks:
                taken.remove(i)
                freed -= b
    return dict(victims=taken, enough=enough, compute_bound=compute_bound)

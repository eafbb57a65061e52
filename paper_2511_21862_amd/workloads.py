"""Seeded synthetic input generators for the mixed-batch paged-attention path.

This module only *produces and moves data*: request lengths, block tables, random
bf16 values, and the packing of values into the paged cache layout.  It holds none
of the attention arithmetic, so that both the HIP path and the CPU oracle can be fed
from it without sharing any of the method's code.

Workload shapes follow the paper's description of a latency-relaxed instance
(Section 3.2.1: online/offline prefill plus offline decode on one instance), its
decode batch sizes "into the hundreds" (Section 2.3) and the request-length statistics of
Table 4 (prompt means 1.2K-2.3K tokens, outputs up to ~1K tokens).  The traces
themselves are not available; the length distributions below stand in for them.

Paged cache layout (bf16, one attention layer), fixed by include/ooco.h:

    k_cache[num_blocks][Hkv][hd/8][BS][8]   element (b, kvh, d, s) at
                                            (((b*Hkv + kvh)*(hd/8) + d//8)*BS + s)*8 + d%8
    v_cache[num_blocks][Hkv][hd][BS]        element (b, kvh, d, s) at
                                            ((b*Hkv + kvh)*hd + d)*BS + s

Token j of sequence i lives in physical block block_tables[i][j // BS], slot j % BS.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, Optional, Sequence, Tuple

import numpy as np

BF16_NAN = np.uint16(0x7FC0)
BF16_INF = np.uint16(0x7F80)


# ----------------------------------------------------------------------------- bf16 bits
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit pattern (uint16), round to nearest even. NaN stays NaN."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    out = rounded.astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out = np.where(nan, BF16_NAN, out)
    return out


def bf16_bits_to_f32(u: np.ndarray) -> np.ndarray:
    """bf16 bit pattern (uint16) -> float32 (exact)."""
    return (np.ascontiguousarray(u, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ----------------------------------------------------------------------------- batch
@dataclass
class Batch:
    """One attention call's inputs.

    Metadata is always numpy on the host.  `q`, `k_cache`, `v_cache` are either numpy
    uint16 arrays (bf16 bit patterns, host) or torch bfloat16 tensors (device).
    """

    Hq: int
    Hkv: int
    hd: int
    BS: int
    num_blocks: int
    block_tables: np.ndarray      # int32 [num_seqs, max_blocks_per_seq]
    seq_lens: np.ndarray          # int32 [num_seqs]   = ctx_lens + q_lens
    ctx_lens: np.ndarray          # int32 [num_seqs]   tokens cached before this step
    query_start_loc: np.ndarray   # int32 [num_seqs+1]
    q: object                     # [T, Hq, hd]
    k_cache: object               # [num_blocks, Hkv, hd/8, BS, 8]
    v_cache: object               # [num_blocks, Hkv, hd, BS]
    name: str = ""
    extra: dict = field(default_factory=dict)

    @property
    def num_seqs(self) -> int:
        return int(self.seq_lens.shape[0])

    @property
    def q_lens(self) -> np.ndarray:
        return np.diff(self.query_start_loc).astype(np.int32)

    @property
    def total_q(self) -> int:
        return int(self.query_start_loc[-1])

    @property
    def max_blocks_per_seq(self) -> int:
        return int(self.block_tables.shape[1])

    @property
    def on_host(self) -> bool:
        return isinstance(self.k_cache, np.ndarray)

    def k_shape(self):
        return (self.num_blocks, self.Hkv, self.hd // 8, self.BS, 8)

    def v_shape(self):
        return (self.num_blocks, self.Hkv, self.hd, self.BS)


def _blocks_needed(seq_lens: np.ndarray, BS: int) -> np.ndarray:
    return (np.asarray(seq_lens, dtype=np.int64) + BS - 1) // BS


def _torch_to_bits(t) -> np.ndarray:
    import torch

    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def _bits_to_torch(a: np.ndarray, device):
    import torch

    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16).to(device)


def build_batch(
    *,
    Hq: int,
    Hkv: int,
    hd: int,
    q_lens: Sequence[int],
    ctx_lens: Sequence[int],
    num_blocks: int,
    seed: int,
    BS: int = 16,
    value_std: float = 1.0,
    poison: bool = False,
    max_blocks_per_seq: Optional[int] = None,
    device: str = "cpu",
    rng: Optional[np.random.Generator] = None,
    name: str = "",
) -> Batch:
    """Deal blocks from a shuffled free list, then fill Q and both pools with N(0, std) bf16.

    Order of random draws: (lengths are drawn by the caller, from the same `rng` when
    given) -> free-list shuffle -> values.  With `poison`, every cache slot that no
    sequence owns (tails of last blocks, unreferenced blocks) is NaN/Inf and unused
    block-table columns are -1; otherwise unused columns are -1 and unowned slots keep
    their random values.
    """
    assert hd % 8 == 0 and Hq % Hkv == 0
    rng = np.random.default_rng(seed) if rng is None else rng
    q_lens = np.asarray(q_lens, dtype=np.int32)
    ctx_lens = np.asarray(ctx_lens, dtype=np.int32)
    seq_lens = (ctx_lens + q_lens).astype(np.int32)
    S = len(seq_lens)
    nb = _blocks_needed(seq_lens, BS)
    if int(nb.sum()) > num_blocks:
        raise ValueError(f"pool of {num_blocks} blocks too small: need {int(nb.sum())}")
    maxb = int(max(int(nb.max()) if S else 0, 1))
    if max_blocks_per_seq is not None:
        if max_blocks_per_seq < maxb:
            raise ValueError("max_blocks_per_seq too small")
        maxb = int(max_blocks_per_seq)

    free = rng.permutation(num_blocks).astype(np.int32)
    block_tables = np.full((S, maxb), -1, dtype=np.int32)
    pos = 0
    for i in range(S):
        n = int(nb[i])
        block_tables[i, :n] = free[pos:pos + n]
        pos += n
    qsl = np.zeros(S + 1, dtype=np.int32)
    qsl[1:] = np.cumsum(q_lens)
    T = int(qsl[-1])

    kshape = (num_blocks, Hkv, hd // 8, BS, 8)
    vshape = (num_blocks, Hkv, hd, BS)
    if device == "cpu":
        q = f32_to_bf16_bits(rng.standard_normal((T, Hq, hd), dtype=np.float32) * np.float32(value_std))
        k = f32_to_bf16_bits(rng.standard_normal(kshape, dtype=np.float32) * np.float32(value_std))
        v = f32_to_bf16_bits(rng.standard_normal(vshape, dtype=np.float32) * np.float32(value_std))
        if poison:
            owned = np.zeros((num_blocks, BS), dtype=bool)
            for i in range(S):
                L = int(seq_lens[i])
                for j in range(int(nb[i])):
                    owned[block_tables[i, j], : min(BS, L - j * BS)] = True
            bad = ~owned
            # alternate NaN / +Inf so that both kinds of poison are exercised
            kb = np.where((np.arange(num_blocks)[:, None] + np.arange(BS)[None, :]) % 2 == 0, BF16_NAN, BF16_INF)
            k[:] = np.where(bad[:, None, None, :, None], kb[:, None, None, :, None], k)
            v[:] = np.where(bad[:, None, None, :], kb[:, None, None, :], v)
    else:
        import torch

        g = torch.Generator(device=device)
        g.manual_seed(int(seed))
        q = torch.empty((T, Hq, hd), dtype=torch.bfloat16, device=device).normal_(0.0, value_std, generator=g)
        k = torch.empty(kshape, dtype=torch.bfloat16, device=device).normal_(0.0, value_std, generator=g)
        v = torch.empty(vshape, dtype=torch.bfloat16, device=device).normal_(0.0, value_std, generator=g)
        if poison:
            raise ValueError("poisoned pools are generated on the host only")

    return Batch(Hq=Hq, Hkv=Hkv, hd=hd, BS=BS, num_blocks=num_blocks, block_tables=block_tables,
                 seq_lens=seq_lens, ctx_lens=ctx_lens.astype(np.int32), query_start_loc=qsl,
                 q=q, k_cache=k, v_cache=v, name=name, extra={"free_list": free, "free_pos": pos})


def replica_tables(b: Batch, max_replicas: int) -> list:
    """Block tables for further copies of the same batch (same lengths) dealt from the blocks the
    shuffled free list still holds, so that successive timed steps touch disjoint physical
    blocks of the pool (every block of a generated pool holds random values)."""
    free, pos = b.extra["free_list"], int(b.extra["free_pos"])
    nb = _blocks_needed(b.seq_lens, b.BS)
    need = int(nb.sum())
    tables = [b.block_tables]
    while len(tables) < max_replicas and pos + need <= len(free):
        bt = np.full_like(b.block_tables, -1)
        for i in range(b.num_seqs):
            n = int(nb[i])
            bt[i, :n] = free[pos:pos + n]
            pos += n
        tables.append(bt)
    return tables


# ----------------------------------------------------------------------------- data movement helpers
def to_device(b: Batch, device: str = "cuda") -> Batch:
    if not b.on_host:
        return b
    return replace(b, q=_bits_to_torch(b.q, device), k_cache=_bits_to_torch(b.k_cache, device),
                   v_cache=_bits_to_torch(b.v_cache, device))


def to_host(b: Batch) -> Batch:
    if b.on_host:
        return b
    return replace(b, q=_torch_to_bits(b.q), k_cache=_torch_to_bits(b.k_cache), v_cache=_torch_to_bits(b.v_cache))


def subset(b: Batch, seq_ids: Sequence[int]) -> Batch:
    """Host batch holding only the chosen sequences, with their blocks renumbered
    0..n-1 in a compact pool (pure data movement; used to hand the oracle a bounded
    sample of a large device-resident batch)."""
    seq_ids = [int(s) for s in seq_ids]
    nb = _blocks_needed(b.seq_lens, b.BS)
    ids = np.concatenate([b.block_tables[s, : int(nb[s])] for s in seq_ids]) if seq_ids else np.zeros(0, np.int32)
    maxb = int(max([int(nb[s]) for s in seq_ids] + [1]))
    bt = np.full((len(seq_ids), maxb), -1, dtype=np.int32)
    pos = 0
    for r, s in enumerate(seq_ids):
        n = int(nb[s])
        bt[r, :n] = np.arange(pos, pos + n, dtype=np.int32)
        pos += n
    ql = b.q_lens[seq_ids] if seq_ids else np.zeros(0, np.int32)
    qsl = np.zeros(len(seq_ids) + 1, dtype=np.int32)
    qsl[1:] = np.cumsum(ql)
    rows = np.concatenate([np.arange(b.query_start_loc[s], b.query_start_loc[s + 1]) for s in seq_ids]) \
        if seq_ids else np.zeros(0, np.int64)
    if b.on_host:
        k = b.k_cache[ids]
        v = b.v_cache[ids]
        q = b.q[rows]
    else:
        import torch

        idx = torch.from_numpy(ids.astype(np.int64)).to(b.k_cache.device)
        ridx = torch.from_numpy(rows.astype(np.int64)).to(b.q.device)
        k = _torch_to_bits(b.k_cache.index_select(0, idx))
        v = _torch_to_bits(b.v_cache.index_select(0, idx))
        q = _torch_to_bits(b.q.index_select(0, ridx))
    return Batch(Hq=b.Hq, Hkv=b.Hkv, hd=b.hd, BS=b.BS, num_blocks=max(int(len(ids)), 1), block_tables=bt,
                 seq_lens=b.seq_lens[seq_ids].copy(), ctx_lens=b.ctx_lens[seq_ids].copy(), query_start_loc=qsl,
                 q=np.ascontiguousarray(q), k_cache=np.ascontiguousarray(k).reshape((-1,) + b.k_shape()[1:]),
                 v_cache=np.ascontiguousarray(v).reshape((-1,) + b.v_shape()[1:]),
                 name=b.name + f"[subset {len(seq_ids)}]", extra={"rows": rows})


def row_sample(b: Batch, pairs: Sequence[Tuple[int, int]]) -> Batch:
    """Host batch with one single-token sequence per sampled query row: (s, t) = row t of sequence s
    of `b` becomes a sequence of ctx_len = ctx_len[s] + t that shares the KV blocks of s (copied once per
    source sequence into a compact pool).  Pure data movement: lets the oracle check sampled rows of a
    large device-resident batch one by one (a chunk row is a single-query decode over its visible keys)."""
    pairs = [(int(s), int(t)) for s, t in pairs]
    need: Dict[int, int] = {}
    for s_, t in pairs:
        assert 0 <= t < int(b.q_lens[s_])
        need[s_] = max(need.get(s_, 0), (int(b.ctx_lens[s_]) + t + 1 + b.BS - 1) // b.BS)
    base, ids, pos = {}, [], 0
    for s_ in sorted(need):
        base[s_] = pos
        ids.append(b.block_tables[s_, : need[s_]])
        pos += need[s_]
    ids = np.concatenate(ids).astype(np.int64) if ids else np.zeros(0, np.int64)
    maxb = max(list(need.values()) + [1])
    bt = np.full((len(pairs), maxb), -1, dtype=np.int32)
    ctx = np.zeros(len(pairs), dtype=np.int32)
    rows = np.zeros(len(pairs), dtype=np.int64)
    for r, (s_, t) in enumerate(pairs):
        ctx[r] = int(b.ctx_lens[s_]) + t
        n = (int(ctx[r]) + 1 + b.BS - 1) // b.BS
        bt[r, :n] = base[s_] + np.arange(n, dtype=np.int32)
        rows[r] = int(b.query_start_loc[s_]) + t
    if b.on_host:
        k, v, q = b.k_cache[ids], b.v_cache[ids], b.q[rows]
    else:
        import torch

        idx = torch.from_numpy(ids).to(b.k_cache.device)
        ridx = torch.from_numpy(rows).to(b.q.device)
        k = _torch_to_bits(b.k_cache.index_select(0, idx))
        v = _torch_to_bits(b.v_cache.index_select(0, idx))
        q = _torch_to_bits(b.q.index_select(0, ridx))
    return Batch(Hq=b.Hq, Hkv=b.Hkv, hd=b.hd, BS=b.BS, num_blocks=max(int(len(ids)), 1), block_tables=bt,
                 seq_lens=ctx + 1, ctx_lens=ctx, query_start_loc=np.arange(len(pairs) + 1, dtype=np.int32),
                 q=np.ascontiguousarray(q), k_cache=np.ascontiguousarray(k).reshape((-1,) + b.k_shape()[1:]),
                 v_cache=np.ascontiguousarray(v).reshape((-1,) + b.v_shape()[1:]),
                 name=b.name + f"[{len(pairs)} sampled rows]", extra={"rows": rows})


def scatter_logical(b: Batch, seq: int, k_bits: np.ndarray, v_bits: np.ndarray) -> None:
    """Write logical K/V (uint16 bf16 bits, [L, Hkv, hd]) of one sequence into a host batch's pools."""
    assert b.on_host
    L = int(b.seq_lens[seq])
    assert k_bits.shape == (L, b.Hkv, b.hd) and v_bits.shape == (L, b.Hkv, b.hd)
    for j in range(L):
        blk, s = int(b.block_tables[seq, j // b.BS]), j % b.BS
        b.k_cache[blk, :, :, s, :] = k_bits[j].reshape(b.Hkv, b.hd // 8, 8)
        b.v_cache[blk, :, :, s] = v_bits[j]


def gather_logical(b: Batch, seq: int):
    """Inverse of scatter_logical: ([L,Hkv,hd], [L,Hkv,hd]) uint16 of one sequence of a host batch."""
    assert b.on_host
    L = int(b.seq_lens[seq])
    k = np.empty((L, b.Hkv, b.hd), dtype=np.uint16)
    v = np.empty((L, b.Hkv, b.hd), dtype=np.uint16)
    for j in range(L):
        blk, s = int(b.block_tables[seq, j // b.BS]), j % b.BS
        k[j] = b.k_cache[blk, :, :, s, :].reshape(b.Hkv, b.hd)
        v[j] = b.v_cache[blk, :, :, s]
    return k, v


def permute_blocks(b: Batch, seed: int) -> Batch:
    """Same logical batch with every physical block moved to a new random id (host batches)."""
    assert b.on_host
    perm = np.random.default_rng(seed).permutation(b.num_blocks).astype(np.int32)  # old id -> new id
    k = np.empty_like(b.k_cache)
    v = np.empty_like(b.v_cache)
    k[perm] = b.k_cache
    v[perm] = b.v_cache
    bt = np.where(b.block_tables >= 0, perm[np.clip(b.block_tables, 0, b.num_blocks - 1)], -1).astype(np.int32)
    return replace(b, k_cache=k, v_cache=v, block_tables=bt)


# ----------------------------------------------------------------------------- length recipes
def lognormal_lengths(rng, n, median, sigma, lo, hi) -> np.ndarray:
    z = rng.standard_normal(n)
    return np.clip(np.rint(np.exp(np.log(median) + sigma * z)), lo, hi).astype(np.int32)


def uniform_lengths(rng, n, lo, hi) -> np.ndarray:
    return rng.integers(lo, hi + 1, size=n).astype(np.int32)


# ----------------------------------------------------------------------------- the five configurations
def config1(device: str = "cpu", poison: bool = False) -> Batch:
    """Tiny mixed batch: 4 decode sequences (37, 64, 100, 129 tokens, the query included)
    and one 32-token prefill chunk without prior context; 4 query heads on 1 KV head, hd 64."""
    seq = np.array([37, 64, 100, 129, 32], dtype=np.int32)
    ql = np.array([1, 1, 1, 1, 32], dtype=np.int32)
    return build_batch(Hq=4, Hkv=1, hd=64, q_lens=ql, ctx_lens=seq - ql, num_blocks=32, seed=0,
                       poison=poison, max_blocks_per_seq=11, device=device, name="cfg1-tiny-mixed")


def config2(device: str = "cuda", value_std: float = 1.0 / np.sqrt(128.0), num_seqs: int = 64,
            num_blocks: int = 32768, seed: int = 2) -> Batch:
    """Decode only, Llama-3-8B-shaped layer: 64 sequences, lengths uniform in [512, 4096]."""
    rng = np.random.default_rng(seed)
    seq = uniform_lengths(rng, num_seqs, 512, 4096)
    ql = np.ones(num_seqs, dtype=np.int32)
    return build_batch(Hq=32, Hkv=8, hd=128, q_lens=ql, ctx_lens=seq - ql, num_blocks=num_blocks, seed=seed,
                       value_std=value_std, device=device, rng=rng, name="cfg2-decode64")


def config3(device: str = "cuda", n_prefill: int = 8, n_decode: int = 128, chunk: int = 512, seed: int = 3,
            Hq: int = 32, Hkv: int = 8, decode_only: bool = False) -> Batch:
    """Co-located mixed batch: prefill chunks on prior context U[0,2048] first, then
    decode sequences with lognormal lengths (median 2048, sigma 0.8, clipped to [128, 8192]).
    `decode_only`: the same decode sequences without the chunks (the lengths are drawn as for the mixed batch)."""
    rng = np.random.default_rng(seed)
    pctx = uniform_lengths(rng, n_prefill, 0, 2048)
    dseq = lognormal_lengths(rng, n_decode, 2048, 0.8, 128, 8192)
    if decode_only:
        n_prefill, pctx = 0, pctx[:0]
    ql = np.concatenate([np.full(n_prefill, chunk, np.int32), np.ones(n_decode, np.int32)])
    ctx = np.concatenate([pctx, dseq - 1]).astype(np.int32)
    need = int(_blocks_needed(ctx + ql, 16).sum())
    nblk = max(32768, int(1.25 * need))
    return build_batch(Hq=Hq, Hkv=Hkv, hd=128, q_lens=ql, ctx_lens=ctx, num_blocks=nblk, seed=seed,
                       device=device, rng=rng, name="cfg3-decode-part" if decode_only else "cfg3-mixed")


def config4(device: str = "cuda", n_decode: int = 512, n_victims: int = 64, seed: int = 4,
            num_blocks: int = 131072) -> Batch:
    """Large offline decode batch, lognormal lengths (median 2048, sigma 1.0, clipped to
    [64, 32768]); `extra['victims']` names the sequences one preemption evicts."""
    rng = np.random.default_rng(seed)
    seq = lognormal_lengths(rng, n_decode, 2048, 1.0, 64, 32768)
    victims = np.sort(rng.choice(n_decode, size=min(n_victims, n_decode), replace=False)).astype(np.int32)
    ql = np.ones(n_decode, np.int32)
    b = build_batch(Hq=32, Hkv=8, hd=128, q_lens=ql, ctx_lens=seq - ql, num_blocks=num_blocks, seed=seed,
                    device=device, rng=rng, name="cfg4-decode512")
    b.extra["victims"] = victims
    return b


def config5(device: str = "cuda", n_decode: int = 32, n_prefill: int = 2, chunk: int = 2048, pctx: int = 4096,
            seed: int = 5, num_blocks: int = 196608, lo: int = 32768, hi: int = 131072) -> Batch:
    """Long-context mixed batch, Qwen2-72B-shaped layer (64 query heads on 8 KV heads)."""
    rng = np.random.default_rng(seed)
    dseq = uniform_lengths(rng, n_decode, lo, hi)
    ql = np.concatenate([np.full(n_prefill, chunk, np.int32), np.ones(n_decode, np.int32)])
    ctx = np.concatenate([np.full(n_prefill, pctx, np.int32), dseq - 1]).astype(np.int32)
    return build_batch(Hq=64, Hkv=8, hd=128, q_lens=ql, ctx_lens=ctx, num_blocks=num_blocks, seed=seed,
                       device=device, rng=rng, name="cfg5-longctx-mixed")


def victim_block_ids(b: Batch, victims: Sequence[int]) -> np.ndarray:
    """Physical block ids owned by the victim sequences, in block-table order (int64)."""
    nb = _blocks_needed(b.seq_lens, b.BS)
    parts = [b.block_tables[int(s), : int(nb[int(s)])] for s in victims]
    return np.concatenate(parts).astype(np.int64) if parts else np.zeros(0, np.int64)

"""Algorithmic work of one attention call: the bytes that must cross HBM and the FLOPs
that must be done, independent of any kernel's tiling.

The paper's operator model (Table 2) counts, for one attention operator,
    FLOPs  = 4 * D_h * S_q * S_kv
    bytes  = 2 * d * (S_q * D_h + S_kv * D_h * H_kv / H_q)
with D_h = Hq*hd the attention hidden size (Table 1) and d bytes per value.  The printed
memory term shows the head ratio upside down; it is read here as H_kv/H_q, the only reading
under which GQA shrinks the KV cache (Section 2.3).  Table 2 ignores causality; prefill work
is therefore also given causal-exact (row t of a chunk on prior context ctx sees ctx+t+1 keys).
"""
from __future__ import annotations

import numpy as np


def table2_flops(D_h: int, S_q: int, S_kv: int) -> int:
    return 4 * D_h * S_q * S_kv


def table2_bytes(D_h: int, S_q: int, S_kv: int, Hq: int, Hkv: int, d: int = 2) -> int:
    assert (S_kv * D_h * Hkv) % Hq == 0
    return 2 * d * (S_q * D_h + S_kv * D_h * Hkv // Hq)


def per_token_kv_bytes(Hkv: int, hd: int, d: int = 2) -> int:
    """K and V bytes of one cached token."""
    return 2 * Hkv * hd * d


def batch_work(Hq, Hkv, hd, BS, seq_lens, q_lens, d: int = 2) -> dict:
    """Sums over a batch.  `bytes_*` follow Table 2 (KV read once + Q read + out written) plus
    the 4-byte block-table entries; `flops_causal` counts only unmasked (row, key) pairs."""
    seq = np.asarray(seq_lens, dtype=np.int64)
    ql = np.asarray(q_lens, dtype=np.int64)
    ctx = seq - ql
    dec = ql == 1
    pre = ql > 1
    T = per_token_kv_bytes(Hkv, hd, d)
    D_h = Hq * hd

    def _bytes(mask):
        return int((seq[mask] * T + ((seq[mask] + BS - 1) // BS) * 4 + 2 * ql[mask] * D_h * d).sum())

    pairs = ql * ctx + ql * (ql + 1) // 2          # visible (row, key) pairs per sequence
    return {
        "q_tokens": int(ql.sum()),
        "decode_seqs": int(dec.sum()),
        "prefill_chunks": int(pre.sum()),
        "kv_tokens": int(seq[ql > 0].sum()),
        "decode_kv_tokens": int(seq[dec].sum()),
        "bytes_total": _bytes(ql > 0),
        "bytes_decode": _bytes(dec),
        "bytes_prefill": _bytes(pre),
        "flops_causal": int((4 * D_h * pairs).sum()),
        "flops_causal_prefill": int((4 * D_h * pairs[pre]).sum()),
        "flops_table2": int((4 * D_h * ql * seq).sum()),
        "flops_decode": int((4 * D_h * seq[dec]).sum()),
    }


def block_copy_bytes(num_pairs: int, Hkv: int, hd: int, BS: int, d: int = 2) -> int:
    """Read + write of whole K and V blocks."""
    return 2 * num_pairs * BS * per_token_kv_bytes(Hkv, hd, d)

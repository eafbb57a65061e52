"""Definition-level float64 oracle of causal GQA attention over a paged KV cache.

TEST INFRASTRUCTURE ONLY -- the product path never imports this file.

What is computed (the paper treats attention as one fused softmax(QK^T)V operator whose
score matrix never leaves the chip, Section 3.3.1 and the caption of Figure 2; requests of
different lengths are batched over a non-contiguous KV pool, Section 2.1; decode feeds one
token per request which reads the request's whole KV cache, prefill rows attend causally,
Section 2.3; GQA shares one KV head among Hq/Hkv query heads, Table 1).  The method reaches
this result exactly (up to rounding order), so the oracle is the plain definition:

    for sequence i, query row t (absolute position pos = ctx_len_i + t), query head h,
    kv head kappa = h // (Hq // Hkv):
        K_j, V_j = rows of the cache at block block_tables[i][j // BS], slot j % BS, j = 0..pos
        s_j   = scale * <q[qsl_i + t, h, :], K_j>
        p_j   = exp(s_j - max s) / sum_j exp(s_j - max s)
        out[qsl_i + t, h, :] = sum_j p_j V_j

Inputs are bf16 bit patterns (uint16) widened exactly to float64; all arithmetic is float64;
the output stays float64.  Cache layout (see include/ooco.h):
    k_cache[num_blocks][Hkv][hd/8][BS][8],  v_cache[num_blocks][Hkv][hd][BS].

Pins (tests/test_oracle_pins.py): dense brute force, torch SDPA special cases, closed forms,
softmax-row sums, shift invariance, block-permutation invariance, decode == last prefill row,
chunking invariance, GQA expansion, batch-structure invariance.
"""
from __future__ import annotations

import math

import numpy as np


def widen_bf16(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns -> float64, exactly (bf16 is the top half of an IEEE float32)."""
    u32 = np.asarray(bits, dtype=np.uint16).astype(np.uint32) * np.uint32(65536)
    return u32.view(np.float32).astype(np.float64)


def attn_mixed(q, k_cache, v_cache, block_tables, seq_lens, query_start_loc, ctx_lens,
               scale=None, return_probs=False):
    """float64 [T, Hq, hd] (and, optionally, the list of probability rows)."""
    q = np.asarray(q)
    T, Hq, hd = q.shape
    NB, Hkv, hd8, BS, eight = k_cache.shape
    assert eight == 8 and hd8 * 8 == hd and v_cache.shape == (NB, Hkv, hd, BS)
    assert Hq % Hkv == 0
    g = Hq // Hkv
    if scale is None:
        scale = 1.0 / math.sqrt(hd)
    out = np.zeros((T, Hq, hd), dtype=np.float64)
    probs = []
    num_seqs = len(seq_lens)
    for i in range(num_seqs):
        q0, q1 = int(query_start_loc[i]), int(query_start_loc[i + 1])
        ctx = int(ctx_lens[i])
        assert ctx + (q1 - q0) == int(seq_lens[i]), "seq_len must equal ctx_len + q_len"
        for t in range(q1 - q0):
            pos = ctx + t
            n = pos + 1                     # keys 0..pos, the row's own key included
            for h in range(Hq):
                kap = h // g
                qv = widen_bf16(q[q0 + t, h])
                s = np.empty(n, dtype=np.float64)
                vals = np.empty((n, hd), dtype=np.float64)
                for jb in range((n + BS - 1) // BS):
                    blk = int(block_tables[i][jb])
                    cnt = min(BS, n - jb * BS)
                    # K tile of this block and kv head: [hd/8, cnt, 8] -> [cnt, hd]
                    kt = widen_bf16(k_cache[blk, kap, :, :cnt, :]).transpose(1, 0, 2).reshape(cnt, hd)
                    vt = widen_bf16(v_cache[blk, kap, :, :cnt]).T          # [cnt, hd]
                    s[jb * BS: jb * BS + cnt] = scale * (kt @ qv)
                    vals[jb * BS: jb * BS + cnt] = vt
                e = np.exp(s - s.max())
                p = e / e.sum()
                out[q0 + t, h] = p @ vals
                if return_probs:
                    probs.append(p)
    return (out, probs) if return_probs else out


def block_copy(k_src, v_src, k_dst, v_dst, src_ids, dst_ids):
    """dst_pool[dst_ids[p]] <- src_pool[src_ids[p]] for K and V, whole blocks, in place on the dst arrays."""
    for s, d in zip(src_ids, dst_ids):
        k_dst[int(d)] = k_src[int(s)]
        v_dst[int(d)] = v_src[int(s)]


def kv_append(k_new, v_new, k_cache, v_cache, block_tables, query_start_loc, ctx_lens):
    """Writes the K and V vectors of this step's tokens into their paged slots, in place.

    The paper keeps the K/V of every processed token in the KV cache so that later steps reuse them
    (Section 2.1: the cache is what separates prefill from decode; non-contiguous pool); the token at
    row t of sequence i sits at absolute position pos = ctx_len_i + t, i.e. in physical block
    block_tables[i][pos // BS], slot pos % BS.  k_new, v_new: [T][Hkv][hd] bit patterns (uint16), row
    query_start_loc[i] + t.  Nothing else of the pools changes.  Plain definition, one element at a time.
    Pins: tests/test_oracle_pins.py (hand-evaluated offsets of a tiny example, read-back through an
    independent gather, cache reconstruction, attention after append)."""
    NB, Hkv, hd8, BS, eight = k_cache.shape
    hd = hd8 * 8
    assert eight == 8 and v_cache.shape == (NB, Hkv, hd, BS)
    for i in range(len(ctx_lens)):
        q0, q1 = int(query_start_loc[i]), int(query_start_loc[i + 1])
        for t in range(q1 - q0):
            pos = int(ctx_lens[i]) + t
            blk, slot = int(block_tables[i][pos // BS]), pos % BS
            for kv in range(Hkv):
                for d in range(hd):
                    k_cache[blk, kv, d // 8, slot, d % 8] = k_new[q0 + t, kv, d]
                    v_cache[blk, kv, d, slot] = v_new[q0 + t, kv, d]

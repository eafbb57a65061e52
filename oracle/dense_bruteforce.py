"""Second, independent float64 formulation: dense attention with an explicit mask.

TEST INFRASTRUCTURE ONLY.  Used to pin oracle/ref_numpy.py on tiny inputs.  Differences on
purpose: the cache is addressed through *flat element offsets* computed from the documented
layout formula (not numpy multi-indexing), every sequence is first gathered into contiguous
[L, Hkv, hd] arrays, the whole [q_len, L] score matrix is formed, masked with an explicit
boolean matrix and put through a dense softmax and a dense matmul (Section 3.3.1's
unfused view of the operator).
"""
from __future__ import annotations

import math

import numpy as np


def _f64(bits):
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def gather_sequence(k_flat, v_flat, table_row, L, Hkv, hd, BS):
    K = np.empty((L, Hkv, hd), dtype=np.float64)
    V = np.empty((L, Hkv, hd), dtype=np.float64)
    for j in range(L):
        b = int(table_row[j // BS])
        s = j % BS
        for kh in range(Hkv):
            for d in range(hd):
                K[j, kh, d] = _f64(k_flat[(((b * Hkv + kh) * (hd // 8) + d // 8) * BS + s) * 8 + d % 8])
                V[j, kh, d] = _f64(v_flat[((b * Hkv + kh) * hd + d) * BS + s])
    return K, V


def attn_mixed_dense(q, k_cache, v_cache, block_tables, seq_lens, query_start_loc, ctx_lens, scale=None):
    q = np.asarray(q)
    T, Hq, hd = q.shape
    Hkv = k_cache.shape[1]
    BS = k_cache.shape[3]
    g = Hq // Hkv
    if scale is None:
        scale = 1.0 / math.sqrt(hd)
    k_flat = np.ascontiguousarray(k_cache).reshape(-1)
    v_flat = np.ascontiguousarray(v_cache).reshape(-1)
    out = np.zeros((T, Hq, hd), dtype=np.float64)
    for i in range(len(seq_lens)):
        q0, q1 = int(query_start_loc[i]), int(query_start_loc[i + 1])
        c = q1 - q0
        if c == 0:
            continue
        L = int(seq_lens[i])
        ctx = int(ctx_lens[i])
        K, V = gather_sequence(k_flat, v_flat, block_tables[i], L, Hkv, hd, BS)
        Q = _f64(q[q0:q1])                                   # [c, Hq, hd]
        rows = np.arange(c)[:, None] + ctx                   # absolute position of each query row
        cols = np.arange(L)[None, :]
        visible = cols <= rows                               # causal, own key included
        for h in range(Hq):
            S = scale * (Q[:, h, :] @ K[:, h // g, :].T)     # [c, L]
            S = np.where(visible, S, -np.inf)
            P = np.exp(S - S.max(axis=1, keepdims=True))
            P = P / P.sum(axis=1, keepdims=True)
            out[q0:q1, h, :] = P @ V[:, h // g, :]
    return out

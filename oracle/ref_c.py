"""ctypes loader for oracle/ref_omp.c (TEST INFRASTRUCTURE ONLY).

build() compiles the C file with gcc -fopenmp next to the source; attn_mixed() has the
same signature and meaning as oracle.ref_numpy.attn_mixed.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ref_omp.c")
_LIB = os.path.join(_HERE, "libooco_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        P = ctypes.c_void_p
        lib.ooco_oracle_attn_mixed.restype = ctypes.c_int
        lib.ooco_oracle_attn_mixed.argtypes = [P, P, P, P, P, P, P, P] + [ctypes.c_int] * 6 + [ctypes.c_double,
                                                                                             ctypes.c_int]
        lib.ooco_oracle_block_copy.restype = None
        lib.ooco_oracle_block_copy.argtypes = [P, P, P, P, P, P, ctypes.c_int64] + [ctypes.c_int] * 3
        _lib = lib
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def attn_mixed(q, k_cache, v_cache, block_tables, seq_lens, query_start_loc, ctx_lens, scale=None,
               num_threads: int = 0, return_threads: bool = False):
    lib = _load()
    q = np.ascontiguousarray(q, dtype=np.uint16)
    k = np.ascontiguousarray(k_cache, dtype=np.uint16)
    v = np.ascontiguousarray(v_cache, dtype=np.uint16)
    bt = np.ascontiguousarray(block_tables, dtype=np.int32)
    sl = np.ascontiguousarray(seq_lens, dtype=np.int32)
    qs = np.ascontiguousarray(query_start_loc, dtype=np.int32)
    cl = np.ascontiguousarray(ctx_lens, dtype=np.int32)
    T, Hq, hd = q.shape
    NB, Hkv, _, BS, _ = k.shape
    if scale is None:
        scale = 1.0 / math.sqrt(hd)
    out = np.zeros((T, Hq, hd), dtype=np.float64)
    maxb = bt.shape[1] if bt.ndim == 2 else 1
    rc = lib.ooco_oracle_attn_mixed(_p(q), _p(k), _p(v), _p(bt), _p(sl), _p(qs), _p(cl), _p(out), len(sl), Hq, Hkv,
                                    hd, BS, maxb, float(scale), int(num_threads))
    if rc < 0:
        raise ValueError(f"ooco_oracle_attn_mixed rejected its arguments (code {rc})")
    return (out, rc) if return_threads else out


def block_copy(k_src, v_src, k_dst, v_dst, src_ids, dst_ids):
    lib = _load()
    src = np.ascontiguousarray(src_ids, dtype=np.int64)
    dst = np.ascontiguousarray(dst_ids, dtype=np.int64)
    _, Hkv, hd, BS = v_src.shape
    assert k_dst.flags.c_contiguous and v_dst.flags.c_contiguous
    lib.ooco_oracle_block_copy(_p(k_src), _p(v_src), _p(k_dst), _p(v_dst), _p(src), _p(dst), len(src), Hkv, hd, BS)

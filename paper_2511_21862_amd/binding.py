"""Thin ctypes binding over libooco.so: argument marshalling only.

Function names equal the C entry points of include/ooco.h.  Device arguments are torch
tensors (used purely as device allocations: `.data_ptr()`), host arguments numpy int32 arrays.
Importing this module fails when the HIP library has not been built -- there is no fallback.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libooco.so")

OOCO_OK, OOCO_EINVAL, OOCO_ESHAPE, OOCO_ENOMEM, OOCO_EHIP = 0, -1, -2, -3, -4
_STATUS_NAMES = {0: "OOCO_OK", -1: "OOCO_EINVAL", -2: "OOCO_ESHAPE", -3: "OOCO_ENOMEM", -4: "OOCO_EHIP"}

EXPORTS = ["ooco_ctx_create", "ooco_ctx_destroy", "ooco_last_error", "ooco_set_option", "ooco_plan",
           "ooco_plan_dry_run", "ooco_plan_info", "ooco_plan_kernels", "ooco_profile_read", "ooco_profile_read_calls", "ooco_trace_read", "ooco_attn_mixed", "ooco_attn_mixed_static", "ooco_kv_block_copy", "ooco_kv_append", "ooco_predict_latency", "ooco_mix_decoding_select",
           "ooco_migration_preference", "ooco_migration_select", "ooco_eviction_victims"]

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2511_21862_amd.build` "
                      "(the HIP library is the only implementation; there is no fallback)")

# torch first: its wheel brings a HIP runtime of its own, and the one that is loaded first serves the whole process --
# with libooco.so (linked against the system's runtime) loaded before torch, the process holds two runtimes and the
# second to touch the GPU finds no device
try:
    import torch  # noqa: F401
except ImportError:      # host-only use (planner, model, scheduling functions)
    pass

_lib = ctypes.CDLL(LIB_PATH)
_P = ctypes.c_void_p
_lib.ooco_ctx_create.restype = ctypes.c_int
_lib.ooco_ctx_create.argtypes = [ctypes.POINTER(_P), ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                 ctypes.c_int64, ctypes.c_int, ctypes.c_float, _P, ctypes.c_size_t]
_lib.ooco_ctx_destroy.restype = ctypes.c_int
_lib.ooco_ctx_destroy.argtypes = [_P]
_lib.ooco_last_error.restype = ctypes.c_char_p
_lib.ooco_last_error.argtypes = [_P]
_lib.ooco_set_option.restype = ctypes.c_int
_lib.ooco_set_option.argtypes = [_P, ctypes.c_char_p, ctypes.c_int64]
_lib.ooco_plan.restype = ctypes.c_int
_lib.ooco_plan.argtypes = [_P, ctypes.c_int, _P, _P, _P]
_lib.ooco_plan_dry_run.restype = ctypes.c_int
_lib.ooco_plan_dry_run.argtypes = ([ctypes.c_int] * 6 + [ctypes.c_size_t] + [ctypes.c_int64] * 3 + [ctypes.c_int, _P, _P, _P]
                                   + [_P, ctypes.c_int64, _P, ctypes.c_int64, _P, ctypes.c_char_p, ctypes.c_size_t, _P, ctypes.c_int64, ctypes.c_int64])
_lib.ooco_plan_info.restype = ctypes.c_int
_lib.ooco_plan_info.argtypes = [_P] + [ctypes.POINTER(ctypes.c_int64)] * 5
_lib.ooco_plan_kernels.restype = ctypes.c_int
_lib.ooco_plan_kernels.argtypes = [_P, ctypes.c_char_p, ctypes.c_size_t]
_lib.ooco_profile_read.restype = ctypes.c_int
_lib.ooco_profile_read.argtypes = [_P, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
_lib.ooco_profile_read_calls.restype = ctypes.c_int
_lib.ooco_profile_read_calls.argtypes = [_P, _P, ctypes.c_int64, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
_lib.ooco_trace_read.restype = ctypes.c_int
_lib.ooco_trace_read.argtypes = [_P, _P, ctypes.c_int64, ctypes.POINTER(ctypes.c_int64)]
_lib.ooco_attn_mixed.restype = ctypes.c_int
_lib.ooco_attn_mixed.argtypes = [_P] * 9 + [ctypes.c_int, ctypes.c_int, _P]
_lib.ooco_attn_mixed_static.restype = ctypes.c_int
_lib.ooco_attn_mixed_static.argtypes = ([ctypes.c_int] * 5 + [ctypes.c_float] + [_P] * 11 + [ctypes.c_int, ctypes.c_int, _P,
                                        ctypes.c_char_p, ctypes.c_size_t])
_lib.ooco_kv_block_copy.restype = ctypes.c_int
_lib.ooco_kv_block_copy.argtypes = [_P] * 7 + [ctypes.c_int64, _P]
_lib.ooco_kv_append.restype = ctypes.c_int
_lib.ooco_kv_append.argtypes = [_P] * 8 + [ctypes.c_int, ctypes.c_int, _P]



class ModelParams(ctypes.Structure):
    """ooco_model_params: F_ap, F_ad [FLOP/s], M_a [bytes/s], O_p, O_d [s]."""
    _fields_ = [(n, ctypes.c_double) for n in ("F_ap", "F_ad", "M_a", "O_p", "O_d")]


_lib.ooco_predict_latency.restype = ctypes.c_int
_lib.ooco_predict_latency.argtypes = ([ctypes.POINTER(ModelParams)] + [ctypes.c_int] * 6 + [_P, _P, ctypes.POINTER(ctypes.c_double),
                                      ctypes.c_char_p, ctypes.c_size_t])

_lib.ooco_mix_decoding_select.restype = ctypes.c_int
_lib.ooco_mix_decoding_select.argtypes = ([ctypes.POINTER(ModelParams)] + [ctypes.c_int] * 4 + [ctypes.c_double, ctypes.c_int, _P,
                                          ctypes.c_int, _P, ctypes.c_int, _P, _P, ctypes.POINTER(ctypes.c_double),
                                          ctypes.c_char_p, ctypes.c_size_t])


class OocoError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{_STATUS_NAMES.get(status, status)}: {message}")
        self.status = status
        self.message = message


def _dev(t) -> int:
    """Device pointer of a torch tensor (None -> NULL)."""
    if t is None:
        return 0
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("tensors passed to libooco must be contiguous")
    return t.data_ptr()


def _host_i32(a):
    if a is None:
        return None, 0
    arr = np.ascontiguousarray(a, dtype=np.int32)
    return arr, arr.ctypes.data


def _stream_handle(stream) -> int:
    if stream is None:
        import torch

        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def ooco_last_error(ctx) -> str:
    s = _lib.ooco_last_error(ctx)
    return s.decode() if s else ""


def _check(ctx, status: int):
    if status != OOCO_OK:
        raise OocoError(status, ooco_last_error(ctx))


def ooco_ctx_create(num_q_heads, num_kv_heads, head_dim, block_size, num_blocks, max_blocks_per_seq,
                    softmax_scale=0.0, workspace=None, workspace_bytes=0):
    h = _P()
    st = _lib.ooco_ctx_create(ctypes.byref(h), num_q_heads, num_kv_heads, head_dim, block_size, num_blocks,
                              max_blocks_per_seq, softmax_scale, _dev(workspace), workspace_bytes)
    _check(None, st)
    return h


def ooco_ctx_destroy(ctx) -> None:
    _check(None, _lib.ooco_ctx_destroy(ctx))


def ooco_set_option(ctx, name: str, value: int) -> None:
    _check(ctx, _lib.ooco_set_option(ctx, name.encode() if name is not None else None, value))


def ooco_plan(ctx, num_seqs, h_seq_lens, h_query_start_loc, h_ctx_lens) -> None:
    a, pa = _host_i32(h_seq_lens)
    b, pb = _host_i32(h_query_start_loc)
    c, pc = _host_i32(h_ctx_lens)
    _check(ctx, _lib.ooco_plan(ctx, num_seqs, pa, pb, pc))


def ooco_plan_dry_run(num_q_heads, num_kv_heads, head_dim, block_size, max_blocks_per_seq, num_cus, workspace_bytes,
                      h_seq_lens, h_query_start_loc, h_ctx_lens, decode_segments=0, decode_tail_pct=0,
                      decode_tail_blocks=8, num_seqs=None, xcd_weights=None, prefill_split=0, decode_piece_pad=-1) -> dict:
    """Host-only planner run; returns the work the kernels derive from the plan as numpy arrays."""
    a, pa = _host_i32(h_seq_lens)
    b, pb = _host_i32(h_query_start_loc)
    c, pc = _host_i32(h_ctx_lens)
    n = len(a) if num_seqs is None else num_seqs
    counts = np.zeros(6, dtype=np.int64)
    msg = ctypes.create_string_buffer(512)
    xw, pxw = _host_i32(xcd_weights) if xcd_weights is not None else (None, 0)

    def call(dptr, dcap, pptr, pcap):
        return _lib.ooco_plan_dry_run(num_q_heads, num_kv_heads, head_dim, block_size, max_blocks_per_seq, num_cus,
                                      workspace_bytes, decode_segments, decode_tail_pct, decode_tail_blocks, n, pa, pb, pc,
                                      dptr, dcap, pptr, pcap,
                                      counts.ctypes.data, msg, 512, pxw, prefill_split, decode_piece_pad)

    st = call(0, 0, 0, 0)
    if st != OOCO_OK:
        raise OocoError(st, msg.value.decode())
    d = np.zeros((int(counts[0]), 5), dtype=np.int32)
    p = np.zeros((int(counts[1]), 5), dtype=np.int32)
    st = call(d.ctypes.data, len(d), p.ctypes.data, len(p))
    if st != OOCO_OK:
        raise OocoError(st, msg.value.decode())
    return dict(decode_pieces=d, prefill_tiles=p, decode_runs=int(counts[2]), slots=int(counts[3]),
                tail_runs=int(counts[4]), prefill_parts=int(counts[5]))


def ooco_plan_info(ctx) -> dict:
    v = [ctypes.c_int64() for _ in range(5)]
    _check(ctx, _lib.ooco_plan_info(ctx, *[ctypes.byref(x) for x in v]))
    return dict(decode_waves=v[0].value, prefill_tiles=v[1].value, decode_blocks=v[2].value,
                workspace_used=v[3].value, prefill_parts=v[4].value)


def ooco_plan_kernels(ctx) -> list:
    buf = ctypes.create_string_buffer(256)
    _check(ctx, _lib.ooco_plan_kernels(ctx, buf, 256))
    return [k for k in buf.value.decode().split(";") if k]


def ooco_trace_read(ctx, cap_waves=1 << 16):
    """uint64 [waves, 4] device time stamps (100 MHz) of the last traced call's decode waves."""
    buf = np.zeros((cap_waves, 4), dtype=np.uint64)
    n = ctypes.c_int64()
    _check(ctx, _lib.ooco_trace_read(ctx, buf.ctypes.data, cap_waves, ctypes.byref(n)))
    return buf[: min(n.value, cap_waves)]


def ooco_profile_read_calls(ctx, cap=1024) -> dict:
    """Like ooco_profile_read, plus `per_call` = float64 [calls, 3] (prefill ms, decode ms, whole call ms)."""
    buf = np.zeros((cap, 3), dtype=np.float64)
    ms = (ctypes.c_double * 3)()
    n = ctypes.c_int64()
    _check(ctx, _lib.ooco_profile_read_calls(ctx, buf.ctypes.data, cap, ms, ctypes.byref(n)))
    return dict(prefill_ms=ms[0], decode_ms=ms[1], call_ms=ms[2], calls=n.value, per_call=buf[: min(n.value, cap)])


def ooco_profile_read(ctx) -> dict:
    ms = (ctypes.c_double * 3)()
    n = ctypes.c_int64()
    _check(ctx, _lib.ooco_profile_read(ctx, ms, ctypes.byref(n)))
    return dict(prefill_ms=ms[0], decode_ms=ms[1], call_ms=ms[2], calls=n.value)


def ooco_attn_mixed(ctx, q, k_cache, v_cache, block_tables, seq_lens, query_start_loc, ctx_lens, out, num_seqs,
                    total_q_tokens, stream=None) -> None:
    _check(ctx, _lib.ooco_attn_mixed(ctx, _dev(q), _dev(k_cache), _dev(v_cache), _dev(block_tables), _dev(seq_lens),
                                     _dev(query_start_loc), _dev(ctx_lens), _dev(out), num_seqs, total_q_tokens,
                                     _stream_handle(stream)))


def ooco_attn_mixed_static(num_q_heads, num_kv_heads, head_dim, block_size, max_blocks_per_seq, softmax_scale, h_seq_lens,
                           h_query_start_loc, h_ctx_lens, q, k_cache, v_cache, block_tables, seq_lens, query_start_loc,
                           ctx_lens, out, num_seqs, total_q_tokens, stream=None) -> None:
    a, pa = _host_i32(h_seq_lens)
    b, pb = _host_i32(h_query_start_loc)
    c, pc = _host_i32(h_ctx_lens)
    msg = ctypes.create_string_buffer(512)
    st = _lib.ooco_attn_mixed_static(num_q_heads, num_kv_heads, head_dim, block_size, max_blocks_per_seq, softmax_scale,
                                     pa, pb, pc, _dev(q), _dev(k_cache), _dev(v_cache), _dev(block_tables), _dev(seq_lens),
                                     _dev(query_start_loc), _dev(ctx_lens), _dev(out), num_seqs, total_q_tokens,
                                     _stream_handle(stream), msg, 512)
    if st != OOCO_OK:
        raise OocoError(st, msg.value.decode())


def ooco_kv_block_copy(ctx, k_src, v_src, k_dst, v_dst, src_block_ids, dst_block_ids, num_pairs, stream=None) -> None:
    _check(ctx, _lib.ooco_kv_block_copy(ctx, _dev(k_src), _dev(v_src), _dev(k_dst), _dev(v_dst), _dev(src_block_ids),
                                        _dev(dst_block_ids), num_pairs, _stream_handle(stream)))


def ooco_kv_append(ctx, k_new, v_new, k_cache, v_cache, block_tables, query_start_loc, ctx_lens, num_seqs,
                   total_q_tokens, stream=None) -> None:
    _check(ctx, _lib.ooco_kv_append(ctx, _dev(k_new), _dev(v_new), _dev(k_cache), _dev(v_cache), _dev(block_tables),
                                    _dev(query_start_loc), _dev(ctx_lens), num_seqs, total_q_tokens,
                                    _stream_handle(stream)))


def ooco_predict_latency(params, num_q_heads, num_kv_heads, head_dim, h_query_start_loc, h_ctx_lens,
                         bytes_per_value=2, causal_flops=False) -> dict:
    """params: dict or ModelParams.  Returns the model's outputs by name (argument marshalling only)."""
    p = params if isinstance(params, ModelParams) else ModelParams(**{k: float(params[k]) for k, _ in ModelParams._fields_})
    a, pa = _host_i32(h_query_start_loc)
    c, pc = _host_i32(h_ctx_lens)
    out = (ctypes.c_double * 8)()
    msg = ctypes.create_string_buffer(256)
    st = _lib.ooco_predict_latency(ctypes.byref(p), num_q_heads, num_kv_heads, head_dim, bytes_per_value, int(bool(causal_flops)),
                                   len(c), pa, pc,
                                   out, msg, 256)
    if st != OOCO_OK:
        raise OocoError(st, msg.value.decode())
    names = ("latency", "prefill", "decode", "overhead", "flops", "bytes", "compute_bound", "memory_bound")
    return dict(zip(names, list(out)))


def ooco_mix_decoding_select(params, num_q_heads, num_kv_heads, head_dim, slo_s, online_lens, offline_lens, random_order,
                             bytes_per_value=2) -> dict:
    """Returns dict(selected=bool array over the offline candidates, latency=predicted seconds)."""
    p = params if isinstance(params, ModelParams) else ModelParams(**{k: float(params[k]) for k, _ in ModelParams._fields_})
    on, pon = _host_i32(online_lens)
    off, poff = _host_i32(offline_lens)
    order, pord = _host_i32(random_order)
    sel = np.zeros(max(len(off), 1), dtype=np.uint8)
    lat = ctypes.c_double()
    msg = ctypes.create_string_buffer(256)
    st = _lib.ooco_mix_decoding_select(ctypes.byref(p), num_q_heads, num_kv_heads, head_dim, bytes_per_value, float(slo_s),
                                       len(on), pon, len(off), poff, len(order), pord, sel.ctypes.data, ctypes.byref(lat),
                                       msg, 256)
    if st != OOCO_OK:
        raise OocoError(st, msg.value.decode())
    return dict(selected=sel[: len(off)].astype(bool), latency=lat.value)


_lib.ooco_migration_preference.restype = ctypes.c_int
_lib.ooco_migration_preference.argtypes = ([ctypes.POINTER(ModelParams)] + [ctypes.c_int] * 4 + [ctypes.c_double, ctypes.c_int, _P]
                                           + [ctypes.c_int] * 3 + [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, _P, _P,
                                                                   ctypes.c_char_p, ctypes.c_size_t])
_lib.ooco_migration_select.restype = ctypes.c_int
_lib.ooco_migration_select.argtypes = ([ctypes.POINTER(ModelParams)] + [ctypes.c_int] * 4 + [ctypes.c_double, ctypes.c_int, _P,
                                                                                            ctypes.c_int, _P, ctypes.c_int32,
                                                                                            ctypes.c_int, ctypes.c_int64,
                                                                                            ctypes.c_int, _P, _P,
                                                                                            ctypes.c_char_p, ctypes.c_size_t])
_lib.ooco_eviction_victims.restype = ctypes.c_int
_lib.ooco_eviction_victims.argtypes = [ctypes.c_int, _P, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int, _P, _P, _P,
                                       ctypes.c_char_p, ctypes.c_size_t]

MIGRATION_BRANCHES = ("none", "saturated", "reach", "shortest")


def _model_params(params):
    return params if isinstance(params, ModelParams) else ModelParams(**{k: float(params[k]) for k, _ in ModelParams._fields_})


def ooco_migration_preference(params, num_q_heads, num_kv_heads, head_dim, slo_s, batch_lens, all_included, bs_sat,
                              block_size, capacity_blocks, len_min, len_max, bytes_per_value=2) -> dict:
    """Returns dict(pref=length or None, branch=one of MIGRATION_BRANCHES)."""
    p = _model_params(params)
    b, pb = _host_i32(batch_lens)
    pref, branch = ctypes.c_int32(), ctypes.c_int32()
    msg = ctypes.create_string_buffer(256)
    st = _lib.ooco_migration_preference(ctypes.byref(p), num_q_heads, num_kv_heads, head_dim, bytes_per_value, float(slo_s),
                                        len(b), pb, int(bool(all_included)), bs_sat, block_size, capacity_blocks, len_min,
                                        len_max, ctypes.addressof(pref), ctypes.addressof(branch), msg, 256)
    if st != OOCO_OK:
        raise OocoError(st, msg.value.decode())
    return dict(pref=None if pref.value < 0 else pref.value, branch=MIGRATION_BRANCHES[branch.value])


def ooco_migration_select(params, num_q_heads, num_kv_heads, head_dim, slo_s, batch_lens, relaxed_lens, pref, block_size,
                          capacity_blocks, max_migrate, bytes_per_value=2) -> list:
    """Indices into relaxed_lens of the requests to migrate, in the order taken."""
    p = _model_params(params)
    b, pb = _host_i32(batch_lens)
    r, pr = _host_i32(relaxed_lens)
    chosen = np.zeros(max(1, min(max_migrate, len(r))), dtype=np.int32)
    n = ctypes.c_int32()
    msg = ctypes.create_string_buffer(256)
    st = _lib.ooco_migration_select(ctypes.byref(p), num_q_heads, num_kv_heads, head_dim, bytes_per_value, float(slo_s),
                                    len(b), pb, len(r), pr, pref, block_size, capacity_blocks, max_migrate,
                                    chosen.ctypes.data, ctypes.addressof(n), msg, 256)
    if st != OOCO_OK:
        raise OocoError(st, msg.value.decode())
    return [int(x) for x in chosen[: n.value]]


def ooco_eviction_victims(offline_lens, need_blocks, block_size, batch_size, bs_sat) -> dict:
    """Returns dict(victims=[indices in the order taken], enough=bool)."""
    o, po = _host_i32(offline_lens)
    victims = np.zeros(max(1, len(o)), dtype=np.int32)
    n, enough = ctypes.c_int32(), ctypes.c_int32()
    msg = ctypes.create_string_buffer(256)
    st = _lib.ooco_eviction_victims(len(o), po, need_blocks, block_size, batch_size, bs_sat, victims.ctypes.data,
                                    ctypes.addressof(n), ctypes.addressof(enough), msg, 256)
    if st != OOCO_OK:
        raise OocoError(st, msg.value.decode())
    return dict(victims=[int(x) for x in victims[: n.value]], enough=bool(enough.value))


class Context:
    """RAII holder of one ooco_ctx (no arithmetic here either)."""

    def __init__(self, Hq, Hkv, hd, BS, num_blocks, max_blocks_per_seq, scale=0.0, workspace=None,
                 workspace_bytes=0):
        self.h = ooco_ctx_create(Hq, Hkv, hd, BS, num_blocks, max_blocks_per_seq, scale, workspace, workspace_bytes)
        self._workspace = workspace

    def close(self):
        if self.h is not None:
            ooco_ctx_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    def set_option(self, name, value):
        ooco_set_option(self.h, name, value)

    def plan(self, seq_lens, query_start_loc, ctx_lens):
        ooco_plan(self.h, len(seq_lens), seq_lens, query_start_loc, ctx_lens)

    def plan_info(self):
        return ooco_plan_info(self.h)

    def plan_kernels(self):
        return ooco_plan_kernels(self.h)

    def profile_read_calls(self, cap=1024):
        return ooco_profile_read_calls(self.h, cap)

    def profile_read(self):
        return ooco_profile_read(self.h)

    def trace_read(self):
        return ooco_trace_read(self.h)

    def attn_mixed(self, q, k_cache, v_cache, block_tables, seq_lens, query_start_loc, ctx_lens, out, stream=None):
        ooco_attn_mixed(self.h, q, k_cache, v_cache, block_tables, seq_lens, query_start_loc, ctx_lens, out,
                        int(seq_lens.shape[0]), int(q.shape[0]), stream)

    def kv_append(self, k_new, v_new, k_cache, v_cache, block_tables, query_start_loc, ctx_lens, stream=None):
        ooco_kv_append(self.h, k_new, v_new, k_cache, v_cache, block_tables, query_start_loc, ctx_lens,
                       int(ctx_lens.shape[0]), int(k_new.shape[0]), stream)

    def kv_block_copy(self, k_src, v_src, k_dst, v_dst, src_ids, dst_ids, stream=None):
        ooco_kv_block_copy(self.h, k_src, v_src, k_dst, v_dst, src_ids, dst_ids, int(src_ids.shape[0]), stream)

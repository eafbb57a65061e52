"""Layer-level preemption of an offline decode iteration by an online request (paper Section 3.4.1), built on
the library's calls only: the iteration is a loop of attention layers (one ooco_attn_mixed per layer); a flag
that any host thread may raise is looked at between layers; on preemption the victims named by
ooco_eviction_victims leave the KV pool through ooco_kv_block_copy, the online work runs in the freed blocks,
the victims come back, and the iteration resumes at the layer where it stopped.

Host control flow and data movement only; every number is computed by the library's kernels or host functions.
"""
from __future__ import annotations

import threading
import time
from typing import Callable, Optional

import numpy as np

from . import binding as B
from . import workloads as W


class PreemptFlag:
    """The preemption request: raised from any host thread (a scheduler, a timer), read by the layer loop."""

    def __init__(self):
        self._ev = threading.Event()
        self.t_raised: Optional[float] = None

    def raise_now(self) -> None:
        self.t_raised = time.perf_counter()
        self._ev.set()

    def is_raised(self) -> bool:
        return self._ev.is_set()


def run_layers(num_layers: int, enqueue_layer: Callable[[int], None], stream, flag: Optional[PreemptFlag] = None,
               on_preempt: Optional[Callable[[int], Optional[dict]]] = None, run_ahead: int = 2,
               on_layer: Optional[Callable[[int], None]] = None) -> Optional[dict]:
    """Enqueues layers 0 .. num_layers-1 on `stream`, never more than `run_ahead` layers ahead of the GPU.  Before
    every enqueue the flag is looked at; the first time it is found raised, the layers already enqueued are
    allowed to finish (nothing further is enqueued), `on_preempt(next_layer)` runs -- it may enqueue and wait for
    whatever the preempting request needs -- and the loop then goes on with `next_layer`.  Returns None when no
    preemption happened, else a dict: the layer the iteration resumed at, the time from the raising of the flag
    to the GPU being idle (the preemption latency), the duration of the handler, and the handler's own report."""
    import torch

    events = []
    report = None
    layer = 0
    while layer < num_layers:
        if len(events) >= run_ahead:
            events[-run_ahead].synchronize()
        if flag is not None and report is None and flag.is_raised():
            t_seen = time.perf_counter()
            stream.synchronize()                      # the layers in flight complete
            t_idle = time.perf_counter()
            info = on_preempt(layer) if on_preempt is not None else None
            stream.synchronize()
            t_back = time.perf_counter()
            report = dict(resumed_at_layer=layer, preempt_latency_ms=(t_idle - flag.t_raised) * 1e3,
                          flag_to_seen_ms=(t_seen - flag.t_raised) * 1e3, handler_ms=(t_back - t_idle) * 1e3)
            report.update(info or {})
            events = []
        if on_layer is not None:
            on_layer(layer)
        enqueue_layer(layer)
        ev = torch.cuda.Event()
        ev.record(stream)
        events.append(ev)
        layer += 1
    stream.synchronize()
    return report


class Eviction:
    """Victims of one preemption and their way out of and back into the KV pool.

    `offline_lens` are the KV lengths of the offline requests of the node (block_tables row i belongs to request
    i), `need_blocks` what the online request lacks, `bs_sat` the batch size at which the node's decode step is
    compute-bound: ooco_eviction_victims takes long requests first on a compute-bound node and short ones first
    otherwise.  The victims' blocks are copied, in block-table order, into slots 0..n-1 of the staging pool."""

    def __init__(self, ctx: B.Context, offline_lens, block_tables, need_blocks: int, bs_sat: int, block_size: int = 16):
        import torch

        self.ctx = ctx
        r = B.ooco_eviction_victims(offline_lens, int(need_blocks), block_size, len(offline_lens), int(bs_sat))
        self.victims = list(r["victims"])
        self.enough = bool(r["enough"])
        nb = (np.asarray(offline_lens, dtype=np.int64) + block_size - 1) // block_size
        parts = [np.asarray(block_tables[v, : int(nb[v])], dtype=np.int64) for v in self.victims]
        self.block_ids = np.concatenate(parts) if parts else np.zeros(0, np.int64)
        self.src_d = torch.from_numpy(self.block_ids).cuda()
        self.stage_d = torch.arange(len(self.block_ids), dtype=torch.int64, device="cuda")

    @property
    def num_blocks(self) -> int:
        return int(len(self.block_ids))

    def evict(self, k_cache, v_cache, k_stage, v_stage, stream=None) -> None:
        self.ctx.kv_block_copy(k_cache, v_cache, k_stage, v_stage, self.src_d, self.stage_d, stream)

    def restore(self, k_cache, v_cache, k_stage, v_stage, stream=None, dst_ids=None) -> None:
        """Back into the blocks they came from, or into `dst_ids` (device int64, one per staged block)."""
        self.ctx.kv_block_copy(k_stage, v_stage, k_cache, v_cache, self.stage_d, self.src_d if dst_ids is None else dst_ids,
                               stream)


def staging_pools(b: W.Batch, num_blocks: int):
    """Empty K and V staging pools of `num_blocks` blocks with the geometry of batch `b` (device memory only)."""
    import torch

    return (torch.empty((num_blocks,) + tuple(b.k_cache.shape[1:]), dtype=torch.bfloat16, device="cuda"),
            torch.empty((num_blocks,) + tuple(b.v_cache.shape[1:]), dtype=torch.bfloat16, device="cuda"))

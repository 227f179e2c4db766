"""Trace-driven serving loop: the library's schedulers decide each iteration's prefill and decode batches, the
library's step calls run them through the layer stack on the GPU.

This module only moves descriptors: it copies the scheduler's host arrays to the device, gathers the synthetic
layer-stack inputs of the scheduled tokens, calls the step and reports the time back to the scheduler.  There is
no embedding, sampling or LM head (the path is the layer stack), so the input of the token at position `pos` of
request `rid` is row (rid * 8191 + pos) mod R of a fixed random pool, and a request simply stops after output_len
tokens.
"""
from __future__ import annotations

import time
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np
import torch

from . import binding as nx
from .synth import DecodeBatch, ModelShape, PrefillBatch

ROW_STRIDE = 8191


def token_rows(rid: int, start: int, n: int, pool_rows: int) -> np.ndarray:
    return (rid * ROW_STRIDE + start + np.arange(n, dtype=np.int64)) % pool_rows


@dataclass
class IterationRecord:
    now_s: float
    end_s: float
    step_ms: float                 # host clock around the step, GPU drained on both sides
    prefill_tokens: int
    decode_reqs: int
    kv_used_pages: int
    prefill: List[Tuple[int, int, int]] = field(default_factory=list)   # (request, prefix, chunk)
    decode: List[Tuple[int, int]] = field(default_factory=list)         # (request, context)
    checksum: Optional[Tuple[int, int]] = None


class TraceRunner:
    """One model replica serving one trace.  `split` is (prefill CUs, decode CUs) or None for the serialized step."""

    def __init__(self, shape: ModelShape, n_layers: int, weights_for_layer, *, policy: int, token_budget: int,
                 max_decode_reqs: int, n_pages: int, gamma: float = 15.0, max_prefill_reqs: int = 8,
                 max_positions: int = 10240, split: Optional[Tuple[int, int]] = None, seed: int = 0,
                 pool_rows: int = 16384, page_order=None, device: int = 0):
        self.shape, self.n_layers = shape, n_layers
        self.ctx = nx.Nexus(shape, max_prefill_tokens=token_budget, max_prefill_reqs=max_prefill_reqs,
                            max_decode_reqs=max_decode_reqs, max_positions=max_positions, device=device, n_layers=n_layers)
        for l in range(n_layers):
            self.ctx.load_layer(l, weights_for_layer(l))
        self.kv = self.ctx.alloc_kv(n_pages, n_layers)
        self.sched = nx.Scheduler(policy, token_budget, max_decode_reqs, shape.page_size, n_pages, gamma=gamma,
                                  max_prefill_reqs=max_prefill_reqs, page_order=page_order)
        if split is None:
            self.ctx.set_cu_split(nx.CUS_ALL, nx.CUS_ALL)
        else:
            self.ctx.set_cu_split(*split)
        g = torch.Generator(device=self.ctx.device)
        g.manual_seed(seed * 104729 + 71)
        self.x_pool = torch.randn((pool_rows, shape.hidden), generator=g, device=self.ctx.device).to(torch.bfloat16)
        self.pool_rows = pool_rows
        self.records: List[IterationRecord] = []
        self.keep_outputs = False
        self.outputs = []          # (iteration, y_prefill, y_decode) when keep_outputs

    def submit(self, trace: Sequence[Tuple[float, int, int]]):
        for a, p, o in trace:
            self.sched.submit(a, p, o)

    def _gather(self, rows: np.ndarray) -> torch.Tensor:
        idx = torch.from_numpy(rows).to(self.ctx.device)
        return self.x_pool.index_select(0, idx)

    def step(self, now_s: float, end_s: Optional[float] = None, checksum: bool = False) -> IterationRecord:
        """One iteration starting at now_s.  With end_s the scheduler is told the iteration ended then, whatever
        the step took (a virtual clock: decisions do not depend on the hardware); otherwise at now_s + measured."""
        it = self.sched.next(now_s)
        dev = self.ctx.device
        pb = db = None
        if len(it.prefill_req):
            rows = np.concatenate([token_rows(int(r), int(p), int(n), self.pool_rows)
                                   for r, p, n in zip(it.prefill_req, it.prefill_prefix, it.prefill_chunk)])
            pb = nx.DevPrefill(PrefillBatch(self._gather(rows), it.prefill_cu_chunk, it.prefill_prefix, it.prefill_page_table), dev)
        if len(it.decode_req):
            rows = np.array([token_rows(int(r), int(c), 1, self.pool_rows)[0] for r, c in zip(it.decode_req, it.decode_ctx)])
            db = nx.DevDecode(DecodeBatch(self._gather(rows), it.decode_ctx, it.decode_page_table), dev)
        torch.cuda.synchronize(dev)
        layers = (0, self.n_layers)
        t0 = time.perf_counter()
        if pb is not None and db is not None:
            self.ctx.mixed_step(pb, db, self.kv, layers=layers)
        elif pb is not None:
            self.ctx.prefill_chunk(pb, self.kv, layers=layers)
        elif db is not None:
            self.ctx.decode_step(db, self.kv, layers=layers)
        self.ctx.sync()
        step_ms = (time.perf_counter() - t0) * 1e3
        if end_s is None:
            end_s = now_s + step_ms * 1e-3
        self.sched.commit(end_s)
        rec = IterationRecord(now_s, end_s, step_ms, int(it.prefill_chunk.sum()), len(it.decode_req), it.kv_used_pages,
                              list(zip(it.prefill_req.tolist(), it.prefill_prefix.tolist(), it.prefill_chunk.tolist())),
                              list(zip(it.decode_req.tolist(), it.decode_ctx.tolist())))
        if checksum:
            def h(t):
                return 0 if t is None else int(t.y.view(torch.int16).to(torch.int64).sum().item())
            rec.checksum = (h(pb), h(db))
        if self.keep_outputs:
            self.outputs.append((len(self.records), None if pb is None else pb.y.clone(), None if db is None else db.y.clone()))
        self.records.append(rec)
        return rec

    def run(self, n_iterations: int, fixed_dt: Optional[float] = None, checksum: bool = False):
        """fixed_dt: iteration i runs from i * fixed_dt to (i + 1) * fixed_dt on the scheduler's clock."""
        for _ in range(n_iterations):
            i = len(self.records)
            if fixed_dt is not None:
                self.step(i * fixed_dt, (i + 1) * fixed_dt, checksum)
            else:
                self.step(self.records[-1].end_s if self.records else 0.0, None, checksum)
        return self.records

    def report(self) -> dict:
        """Throughput over the measured step times plus the scheduler's serving metrics on its own clock."""
        busy = [r for r in self.records if r.prefill_tokens or r.decode_reqs]
        tokens = sum(r.prefill_tokens + r.decode_reqs for r in busy)
        gpu_s = sum(r.step_ms for r in busy) * 1e-3
        out = self.sched.summary()
        out.update({"iterations": len(self.records), "busy_iterations": len(busy), "tokens": tokens,
                    "gpu_seconds": gpu_s, "tokens_per_s": tokens / gpu_s if gpu_s else 0.0,
                    "mean_step_ms": 1e3 * gpu_s / len(busy) if busy else 0.0})
        return out

    def close(self):
        self.sched.close()
        self.ctx.close()

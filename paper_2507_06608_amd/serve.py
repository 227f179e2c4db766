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
                 pool_rows: int = 16384, page_order=None, device: int = 0, fused: bool = False):
        self.shape, self.n_layers = shape, n_layers
        # fused: coupled iterations run as ONE batch (the engine without phase separation), so the prefill side of
        # the context must hold the decode requests as well
        extra = max_decode_reqs if fused else 0
        self.ctx = nx.Nexus(shape, max_prefill_tokens=token_budget + extra, max_prefill_reqs=max_prefill_reqs + extra,
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
        self.split = split
        g = torch.Generator(device=self.ctx.device)
        g.manual_seed(seed * 104729 + 71)
        self.x_pool = torch.randn((pool_rows, shape.hidden), generator=g, device=self.ctx.device).to(torch.bfloat16)
        torch.cuda.synchronize(self.ctx.device)
        # CU-masked streams are blocking streams: anything issued on the NULL stream (torch's default) would wait
        # for a running phase and hold the next one back.  The loop's own copies and gathers go to a side stream.
        self.side = torch.cuda.Stream(device=self.ctx.device)
        self.pool_rows = pool_rows
        self.fused = fused
        self.records: List[IterationRecord] = []
        self.keep_outputs = False
        self.outputs = []          # (iteration, y_prefill, y_decode) when keep_outputs

    def submit(self, trace: Sequence[Tuple[float, int, int]]):
        for a, p, o in trace:
            self.sched.submit(a, p, o)

    def _gather(self, rows: np.ndarray) -> torch.Tensor:
        idx = torch.from_numpy(rows).to(self.ctx.device)
        return self.x_pool.index_select(0, idx)

    def _prefill_batch(self, it):
        with torch.cuda.stream(self.side):
            rows = np.concatenate([token_rows(int(r), int(p), int(n), self.pool_rows)
                                   for r, p, n in zip(it.prefill_req, it.prefill_prefix, it.prefill_chunk)])
            b = nx.DevPrefill(PrefillBatch(self._gather(rows), it.prefill_cu_chunk, it.prefill_prefix, it.prefill_page_table),
                              self.ctx.device)
        return b

    def _decode_batch(self, it):
        with torch.cuda.stream(self.side):
            rows = (it.decode_req.astype(np.int64) * ROW_STRIDE + it.decode_ctx) % self.pool_rows
            b = nx.DevDecode(DecodeBatch(self._gather(rows), it.decode_ctx, it.decode_page_table), self.ctx.device)
        return b

    def step(self, now_s: float, end_s: Optional[float] = None, checksum: bool = False) -> IterationRecord:
        """One iteration starting at now_s.  With end_s the scheduler is told the iteration ended then, whatever
        the step took (a virtual clock: decisions do not depend on the hardware); otherwise at now_s + measured."""
        it = self.sched.next(now_s)
        pb = self._prefill_batch(it) if len(it.prefill_req) else None
        db = self._decode_batch(it) if len(it.decode_req) else None
        self.side.synchronize()
        layers = (0, self.n_layers)
        if self.split is not None:
            # an iteration with one phase only takes every CU (both layouts stay alive, switching costs nothing)
            if pb is not None and db is not None:
                self.ctx.set_cu_split(*self.split)
            else:
                self.ctx.set_cu_split(nx.CUS_ALL, nx.CUS_ALL)
        fb = None
        if self.fused and pb is not None and db is not None:
            # one chunked-prefill batch whose last requests are the decode requests, as one-token chunks
            with torch.cuda.stream(self.side):
                width = max(it.prefill_page_table.shape[1], it.decode_page_table.shape[1])

                def pad(t):
                    out = np.full((t.shape[0], width), -1, np.int32)
                    out[:, :t.shape[1]] = t
                    return out
                n_p = int(it.prefill_cu_chunk[-1])
                cu = np.concatenate([it.prefill_cu_chunk, n_p + 1 + np.arange(len(it.decode_req), dtype=np.int32)]).astype(np.int32)
                fb = nx.DevPrefill(PrefillBatch(torch.cat([pb.x, db.x], 0), cu,
                                                np.concatenate([it.prefill_prefix, it.decode_ctx]).astype(np.int32),
                                                np.concatenate([pad(it.prefill_page_table), pad(it.decode_page_table)], 0)), self.ctx.device)
            self.side.synchronize()
        t0 = time.perf_counter()
        if fb is not None:
            self.ctx.fused_step(fb, len(it.decode_req), int(it.decode_ctx.max()) + 1, self.kv, layers=layers)
        elif pb is not None and db is not None:
            self.ctx.mixed_step(pb, db, self.kv, layers=layers)
        elif pb is not None:
            self.ctx.prefill_chunk(pb, self.kv, layers=layers)
        elif db is not None:
            self.ctx.decode_step(db, self.kv, layers=layers)
        self.ctx.sync()
        step_ms = (time.perf_counter() - t0) * 1e3
        if fb is not None:
            pb.y, db.y = fb.y[:pb.x.shape[0]], fb.y[pb.x.shape[0]:]
        if end_s is None:
            end_s = now_s + step_ms * 1e-3
        self.sched.commit(end_s)
        rec = IterationRecord(now_s, end_s, step_ms, int(it.prefill_chunk.sum()), len(it.decode_req), it.kv_used_pages,
                              list(zip(it.prefill_req.tolist(), it.prefill_prefix.tolist(), it.prefill_chunk.tolist())),
                              list(zip(it.decode_req.tolist(), it.decode_ctx.tolist())))
        if checksum:
            def h(t):
                return 0 if t is None else int(t.y.view(torch.int16).to(torch.int64).sum().item())
            with torch.cuda.stream(self.side):
                rec.checksum = (h(pb), h(db))
        if self.keep_outputs:
            with torch.cuda.stream(self.side):
                self.outputs.append((len(self.records), None if pb is None else pb.y.clone(), None if db is None else db.y.clone()))
            self.side.synchronize()
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

    def run_until_done(self, arrivals: Sequence[float], max_iterations: int = 100000):
        """Coupled iterations on the measured clock until every submitted request has finished; the clock jumps to
        the next arrival when an iteration finds nothing to do."""
        arrivals = sorted(arrivals)
        now = 0.0
        for _ in range(max_iterations):
            rec = self.step(now)
            now = rec.end_s
            if not rec.prefill_tokens and not rec.decode_reqs:
                if self.sched.summary()["n_finished"] == len(arrivals):
                    return self.records
                later = [a for a in arrivals if a > now]
                if later:
                    now = later[0]
        raise RuntimeError("trace did not finish")

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


class DecoupledRunner(TraceRunner):
    """The two phases as independent loops on one host thread (Sec. 5 runs them as separate coroutines): each phase
    launches its next step as soon as its previous one has completed, whatever the other phase is doing, so decode
    steps are not stretched to the length of a prefill chunk.  Needs a partitioned layout (two streams).

    The scheduler's clock is the host's, started at the first call, and jumps over stretches in which neither
    phase has anything to do (to the next arrival)."""

    def __init__(self, *args, **kwargs):
        self.borrow_idle_cus = kwargs.pop("borrow_idle_cus", True)
        super().__init__(*args, **kwargs)
        assert self.split is not None, "independent phase loops need a partitioned layout"
        # the partition controller (Alg. 1), off unless enable_controller() is called
        self.calibration = None
        # The controller moves the split in steps of 32 CUs (4 per XCD, one per shader engine of every XCD): workgroups
        # are dealt to the shader engines evenly whatever the CU mask, so a share that leaves one engine a CU short
        # runs no faster than the next lower multiple of 32 (measured on MI355X: decode on 72, 80 and 88 CUs takes
        # the time it takes on 64).
        self.ctrl = dict(alpha=1.3, beta=1.1, delta=1, kv_switch=0.7, total=8)
        self.switches: List[tuple] = []  # (time_s, old prefill CUs, new prefill CUs, host ms spent switching)
        self._last_shape = {}            # phase -> the quantities of its last batch the cost model needs
        self.calls: List[tuple] = []     # (op, phase, time, batch) in call order, for replay against another scheduler
        self.phase_records = {nx.PHASE_PREFILL: [], nx.PHASE_DECODE: []}   # (start_s, end_s, gpu_ms, tokens, host ms spent launching, ran alone)

    def _launch(self, phase: int, it, other_idle: bool) -> tuple:
        layers = (0, self.n_layers)
        # a phase that has the GPU to itself takes every CU (switching between the partitioned pair and the
        # unpartitioned stream costs nothing); the other phase may start on its own share before this step ends
        if self.borrow_idle_cus and other_idle:
            self.ctx.set_cu_split(nx.CUS_ALL, nx.CUS_ALL)
        else:
            self.ctx.set_cu_split(*self.split)
        if phase == nx.PHASE_PREFILL:
            b = self._prefill_batch(it)
            self.side.synchronize()          # the gather only; the other phase keeps running
            self.ctx.prefill_chunk(b, self.kv, layers=layers)
            desc = list(zip(it.prefill_req.tolist(), it.prefill_prefix.tolist(), it.prefill_chunk.tolist()))
            return b, desc, int(it.prefill_chunk.sum())
        b = self._decode_batch(it)
        self.side.synchronize()
        self.ctx.decode_step(b, self.kv, layers=layers)
        return b, list(zip(it.decode_req.tolist(), it.decode_ctx.tolist())), len(it.decode_req)

    def enable_controller(self, calibration, **params):
        """Repartition at run time: whenever a prefill batch is about to start next to a live decode pool, the
        library's controller is asked for the split (decode-prioritised above the KV-usage switch point,
        prefill-prioritised below, changes smaller than delta steps suppressed) and another stream pair is selected
        if it answers with a new one.  The switch waits for nothing: the decode step in flight finishes on its old
        share, the next one starts on the new pair (the library orders it after the old one)."""
        self.calibration = calibration
        self.ctrl.update(params)
        # Sec. 5: every layout the controller can choose exists before serving starts
        n_cus, total = self.ctx.cu_count, self.ctrl["total"]
        step = n_cus // total
        self.ctx.prepare_cu_splits([(step * k, n_cus - step * k) for k in range(1, total)])

    def _batch_shape(self, phase: int, it):
        if phase == nx.PHASE_PREFILL:
            pre, n = it.prefill_prefix.astype(np.float64), it.prefill_chunk.astype(np.float64)
            return dict(tokens=float(n.sum()), pairs=float((n * pre + n * (n + 1) / 2).sum()), kv=float((pre + n).sum()))
        return dict(reqs=float(len(it.decode_req)), kv=float((it.decode_ctx.astype(np.float64) + 1).sum()))

    def _maybe_repartition(self, now: float, kv_usage: float):
        p, d = self._last_shape.get(nx.PHASE_PREFILL), self._last_shape.get(nx.PHASE_DECODE)
        if self.calibration is None or p is None or d is None:
            return
        alg_p, alg_d = nx.cost_describe(self.shape, self.n_layers, p["tokens"], p["pairs"], p["kv"], d["reqs"], d["kv"])
        model = self.calibration.model(alg_p, alg_d)
        c = self.ctrl
        n_cus = self.ctx.cu_count
        step = n_cus // c["total"]
        cur = self.split[0] // step
        new = model.partition_controller(kv_usage, c["kv_switch"], cur, c["total"], c["alpha"], c["beta"], c["delta"])
        if new != cur:
            t_l = time.perf_counter()
            self.ctx.set_cu_split(step * new, n_cus - step * new)     # a pointer switch; nothing in flight is waited for
            self.switches.append((now, self.split[0], step * new, (time.perf_counter() - t_l) * 1e3))
            self.split = (step * new, n_cus - step * new)

    def run_decoupled(self, arrivals: Sequence[float], max_wall_s: float = 120.0):
        """Runs until every submitted request has finished.  `arrivals`: the arrival times that were submitted
        (to know where to jump when idle)."""
        arrivals = sorted(arrivals)
        t0, skipped = time.perf_counter(), 0.0
        busy = {nx.PHASE_PREFILL: None, nx.PHASE_DECODE: None}
        n_total, n_visible = len(arrivals), 0
        # an idle phase asks its scheduler again only when something it could act on has changed: a commit of
        # either phase (requests become ready, pages come back) or a new arrival becoming visible
        ask = {nx.PHASE_PREFILL: True, nx.PHASE_DECODE: True}
        while True:
            for phase in (nx.PHASE_DECODE, nx.PHASE_PREFILL):
                if busy[phase] is not None and self.ctx.phase_done(phase):
                    end = time.perf_counter() - t0 + skipped
                    gpu_ms = self.ctx.phase_wait(phase)
                    self.sched.commit_phase(phase, end)
                    b, desc, start, tokens, launch_ms, alone = busy[phase]
                    self.calls.append(("commit", phase, end, None))
                    self.phase_records[phase].append((start, end, gpu_ms, tokens, launch_ms, alone))
                    if self.keep_outputs:
                        with torch.cuda.stream(self.side):
                            self.outputs.append((phase, desc, b.y.clone()))
                        self.side.synchronize()
                    busy[phase] = None
                    ask[nx.PHASE_PREFILL] = ask[nx.PHASE_DECODE] = True
            now = time.perf_counter() - t0 + skipped
            while n_visible < n_total and arrivals[n_visible] <= now:
                n_visible += 1
                ask[nx.PHASE_PREFILL] = True
            work = {}
            for phase in (nx.PHASE_DECODE, nx.PHASE_PREFILL):
                if busy[phase] is None and ask[phase]:
                    ask[phase] = False
                    it = self.sched.next_phase(phase, now)
                    if len(it.prefill_req) if phase == nx.PHASE_PREFILL else len(it.decode_req):
                        work[phase] = it
            for phase, it in work.items():
                self._last_shape[phase] = self._batch_shape(phase, it)
            if nx.PHASE_PREFILL in work and (busy[nx.PHASE_DECODE] is not None or nx.PHASE_DECODE in work):
                it = work[nx.PHASE_PREFILL]
                self._maybe_repartition(now, it.kv_used_pages / it.kv_total_pages)
            for phase, it in work.items():
                alone = busy[1 - phase] is None and (1 - phase) not in work
                t_l = time.perf_counter()
                b, desc, tokens = self._launch(phase, it, alone)
                busy[phase] = (b, desc, now, tokens, (time.perf_counter() - t_l) * 1e3, alone)
                self.calls.append(("next", phase, now, desc))
            if busy[nx.PHASE_PREFILL] is None and busy[nx.PHASE_DECODE] is None:
                if n_visible == n_total and self.sched.summary()["n_finished"] == n_total:
                    break
                if n_visible < n_total:       # nothing in flight and nothing to start: jump to the next arrival
                    skipped += max(0.0, arrivals[n_visible] - (time.perf_counter() - t0 + skipped))
            if time.perf_counter() - t0 > max_wall_s:
                raise RuntimeError("decoupled run exceeded its wall-clock limit")
        self.ctx.sync()

    def report_decoupled(self) -> dict:
        out = self.sched.summary()
        for phase, name in ((nx.PHASE_PREFILL, "prefill"), (nx.PHASE_DECODE, "decode")):
            recs = self.phase_records[phase]
            out[f"{name}_steps"] = len(recs)
            out[f"{name}_mean_gpu_ms"] = float(np.mean([r[2] for r in recs])) if recs else 0.0
            out[f"{name}_mean_wall_ms"] = float(np.mean([(r[1] - r[0]) * 1e3 for r in recs])) if recs else 0.0
            out[f"{name}_max_gpu_ms"] = float(np.max([r[2] for r in recs])) if recs else 0.0
            out[f"{name}_max_wall_ms"] = float(np.max([(r[1] - r[0]) * 1e3 for r in recs])) if recs else 0.0
        allrec = self.phase_records[nx.PHASE_PREFILL] + self.phase_records[nx.PHASE_DECODE]
        if allrec:
            # the GPU is busy from the first launch to the last completion, minus the stretches with nothing in flight
            spans = sorted((r[0], r[1]) for r in allrec)
            busy_s, cur0, cur1 = 0.0, spans[0][0], spans[0][1]
            for a, b in spans[1:]:
                if a > cur1:
                    busy_s += cur1 - cur0
                    cur0, cur1 = a, b
                else:
                    cur1 = max(cur1, b)
            busy_s += cur1 - cur0
            tokens = sum(r[3] for r in allrec)
            out.update({"tokens": tokens, "gpu_seconds": busy_s, "tokens_per_s": tokens / busy_s})
        return out

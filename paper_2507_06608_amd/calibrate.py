"""Calibration of the partition cost model from this machine's own measurements (Sec. 4.1.1: the saturation share
and the decay coefficient of every operator are extracted from runs at varying compute shares).

Orchestration only: the steps run in the library, the kernel times come from its tracer, the curve fit and the
model arithmetic are library calls.  Each phase runs alone on 4, 8, ..., 28 of 32 steps of the chip (one step = one
CU in each XCD) and on all of it; traced kernel durations are grouped into the five modelled operators (QKV +
rotary, attention + merge, O, gate/up, down; each norm with the GEMM it feeds) and scaled so that they add up to
the phase as it runs untraced (the gaps between dependent launches belong to the phase but to no kernel).
"""
from __future__ import annotations

import time
from dataclasses import dataclass
from typing import List, Sequence, Tuple

from . import binding as nx

PEAK_FLOPS, PEAK_BW = 2.5e15, 8.0e12
TOTAL_SHARES = 32

PREFILL_OPS = (("gemm_qkv", "rope_append"), ("attn_prefill", "attn_merge"), ("gemm_o",), ("gemm_gate_up",), ("gemm_down", "splitk_reduce"))
DECODE_OPS = (("gemm_qkv", "rope_append"), ("attn_decode", "attn_merge"), ("gemm_o",), ("gemm_gate_up",), ("gemm_down", "splitk_reduce"))


def operator_times(ctx, phase: int, run, groups, reps: int = 4) -> List[float]:
    """Seconds per step of each operator of `phase`, `run()` launching one step of that phase alone."""
    per_kernel = {}
    for k in {k for g in groups for k in g} | {"rmsnorm"}:
        ctx.trace_begin(phase, k)
        for _ in range(reps):
            run()
        ms, n = ctx.trace_read()
        per_kernel[k] = ms * 1e-3 * n / reps
    t = [sum(per_kernel[k] for k in g) for g in groups]
    t[0] += per_kernel["rmsnorm"] / 2
    t[3] += per_kernel["rmsnorm"] / 2
    ctx.sync()
    t0 = time.perf_counter()
    for _ in range(4 * reps):
        run()
    ctx.sync()
    phase_s = (time.perf_counter() - t0) / (4 * reps)
    scale = phase_s / sum(t)
    return [v * scale for v in t]


@dataclass
class Calibration:
    """Per operator and phase: effective work per algorithmic flop, saturation share, decay coefficient."""
    shares: List[int]
    prefill_times: List[List[float]]      # [share][operator] seconds
    decode_times: List[List[float]]
    prefill_fit: List[Tuple[float, float, float]]   # (effective flops / algorithmic flops, r_sat, lambda)
    decode_fit: List[Tuple[float, float, float]]

    def model(self, alg_prefill, alg_decode) -> "nx.CostModel":
        """The latency model of a batch from its algorithmic description (nx.cost_describe)."""
        def ops(alg, fit):
            return [(max(flops, 1.0) * k, nbytes, r_sat, lam, kind) for (flops, nbytes, _, _, kind), (k, r_sat, lam) in zip(alg, fit)]
        return nx.CostModel(PEAK_FLOPS, PEAK_BW, ops(alg_prefill, self.prefill_fit), ops(alg_decode, self.decode_fit))


def calibrate(ctx, kv, pb, db, alg_prefill, alg_decode, layers=(0, 1), shares: Sequence[int] = tuple(range(4, 32, 4)) + (32,)) -> Calibration:
    """Runs the two phases of (pb, db) alone at every share and fits every operator.  alg_*: nx.cost_describe of the
    same batch and layer count.  Leaves the context on the unpartitioned layout."""
    times = {nx.PHASE_PREFILL: [], nx.PHASE_DECODE: []}
    for s in shares:
        for phase, groups, run in ((nx.PHASE_PREFILL, PREFILL_OPS, lambda: ctx.prefill_chunk(pb, kv, layers=layers)),
                                   (nx.PHASE_DECODE, DECODE_OPS, lambda: ctx.decode_step(db, kv, layers=layers))):
            if s == TOTAL_SHARES:
                ctx.set_cu_split(nx.CUS_ALL, nx.CUS_ALL)
            elif phase == nx.PHASE_PREFILL:
                ctx.set_cu_split(8 * s, 256 - 8 * s)
            else:
                ctx.set_cu_split(256 - 8 * s, 8 * s)
            for _ in range(2):
                run()
            ctx.sync()
            times[phase].append(operator_times(ctx, phase, run, groups))
    rs = [s / TOTAL_SHARES for s in shares]

    def fit(alg, rows):
        out = []
        for i, (flops, _, _, _, _) in enumerate(alg):
            c, r_sat, lam = nx.cost_fit(rs, [row[i] for row in rows], PEAK_FLOPS)
            out.append((c / max(flops, 1.0), r_sat, lam))
        return out
    ctx.set_cu_split(nx.CUS_ALL, nx.CUS_ALL)
    return Calibration(list(shares), times[nx.PHASE_PREFILL], times[nx.PHASE_DECODE], fit(alg_prefill, times[nx.PHASE_PREFILL]),
                       fit(alg_decode, times[nx.PHASE_DECODE]))

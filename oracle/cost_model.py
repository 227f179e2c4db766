"""TEST INFRASTRUCTURE ONLY -- plain fp64 reference of the paper's partition controller.

What it follows, in the paper's order and notation:

* Sec. 4.1.1, Eq. 5-6: a phase's latency is the sum over its operators of max(compute time, memory time).
* Sec. 4.1.1, Eq. 7: compute time of an operator with c flops on a share r of the GPU is c / (r C) up to the
  operator's saturation share R_sat, and c / (R_sat C) * (1 + lambda (r - R_sat)) beyond it.
* Sec. 4.1.1, Eq. 8-9 and the unnumbered bandwidth formula between them: decode attention shares the memory
  bandwidth B with whatever prefill is doing.  P_attn = (time prefill spends in attention) / (prefill time);
  during that fraction decode gets the share m_d / (m_d + m_p1) of B, during the rest m_d / (m_d + m_p2).
* Sec. 4.1.2: the two constrained objectives and the switch between them on KV-cache usage.
* Alg. 1: the two-phase greedy adjustment and the buffer zone.

Nothing here is imported by the product; only tests/ and the GPU validation test call it.  Readings taken where
the paper leaves a choice are marked "reading" below.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Sequence, Tuple

PREFILL, DECODE = 0, 1
DENSE, ATTENTION = 0, 1


@dataclass
class Op:
    c: float        # flops
    m: float        # bytes moved
    r_sat: float    # saturation share, in (0, 1]
    lam: float      # decay coefficient beyond saturation
    kind: int       # DENSE or ATTENTION


@dataclass
class Model:
    C: float                # peak flop/s
    B: float                # peak bytes/s
    prefill: List[Op]
    decode: List[Op]


def compute_latency(c: float, r: float, C: float, r_sat: float, lam: float) -> float:
    """Eq. 7."""
    if r <= r_sat:
        return c / (r * C)
    return c / (r_sat * C) * (1.0 + lam * (r - r_sat))


def prefill_latency(model: Model, r_p: float) -> float:
    """Eq. 5; prefill memory time is taken at peak bandwidth (Sec. 4.1.1, last paragraph)."""
    return sum(max(compute_latency(o.c, r_p, model.C, o.r_sat, o.lam), o.m / model.B) for o in model.prefill)


def prefill_attention_time(model: Model, r_p: float) -> float:
    """reading: the time of the prefill attention operators as the model itself estimates it at share r_p."""
    return sum(max(compute_latency(o.c, r_p, model.C, o.r_sat, o.lam), o.m / model.B)
               for o in model.prefill if o.kind == ATTENTION)


def p_attn(model: Model, r_p: float) -> float:
    """Eq. 8."""
    return prefill_attention_time(model, r_p) / prefill_latency(model, r_p)


def decode_bandwidth(model: Model, r_p: float) -> float:
    """The bandwidth left to decode attention while prefill runs on the share r_p.  r_p = 0 means there is no
    prefill at all (decode by itself gets the whole bandwidth)."""
    if r_p <= 0.0:
        return model.B
    m_d = sum(o.m for o in model.decode if o.kind == ATTENTION)
    m_p1 = sum(o.m for o in model.prefill if o.kind == ATTENTION)
    m_p2 = sum(o.m for o in model.prefill if o.kind == DENSE)
    if m_d <= 0.0:
        return model.B
    pa = p_attn(model, r_p)
    return (m_d / (m_d + m_p1) * pa + m_d / (m_d + m_p2) * (1.0 - pa)) * model.B


def decode_latency(model: Model, r_d: float, r_p: float) -> float:
    """Eq. 6, with Eq. 9 for the attention operators (each gets its bytes over the contended bandwidth) and peak
    bandwidth for every other operator."""
    bd = decode_bandwidth(model, r_p)
    t = 0.0
    for o in model.decode:
        mem = o.m / (bd if o.kind == ATTENTION else model.B)
        t += max(compute_latency(o.c, r_d, model.C, o.r_sat, o.lam), mem)
    return t


def cost_model(model: Model, phase: int, share: int, total: int) -> float:
    """CostModel(phase, R) of Alg. 1 with shares counted in `total` equal steps (the paper uses total = 100).
    The other phase holds the remaining total - share steps.
    reading: Alg. 1 obtains the reference latency T^opt from this same function at R = 100, where the other phase
    would hold nothing and Eq. 8 has no value; the other phase then sits at its floor of one step (no partition
    gives it less), so T^opt of decode carries the same kind of contention term as the latencies it is compared
    with."""
    if phase == PREFILL:
        return prefill_latency(model, share / total)
    return decode_latency(model, share / total, max(total - share, 1) / total)


def adjust_partition(model: Model, target: int, r_p_cur: int, total: int, alpha: float, beta: float) -> Tuple[int, int]:
    """AdjustPartition of Alg. 1.  Returns (new prefill share, number of cost-model evaluations).
    reading: both phases keep at least one step, so the loops stop at 1 and at total - 1."""
    other = DECODE if target == PREFILL else PREFILL
    slack = beta if target == PREFILL else alpha
    evals = 1
    t_opt = cost_model(model, other, total, total)
    r = r_p_cur if target == PREFILL else total - r_p_cur
    r = min(max(r, 1), total - 1)
    # phase 1: give up share until the other phase meets its budget
    while r > 1:
        evals += 1
        if cost_model(model, other, total - r, total) <= slack * t_opt:
            break
        r -= 1
    # phase 2: take share back while it still does
    while r < total - 1:
        evals += 1
        if cost_model(model, other, total - (r + 1), total) > slack * t_opt:
            break
        r += 1
    return (r if target == PREFILL else total - r), evals


def partition_controller(model: Model, kv_u: float, kv_switch: float, r_p_cur: int, total: int, alpha: float,
                         beta: float, delta: int) -> int:
    """PartitionController of Alg. 1: decode-prioritised above the KV-usage switch point, prefill-prioritised at or
    below it; changes smaller than delta steps are suppressed."""
    target = DECODE if kv_u > kv_switch else PREFILL
    r_new, _ = adjust_partition(model, target, r_p_cur, total, alpha, beta)
    return r_p_cur if abs(r_new - r_p_cur) < delta else r_new


def brute_force(model: Model, target: int, total: int, alpha: float, beta: float) -> int:
    """The constrained optimum of Sec. 4.1.2 by exhaustive scan over 1 .. total - 1: the prefill share minimising
    the target's latency among those that keep the other phase within its budget; when none does, the share
    that gives the other phase the most (what the greedy's first loop ends at)."""
    best, best_t = None, None
    for r_p in range(1, total):
        t_p = cost_model(model, PREFILL, r_p, total)
        t_d = cost_model(model, DECODE, total - r_p, total)
        if target == PREFILL:
            ok, t = t_d <= beta * cost_model(model, DECODE, total, total), t_p
        else:
            ok, t = t_p <= alpha * cost_model(model, PREFILL, total, total), t_d
        if ok and (best is None or t < best_t):
            best, best_t = r_p, t
    if best is None:
        return 1 if target == PREFILL else total - 1
    return best


def fit_op(rs: Sequence[float], ts: Sequence[float], C: float) -> Tuple[float, float, float]:
    """reading (the paper only says the two parameters are extracted from measurements at varying shares): least
    squares in relative error over the candidate saturation points.  For a candidate R_sat taken from the measured
    shares, the effective work c is the mean of t r C over the points at or below it, lambda the least-squares
    slope of t / t_sat - 1 against r - R_sat over the points above it (0 when there are none).  Returns
    (c, R_sat, lambda) of the candidate with the smallest sum of squared relative errors; ties to the larger
    R_sat."""
    pts = sorted(zip(rs, ts))
    best = None
    for k in range(len(pts)):
        r_sat = pts[k][0]
        below = [(r, t) for r, t in pts if r <= r_sat]
        above = [(r, t) for r, t in pts if r > r_sat]
        c = sum(t * r * C for r, t in below) / len(below)
        t_sat = c / (r_sat * C)
        lam = 0.0
        if above:
            num = sum((t / t_sat - 1.0) * (r - r_sat) for r, t in above)
            den = sum((r - r_sat) ** 2 for r, t in above)
            lam = num / den
        err = sum(((compute_latency(c, r, C, r_sat, lam) - t) / t) ** 2 for r, t in pts)
        if best is None or err <= best[0]:
            best = (err, c, r_sat, lam)
    return best[1], best[2], best[3]

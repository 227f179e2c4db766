"""Plausible mistakes planted in a copy of the cost-model oracle: every one of them must make a pin fail."""
import importlib
import os
import types

import pytest

import tests.test_cost_model_pins as pins

SRC = os.path.join(os.path.dirname(os.path.dirname(__file__)), "oracle", "cost_model.py")

MUTATIONS = [
    ("decay term dropped beyond saturation", "c / (r_sat * C) * (1.0 + lam * (r - r_sat))", "c / (r_sat * C)"),
    ("saturated branch divides by r instead of R_sat", "c / (r_sat * C) * (1.0", "c / (r * C) * (1.0"),
    ("prefill latency adds compute and memory instead of taking the larger",
     "return sum(max(compute_latency(o.c, r_p, model.C, o.r_sat, o.lam), o.m / model.B) for o in model.prefill)",
     "return sum(compute_latency(o.c, r_p, model.C, o.r_sat, o.lam) + o.m / model.B for o in model.prefill)"),
    ("P_attn inverted", "return prefill_attention_time(model, r_p) / prefill_latency(model, r_p)",
     "return 1.0 - prefill_attention_time(model, r_p) / prefill_latency(model, r_p)"),
    ("attention and dense prefill traffic swapped",
     "m_p1 = sum(o.m for o in model.prefill if o.kind == ATTENTION)", "m_p1 = sum(o.m for o in model.prefill if o.kind == DENSE)"),
    ("decode attention ignores the contended bandwidth", "mem = o.m / (bd if o.kind == ATTENTION else model.B)", "mem = o.m / model.B"),
    ("every decode operator contended", "mem = o.m / (bd if o.kind == ATTENTION else model.B)", "mem = o.m / bd"),
    ("slack of the wrong phase", "slack = beta if target == PREFILL else alpha", "slack = alpha if target == PREFILL else beta"),
    ("ideal latency of the other phase taken under contention", "t_opt = cost_model(model, other, total, total)",
     "t_opt = cost_model(model, other, total - 1, total)"),
    ("second loop tests the current share, not the next", "cost_model(model, other, total - (r + 1), total) > slack * t_opt",
     "cost_model(model, other, total - r, total) > slack * t_opt"),
    ("buffer zone includes delta itself", "abs(r_new - r_p_cur) < delta", "abs(r_new - r_p_cur) <= delta"),
    ("mode switch at the threshold goes the wrong way", "DECODE if kv_u > kv_switch else PREFILL", "DECODE if kv_u >= kv_switch else PREFILL"),
    ("decode share mistaken for the prefill share", "return decode_latency(model, share / total, max(total - share, 1) / total)",
     "return decode_latency(model, max(total - share, 1) / total, share / total)"),
    ("reference latency of decode taken without any contention", "return decode_latency(model, share / total, max(total - share, 1) / total)",
     "return decode_latency(model, share / total, (total - share) / total)"),
]


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_pins_catch(name, old, new, monkeypatch):
    src = open(SRC).read()
    assert src.count(old) == 1, f"mutation site not found exactly once: {old}"
    mod = types.ModuleType("cost_model_mutant")
    mod.__dict__["__name__"] = "cost_model_mutant"
    import sys
    sys.modules["cost_model_mutant"] = mod  # dataclasses look the module up by name
    try:
        exec(compile(src.replace(old, new), SRC, "exec"), mod.__dict__)
        monkeypatch.setattr(pins, "cm", mod)
        failed = False
        for fn in (pins.test_worked_example_by_hand, pins.test_compute_curve_closed_forms,
                   pins.test_phase_latency_is_sum_of_roofline_maxima, pins.test_contention_limits,
                   pins.test_greedy_equals_exhaustive_search_when_latency_is_monotone,
                   pins.test_controller_switch_and_buffer_zone, pins.test_fit_recovers_known_parameters):
            try:
                fn()
            except Exception:
                failed = True
                break
        assert failed, f"no pin noticed: {name}"
    finally:
        sys.modules.pop("cost_model_mutant", None)

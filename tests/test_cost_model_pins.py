"""Pins of the cost-model oracle (oracle/cost_model.py) against things it does not define itself: a worked example
computed by hand (tests/golden/cost_model_worked_example.txt), closed forms and limits of Eq. 5-9, exhaustive search
for Alg. 1, and synthetic curves with known parameters for the fit."""
import math
import os
import random

import pytest

from oracle import cost_model as cm

GOLD = os.path.join(os.path.dirname(__file__), "golden", "cost_model_worked_example.txt")


def worked_model():
    return cm.Model(C=20.0, B=10.0,
                    prefill=[cm.Op(40, 20, 0.5, -0.2, cm.DENSE), cm.Op(10, 30, 1.0, 0.0, cm.ATTENTION)],
                    decode=[cm.Op(4, 10, 0.25, 0.0, cm.DENSE), cm.Op(2, 20, 0.5, 0.0, cm.ATTENTION)])


def gold():
    out = {}
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        k, v = line.split()
        out[k] = float(v)
    return out


def test_worked_example_by_hand():
    g, m = gold(), worked_model()
    for name, r in (("1/4", 0.25), ("1/2", 0.5), ("3/4", 0.75), ("1", 1.0)):
        assert cm.prefill_latency(m, r) == pytest.approx(g["prefill_latency_r" + name], rel=1e-12)
    for name, r in (("3/4", 0.75), ("1/2", 0.5), ("1/4", 0.25)):
        assert cm.p_attn(m, r) == pytest.approx(g["p_attn_r" + name], rel=1e-12)
        assert cm.decode_bandwidth(m, r) == pytest.approx(g["decode_bandwidth_rp" + name], rel=1e-12)
        assert cm.decode_latency(m, 1.0 - r, r) == pytest.approx(g["decode_latency_rp" + name], rel=1e-12)
    assert cm.decode_latency(m, 1.0, 0.0) == pytest.approx(g["decode_latency_alone"], rel=1e-12)
    # CostModel(phase, R) of Alg. 1 on 4 steps is the same thing
    assert cm.cost_model(m, cm.DECODE, 2, 4) == pytest.approx(g["decode_latency_rp1/2"], rel=1e-12)
    assert cm.cost_model(m, cm.DECODE, 4, 4) == pytest.approx(g["decode_latency_reference"], rel=1e-12)
    assert cm.cost_model(m, cm.PREFILL, 3, 4) == pytest.approx(6.8, rel=1e-12)
    for beta, key in ((1.02, "greedy_prefill_beta1.02"), (1.029, "greedy_prefill_beta1.029"), (1.03, "greedy_prefill_beta1.03")):
        assert cm.adjust_partition(m, cm.PREFILL, 2, 4, 1.3, beta)[0] == int(g[key])
    for alpha, key in ((1.05, "greedy_decode_alpha1.05"), (1.1, "greedy_decode_alpha1.1"), (2.0, "greedy_decode_alpha2")):
        assert cm.adjust_partition(m, cm.DECODE, 2, 4, alpha, 1.1)[0] == int(g[key])


def test_compute_curve_closed_forms():
    C = 3.0e12
    for c, r_sat, lam in ((1e9, 0.4, -0.3), (5e10, 1.0, 0.0), (2e8, 0.1, 0.05)):
        # inverse scaling below saturation: t * r is constant and equals c / C
        for r in (0.01, r_sat / 3, r_sat):
            assert cm.compute_latency(c, r, C, r_sat, lam) * r == pytest.approx(c / C, rel=1e-13)
        # continuous at the saturation point, linear beyond it with slope lambda * t_sat
        t_sat = c / (r_sat * C)
        eps = 1e-9
        assert cm.compute_latency(c, r_sat + eps, C, r_sat, lam) == pytest.approx(t_sat, rel=1e-6)
        if r_sat < 1.0:
            r1, r2 = r_sat + 0.1 * (1 - r_sat), 1.0
            slope = (cm.compute_latency(c, r2, C, r_sat, lam) - cm.compute_latency(c, r1, C, r_sat, lam)) / (r2 - r1)
            assert slope == pytest.approx(lam * t_sat, rel=1e-9)
    # lambda = 0: flat beyond saturation (the "saturates early" curve of Sec. 3.2)
    assert cm.compute_latency(1.0, 0.9, 1.0, 0.5, 0.0) == cm.compute_latency(1.0, 0.5, 1.0, 0.5, 0.0) == 2.0


def test_phase_latency_is_sum_of_roofline_maxima():
    # one compute-bound and one memory-bound operator: Eq. 5 must take the larger term of each, not of the sums
    m = cm.Model(C=10.0, B=10.0, prefill=[cm.Op(100, 1, 1.0, 0.0, cm.DENSE), cm.Op(1, 100, 1.0, 0.0, cm.DENSE)], decode=[])
    assert cm.prefill_latency(m, 1.0) == pytest.approx(10.0 + 10.0)
    assert cm.prefill_latency(m, 0.5) == pytest.approx(20.0 + 10.0)  # only the compute-bound one scales


def test_contention_limits():
    m = worked_model()
    # no prefill memory traffic -> decode keeps the whole bandwidth whatever the overlap
    quiet = cm.Model(m.C, m.B, [cm.Op(40, 0, 0.5, -0.2, cm.DENSE), cm.Op(10, 0, 1.0, 0.0, cm.ATTENTION)], m.decode)
    assert cm.decode_bandwidth(quiet, 0.5) == pytest.approx(m.B)
    # no prefill at all
    assert cm.decode_bandwidth(m, 0.0) == m.B
    # P_attn is a probability and the effective bandwidth lies between the two pure cases
    for r in (0.1, 0.5, 0.9):
        pa = cm.p_attn(m, r)
        assert 0.0 <= pa <= 1.0
        lo, hi = sorted((20 / 50 * m.B, 20 / 40 * m.B))
        assert lo - 1e-12 <= cm.decode_bandwidth(m, r) <= hi + 1e-12
    # more prefill KV traffic (the paper's Sec. 3.3 experiment) -> slower decode at a fixed partition
    heavy = cm.Model(m.C, m.B, [m.prefill[0], cm.Op(10, 150, 1.0, 0.0, cm.ATTENTION)], m.decode)
    assert cm.decode_latency(heavy, 0.5, 0.5) > cm.decode_latency(m, 0.5, 0.5)
    # decode operators other than attention never see the contention
    only_dense = cm.Model(m.C, m.B, m.prefill, [cm.Op(4, 10, 0.25, 0.0, cm.DENSE)])
    assert cm.decode_latency(only_dense, 0.5, 0.5) == pytest.approx(cm.decode_latency(only_dense, 0.5, 0.0))


def random_model(rng):
    def ops(n_dense, scale):
        o = [cm.Op(rng.uniform(0.1, 10) * scale, rng.uniform(0.1, 10), rng.uniform(0.2, 1.0), rng.uniform(-0.3, 0.0), cm.DENSE)
             for _ in range(n_dense)]
        o.append(cm.Op(rng.uniform(0.1, 10) * scale, rng.uniform(0.1, 30), rng.uniform(0.2, 1.0), rng.uniform(-0.3, 0.0), cm.ATTENTION))
        return o
    return cm.Model(C=rng.uniform(5, 50), B=rng.uniform(5, 50), prefill=ops(4, 10.0), decode=ops(4, 0.3))


def test_greedy_equals_exhaustive_search_when_latency_is_monotone():
    rng = random.Random(7)
    total, checked = 32, 0
    for _ in range(300):
        m = random_model(rng)
        alpha, beta = rng.uniform(1.02, 3.0), rng.uniform(1.02, 3.0)
        tp = [cm.cost_model(m, cm.PREFILL, r, total) for r in range(1, total)]
        td = [cm.cost_model(m, cm.DECODE, r, total) for r in range(1, total)]
        if any(b > a for a, b in zip(tp, tp[1:])) or any(b > a for a, b in zip(td, td[1:])):
            continue  # the greedy presumes that more share never hurts; skip the rare model where contention inverts it
        checked += 1
        for target in (cm.PREFILL, cm.DECODE):
            want = cm.brute_force(m, target, total, alpha, beta)
            for start in (1, 7, 16, 31):
                got, evals = cm.adjust_partition(m, target, start, total, alpha, beta)
                assert got == want, (target, start)
                assert evals <= 2 + 2 * total
    assert checked > 150


def test_controller_switch_and_buffer_zone():
    m = worked_model()
    # KV usage at or below the switch point -> prefill-prioritised, above -> decode-prioritised
    assert cm.partition_controller(m, 0.3, 0.5, 2, 4, 1.1, 1.8, 1) == cm.adjust_partition(m, cm.PREFILL, 2, 4, 1.1, 1.8)[0] == 3
    assert cm.partition_controller(m, 0.5, 0.5, 2, 4, 1.1, 1.8, 1) == 3
    assert cm.partition_controller(m, 0.7, 0.5, 3, 4, 2.0, 1.8, 1) == cm.adjust_partition(m, cm.DECODE, 3, 4, 2.0, 1.8)[0] == 1
    # a change smaller than delta is suppressed, one of exactly delta goes through
    assert cm.partition_controller(m, 0.3, 0.5, 2, 4, 1.1, 1.8, 2) == 2
    assert cm.partition_controller(m, 0.7, 0.5, 3, 4, 2.0, 1.8, 2) == 1
    assert cm.partition_controller(m, 0.7, 0.5, 3, 4, 2.0, 1.8, 3) == 3


def test_fit_recovers_known_parameters():
    C = 1.0e3
    rs = [i / 16 for i in range(1, 17)]
    for c, r_sat, lam in ((50.0, 0.5, -0.25), (7.0, 0.25, 0.0), (300.0, 1.0, 0.0), (20.0, 0.75, -0.4)):
        ts = [cm.compute_latency(c, r, C, r_sat, lam) for r in rs]
        c_f, r_f, l_f = cm.fit_op(rs, ts, C)
        assert c_f == pytest.approx(c, rel=1e-9)
        assert r_f == pytest.approx(r_sat)
        assert l_f == pytest.approx(lam, abs=1e-9)
    # with 2% multiplicative noise the parameters move by a few percent only
    rng = random.Random(3)
    ts = [cm.compute_latency(50.0, r, C, 0.5, -0.25) * (1 + rng.uniform(-0.02, 0.02)) for r in rs]
    c_f, r_f, l_f = cm.fit_op(rs, ts, C)
    assert c_f == pytest.approx(50.0, rel=0.05) and abs(r_f - 0.5) <= 1 / 16 + 1e-12 and l_f == pytest.approx(-0.25, abs=0.1)

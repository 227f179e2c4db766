"""The library's partition controller (host-only entry points of the C ABI) against the cost-model oracle, on random
models and on the worked example.  No GPU is needed: the functions touch host memory only."""
import random

import pytest

from oracle import cost_model as cm
from paper_2507_06608_amd import binding as nx
from paper_2507_06608_amd import synth
from tests.test_cost_model_pins import gold, random_model, worked_model


def to_lib(m: cm.Model) -> nx.CostModel:
    conv = lambda ops: [(o.c, o.m, o.r_sat, o.lam, o.kind) for o in ops]
    return nx.CostModel(m.C, m.B, conv(m.prefill), conv(m.decode))


def test_latency_matches_oracle_and_worked_example():
    g, m = gold(), worked_model()
    lm = to_lib(m)
    assert lm.latency(nx.PHASE_PREFILL, 3, 4) == pytest.approx(g["prefill_latency_r3/4"], rel=1e-12)
    assert lm.latency(nx.PHASE_DECODE, 2, 4) == pytest.approx(g["decode_latency_rp1/2"], rel=1e-12)
    assert lm.latency(nx.PHASE_DECODE, 4, 4) == pytest.approx(g["decode_latency_reference"], rel=1e-12)
    rng = random.Random(11)
    for _ in range(100):
        m = random_model(rng)
        lm = to_lib(m)
        total = rng.choice((4, 32, 100))
        for share in {1, total // 2, total - 1, total}:
            for phase in (cm.PREFILL, cm.DECODE):
                assert lm.latency(phase, share, total) == pytest.approx(cm.cost_model(m, phase, share, total), rel=1e-12)


def test_greedy_and_controller_match_oracle():
    g, m = gold(), worked_model()
    lm = to_lib(m)
    for beta, key in ((1.02, "greedy_prefill_beta1.02"), (1.029, "greedy_prefill_beta1.029"), (1.03, "greedy_prefill_beta1.03")):
        assert lm.adjust_partition(nx.PHASE_PREFILL, 2, 4, 1.3, beta)[0] == int(g[key])
    for alpha, key in ((1.05, "greedy_decode_alpha1.05"), (1.1, "greedy_decode_alpha1.1"), (2.0, "greedy_decode_alpha2")):
        assert lm.adjust_partition(nx.PHASE_DECODE, 2, 4, alpha, 1.1)[0] == int(g[key])
    rng = random.Random(5)
    for _ in range(200):
        m = random_model(rng)
        lm = to_lib(m)
        total = rng.choice((8, 32, 100))
        alpha, beta = rng.uniform(1.0, 3.0), rng.uniform(1.0, 3.0)
        cur = rng.randrange(0, total + 1)
        for target in (cm.PREFILL, cm.DECODE):
            want, evals = cm.adjust_partition(m, target, cur, total, alpha, beta)
            got, n = lm.adjust_partition(target, cur, total, alpha, beta)
            assert (got, n) == (want, evals)
        kv_u, kv_s, delta = rng.random(), rng.random(), rng.randrange(0, 6)
        cur = rng.randrange(1, total)
        assert lm.partition_controller(kv_u, kv_s, cur, total, alpha, beta, delta) == \
            cm.partition_controller(m, kv_u, kv_s, cur, total, alpha, beta, delta)


def test_fit_matches_oracle():
    rng = random.Random(9)
    for _ in range(50):
        C = rng.uniform(1e2, 1e4)
        n = rng.randrange(1, 12)
        rs = sorted(rng.sample([i / 32 for i in range(1, 33)], n))
        c, r_sat, lam = rng.uniform(1, 100), rng.choice(rs), rng.uniform(-0.5, 0.1)
        ts = [cm.compute_latency(c, r, C, r_sat, lam) * (1 + rng.uniform(-0.03, 0.03)) for r in rs]
        want = cm.fit_op(rs, ts, C)
        got = nx.cost_fit(rs, ts, C)
        assert got[1] == pytest.approx(want[1])
        assert got[0] == pytest.approx(want[0], rel=1e-10) and got[2] == pytest.approx(want[2], rel=1e-8, abs=1e-12)


def test_describe_counts_the_layer():
    s = synth.SHAPES["llama3_8b"]
    p, d = nx.cost_describe(s, 1, 512, 917760, 2048, 64, 148666 + 64)
    # the totals the survey gives for this workload: 223.3 GFLOP of projections + 15.0 of attention; 436 MB of weights
    assert sum(o[0] for i, o in enumerate(p) if i != 1) == pytest.approx(2.0 * 512 * s.params_per_layer, rel=1e-12)
    assert p[1][0] == pytest.approx(4.0 * 128 * 32 * 917760) and p[1][0] / 1e9 == pytest.approx(15.0, abs=0.1)
    assert sum(o[1] for i, o in enumerate(d) if i != 1) == pytest.approx(2.0 * s.params_per_layer)
    assert d[1][1] == pytest.approx((148666 + 64) * 4096.0) and p[1][1] == pytest.approx(2048 * 4096.0)
    assert [o[4] for o in p] == [0, 1, 0, 0, 0] and all(o[2] == 1.0 and o[3] == 0.0 for o in p + d)
    p2, _ = nx.cost_describe(s, 3, 512, 917760, 2048, 64, 1000)
    assert p2[3][0] == pytest.approx(3 * p[3][0])


def test_argument_errors():
    lm = to_lib(worked_model())
    for bad in ((nx.PHASE_PREFILL, 0, 4), (nx.PHASE_PREFILL, 5, 4), (7, 1, 4)):
        with pytest.raises(nx.NexusError):
            lm.latency(*bad)
    with pytest.raises(nx.NexusError):
        lm.adjust_partition(nx.PHASE_PREFILL, 2, 1, 1.3, 1.1)
    with pytest.raises(nx.NexusError):
        lm.adjust_partition(nx.PHASE_PREFILL, 2, 4, 0.9, 1.1)
    with pytest.raises(nx.NexusError):
        nx.CostModel(1.0, 1.0, [(1.0, 1.0, 0.0, 0.0, 0)], []).latency(nx.PHASE_PREFILL, 1, 2)
    with pytest.raises(nx.NexusError):
        nx.cost_fit([0.5, 1.5], [1.0, 1.0], 1.0)

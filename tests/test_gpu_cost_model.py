"""Validation of the partition cost model (Sec. 4.1) against measurements on the GPU: the per-operator saturation
curves are extracted from traced kernel times of each phase alone on varying CU shares (as the paper prescribes),
and the calibrated model's predictions are compared with the measured concurrent step and the measured choice."""
import numpy as np
import pytest
import torch

from oracle import cost_model as cm
from paper_2507_06608_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def nx():
    from paper_2507_06608_amd import binding
    binding.lib()          # fails loudly if the library was not built
    assert torch.cuda.is_available()
    return binding

PEAK_FLOPS, PEAK_BW = 2.5e15, 8.0e12
TOTAL = 32  # one step = one CU in each of the 8 XCDs


def test_calibrated_model_against_measured_splits(nx):
    print("[gpu test] cost model calibration and validation", flush=True)
    wl = synth.config(2, seed=0, kv_device="cuda:0")
    w = synth.make_weights(wl.shape, 0)
    ctx = nx.context_for(wl)
    ctx.load_layer(0, w)
    kv = ctx.make_kv(wl.k_pool, wl.v_pool)
    pb, db = nx.DevPrefill(wl.prefill, ctx.device), nx.DevDecode(wl.decode, ctx.device)
    p, d = wl.prefill, wl.decode
    pairs = float(sum(int(n) * int(pre) + int(n) * (int(n) + 1) // 2 for n, pre in zip(p.chunk_len, p.prefix_len)))
    kv_p = float((p.prefix_len + p.chunk_len).sum())
    kv_d = float((d.ctx_len + 1).sum())
    alg_p, alg_d = nx.cost_describe(wl.shape, 1, p.n_tokens, pairs, kv_p, d.n_reqs, kv_d)

    from paper_2507_06608_amd.calibrate import calibrate
    cal = calibrate(ctx, kv, pb, db, alg_p, alg_d)
    ops_p = [(f * k, m, r, l, kind) for (f, m, _, _, kind), (k, r, l) in zip(alg_p, cal.prefill_fit)]
    ops_d = [(f * k, m, r, l, kind) for (f, m, _, _, kind), (k, r, l) in zip(alg_d, cal.decode_fit)]
    for name, ops in (("prefill", ops_p), ("decode", ops_d)):
        print(f"[cost model] {name} operators (effective GFLOP, R_sat, lambda): " +
              ", ".join(f"({o[0] / 1e9:.1f}, {o[2]:.3f}, {o[3]:+.2f})" for o in ops), flush=True)
    model = nx.CostModel(PEAK_FLOPS, PEAK_BW, ops_p, ops_d)
    oracle_model = cm.Model(PEAK_FLOPS, PEAK_BW, [cm.Op(*o) for o in ops_p], [cm.Op(*o) for o in ops_d])

    cands = list(range(32, 256, 32))
    prof = ctx.profile_split(pb, db, kv, cands, nx.POLICY_MIN_STEP, repeats=5)

    # (a) Eq. 5-6 with the calibrated curves against each phase timed alone, untraced, on its share (the
    # contention term is off for a phase on its own: the other phase has no operators)
    alone_p = nx.CostModel(PEAK_FLOPS, PEAK_BW, ops_p, [])
    alone_d = nx.CostModel(PEAK_FLOPS, PEAK_BW, [], ops_d)
    mp = [alone_p.latency(nx.PHASE_PREFILL, c // 8, TOTAL) * 1e3 for c in cands]
    md = [alone_d.latency(nx.PHASE_DECODE, TOTAL - c // 8, TOTAL) * 1e3 for c in cands]
    print("[cost model] prefill CUs:            " + " ".join(f"{c:7d}" for c in cands))
    print("[cost model] prefill alone, model ms:" + " ".join(f"{t:7.3f}" for t in mp))
    print("[cost model] prefill alone, timed ms:" + " ".join(f"{t:7.3f}" for t in prof["t_prefill_ms"]))
    print("[cost model] decode alone, model ms: " + " ".join(f"{t:7.3f}" for t in md))
    print("[cost model] decode alone, timed ms: " + " ".join(f"{t:7.3f}" for t in prof["t_decode_ms"]), flush=True)
    for c, a, b in zip(cands, mp, prof["t_prefill_ms"]):
        assert a == pytest.approx(b, rel=0.2), ("prefill alone", c)
    for c, a, b in zip(cands, md, prof["t_decode_ms"]):
        assert a == pytest.approx(b, rel=0.2), ("decode alone", c)

    # (b) concurrent step: prediction max(T_prefill(R_p), T_decode(1 - R_p | R_p)) against the measured step
    pred = []
    for c in cands:
        s = c // 8
        tp, td = model.latency(nx.PHASE_PREFILL, s, TOTAL), model.latency(nx.PHASE_DECODE, TOTAL - s, TOTAL)
        assert tp == pytest.approx(cm.cost_model(oracle_model, cm.PREFILL, s, TOTAL), rel=1e-12)
        assert td == pytest.approx(cm.cost_model(oracle_model, cm.DECODE, TOTAL - s, TOTAL), rel=1e-12)
        pred.append(max(tp, td) * 1e3)
    print("[cost model] prefill CUs:        " + " ".join(f"{c:7d}" for c in cands))
    print("[cost model] predicted step ms:  " + " ".join(f"{t:7.3f}" for t in pred))
    print("[cost model] measured step ms:   " + " ".join(f"{t:7.3f}" for t in prof["t_step_ms"]), flush=True)
    for c, a, b in zip(cands, pred, prof["t_step_ms"]):
        assert a == pytest.approx(b, rel=0.25), ("concurrent step", c)
    assert abs(int(np.argmin(pred)) - int(np.argmin(prof["t_step_ms"]))) <= 1

    # (c) the greedy search on the model against the same objectives applied to the measured curves
    for target, policy in ((nx.PHASE_PREFILL, nx.POLICY_PREFILL_PRIORITIZED), (nx.PHASE_DECODE, nx.POLICY_DECODE_PRIORITIZED)):
        share, evals = model.adjust_partition(target, TOTAL // 2, TOTAL, 1.3, 1.1)
        i = nx.choose_split(prof["t_prefill_ms"], prof["t_decode_ms"], prof["t_step_ms"], prof["t_prefill_all_ms"],
                            prof["t_decode_all_ms"], policy, 1.3, 1.1)
        print(f"[cost model] target {'prefill' if target == nx.PHASE_PREFILL else 'decode'}: model picks {8 * share} prefill CUs "
              f"in {evals} evaluations, measured curves pick {cands[i]}", flush=True)
        # the budget cuts a nearly flat stretch of the curve, so a model error of 10 % moves the pick by two
        # candidates (the candidates are 32 CUs apart, the model searches in steps of 8)
        assert abs(8 * share - cands[i]) <= 64

    # (d) Eq. 9: at a fixed partition and with the prefill operators' times unchanged (so P_attn of Eq. 8 stays put),
    # more bytes moved by the prefill attention can only slow the modelled decode.  (With the attention's time growing
    # along, P_attn grows too, and while the prefill attention moves fewer bytes than the prefill GEMMs -- 41 MB
    # against 436 MB here -- Eq. 8-9 then hand decode MORE bandwidth: that is the model, not a monotone law.)
    def with_prefix(kv_tokens):
        a_p, a_d = nx.cost_describe(wl.shape, 1, p.n_tokens, p.n_tokens * kv_tokens, kv_tokens, d.n_reqs, kv_d)
        op = [(ops_p[i][0], a_p[i][1], ops_p[i][2], ops_p[i][3], ops_p[i][4]) for i in range(5)]
        return nx.CostModel(PEAK_FLOPS, PEAK_BW, op, ops_d).latency(nx.PHASE_DECODE, 16, TOTAL)
    assert with_prefix(10000) >= with_prefix(2000)
    ctx.close()

"""Pins of the scheduler oracle (Sec. 4.3, Eq. 10, Alg. 2): a hand-computed example, limiting cases that reduce to
textbook policies, a brute-force optimality check, starvation behaviour and conservation invariants."""
import itertools
import os
import random

from oracle import scheduler as sch

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "scheduler_worked_example.txt")


def _golden():
    out = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        key, *vals = line.split()
        out.setdefault(key, []).append(vals)
    return out


def _pairs(vals):
    return [tuple(int(x) for x in v.split(":")) for v in vals]


def test_worked_example_ordering_and_filling():
    g = _golden()
    reqs = []
    for rid, arrival, prompt, prefilled in g["A.request"]:
        reqs.append(sch.Request(int(rid), float(arrival), int(prompt), 1, prefilled=int(prefilled)))
    now, gamma, budget = 10.0, 15.0, 1000
    scores = [sch.spf_score(r.remaining, now - r.arrival, gamma) for r in reqs]
    assert scores == [float(x) for x in g["A.spf_scores"][0]]
    spf = sch.order_queue(reqs, now, sch.SPF, gamma)
    assert [r.rid for r in spf] == [int(x) for x in g["A.spf_order"][0]]
    as_pairs = lambda batch: [(r.rid, n) for r, n in batch]
    assert as_pairs(sch.fill_batch(spf, budget, chunk_tail=False)) == _pairs(g["A.spf_batch_printed"][0])
    assert as_pairs(sch.fill_batch(spf, budget, chunk_tail=True)) == _pairs(g["A.spf_batch_tail"][0])
    fcfs = sch.order_queue(reqs, now, sch.FCFS, gamma)
    assert as_pairs(sch.fill_batch(fcfs, budget, chunk_tail=False)) == _pairs(g["A.fcfs_batch_printed"][0])
    assert as_pairs(sch.fill_batch(fcfs, budget, chunk_tail=True)) == _pairs(g["A.fcfs_batch_tail"][0])


def test_worked_example_loop_timeline():
    g = _golden()
    loop = sch.Loop(sch.FCFS, budget=100, max_decode=2, page_size=16, n_pages=64)
    loop.submit(0.0, 150, 3)
    loop.submit(0.5, 60, 2)
    its = sch.run_virtual(loop, 4, 1.0)
    for i, it in enumerate(its):
        assert it.prefill == _pairs(g["B.prefill"][i][1:]), i
        assert it.decode == _pairs(g["B.decode"][i][1:]), i
    assert [it.kv_used_pages for it in its] == [int(x) for x in g["B.kv_used"][0]]
    assert loop.ttft() == [float(x) for x in g["B.ttft"][0]]
    assert sorted(loop.tbt()) == [float(x) for x in g["B.tbt"][0]]
    assert loop.normalized_latency() == [float(x) for x in g["B.normalized_latency"][0]]
    assert len(loop.free) == 64 and loop.reserved_total == 0


def test_worked_example_independent_phase_ticks():
    import pytest
    g = _golden()
    loop = sch.Loop(sch.FCFS, budget=100, max_decode=2, page_size=16, n_pages=64)
    loop.submit(0.0, 150, 4)
    loop.submit(0.0, 40, 2)
    loop.submit(0.5, 250, 1)
    used = []
    for t, op, *expect in g["C.step"]:
        got = getattr(loop, op)(float(t))
        if op.startswith("next"):
            assert got == _pairs(expect), (t, op)
        used.append(loop.kv_used_pages)
    assert used == [int(x) for x in g["C.kv_used"][0]]
    assert loop.ttft() == pytest.approx([float(x) for x in g["C.ttft"][0]], abs=1e-12)
    assert loop.tbt() == pytest.approx([float(x) for x in g["C.tbt"][0]], abs=1e-12)
    assert loop.normalized_latency() == pytest.approx([float(x) for x in g["C.normalized_latency"][0]], abs=1e-12)
    assert len(loop.free) == 64 and loop.reserved_total == 0


def test_limits_of_gamma_are_shortest_first_and_arrival_order():
    rng = random.Random(1)
    reqs = [sch.Request(i, rng.uniform(0, 50), rng.randint(1, 5000), 1, prefilled=0) for i in range(40)]
    now = 60.0
    by_len = sorted(reqs, key=lambda r: (r.prompt_len, r.arrival, r.rid))
    assert [r.rid for r in sch.order_queue(reqs, now, sch.SPF, 0.0)] == [r.rid for r in by_len]
    by_arrival = sorted(reqs, key=lambda r: (r.arrival, r.rid))
    assert [r.rid for r in sch.order_queue(reqs, now, sch.SPF, 1e9)] == [r.rid for r in by_arrival]
    assert [r.rid for r in sch.order_queue(reqs, now, sch.FCFS, 15.0)] == [r.rid for r in by_arrival]
    # the score falls with age at the rate gamma, and only `remaining` counts once a request is partly prefilled
    assert sch.spf_score(100, 2.0, 15.0) - sch.spf_score(100, 3.0, 15.0) == 15.0
    partly = sch.Request(0, 0.0, 4000, 1, prefilled=3900)
    fresh = sch.Request(1, 0.0, 200, 1)
    assert [r.rid for r in sch.order_queue([fresh, partly], 0.0, sch.SPF, 15.0)] == [0, 1]


def _mean_ttft(order, prompts, budget):
    rank = {rid: i for i, rid in enumerate(order or [])}
    loop = sch.Loop(sch.SPF, budget, max_decode=1, page_size=16, n_pages=4096, gamma=0.0,
                    priority=(lambda q, now: sorted(q, key=lambda r: rank[r.rid])) if order is not None else None)
    for p in prompts:
        loop.submit(0.0, p, 1)
    sch.run_virtual(loop, 64, 1.0)
    t = loop.ttft()
    assert len(t) == len(prompts)
    return sum(t) / len(t)


def test_shortest_first_minimises_mean_ttft_by_brute_force():
    """All requests present at time 0, work-conserving batches: the k-th completion happens after the sum of the
    first k prompts, so the ascending order minimises every completion time at once (the textbook
    shortest-job-first argument).  Checked against every priority order of up to six requests."""
    rng = random.Random(7)
    for trial in range(6):
        n = rng.randint(3, 6)
        prompts = [rng.randint(1, 700) for _ in range(n)]
        best = min(_mean_ttft(list(p), prompts, 256) for p in itertools.permutations(range(n)))
        assert _mean_ttft(None, prompts, 256) == best, (trial, prompts)
    # and arrival order is strictly worse on the classic case of one long prompt ahead of short ones
    prompts = [2000, 100, 100, 100]
    assert _mean_ttft(None, prompts, 256) < _mean_ttft([0, 1, 2, 3], prompts, 256)


def test_age_term_prevents_starvation():
    """A long prompt behind a steady stream of short ones that always fill the budget: without the age term it is
    never scheduled, with it the prompt overtakes once gamma * age exceeds the length difference."""
    dt, budget, long_len, short_len = 0.05, 200, 4000, 100

    def first_token_of_long(gamma, iters):
        loop = sch.Loop(sch.SPF, budget, max_decode=1, page_size=16, n_pages=1 << 16, gamma=gamma)
        loop.submit(0.0, long_len, 1)
        for i in range(iters):
            loop.submit(i * dt, short_len, 1)
            loop.submit(i * dt, short_len, 1)
        sch.run_virtual(loop, iters, dt)
        return loop.reqs[0].first_token_time
    assert first_token_of_long(0.0, 400) is None
    gamma = 1500.0
    t = first_token_of_long(gamma, 400)
    overtake = (long_len - short_len) / gamma            # age at which the long prompt scores below a fresh short one
    assert t is not None and overtake < t <= overtake + (long_len / budget + 2) * dt


def test_printed_rule_never_schedules_a_prompt_longer_than_the_budget():
    loop = sch.Loop(sch.FCFS, budget=100, max_decode=1, page_size=16, n_pages=256, chunk_tail=False)
    loop.submit(0.0, 101, 1)
    loop.submit(0.0, 50, 1)
    its = sch.run_virtual(loop, 20, 1.0)
    assert all(it.prefill == [] for it in its)           # head of the queue never fits and nothing may pass it
    loop = sch.Loop(sch.FCFS, budget=100, max_decode=1, page_size=16, n_pages=256, chunk_tail=True)
    loop.submit(0.0, 101, 1)
    loop.submit(0.0, 50, 1)
    its = sch.run_virtual(loop, 3, 1.0)
    assert [it.prefill for it in its] == [[(0, 0, 100)], [(0, 100, 1), (1, 0, 50)], []]
    # a request that fills the budget exactly does fit (Alg. 2 compares with <=)
    loop = sch.Loop(sch.FCFS, budget=100, max_decode=1, page_size=16, n_pages=256, chunk_tail=False)
    loop.submit(0.0, 60, 1)
    loop.submit(0.0, 40, 1)
    assert loop.next(0.0).prefill == [(0, 0, 60), (1, 0, 40)]


def random_trace(seed, n, rate, prompt_cap=4000):
    rng = random.Random(seed)
    t, out = 0.0, []
    for _ in range(n):
        t += rng.expovariate(rate)
        out.append((t, min(prompt_cap, max(1, int(rng.lognormvariate(6.0, 1.0)))), max(1, int(rng.lognormvariate(3.0, 0.8)))))
    return out


def test_conservation_invariants_on_random_traces():
    for seed, policy in ((1, sch.FCFS), (2, sch.SPF), (3, sch.SPF)):
        trace = random_trace(seed, 120, rate=25.0)
        budget, cap, ps, dt = 512, 24, 16, 0.05
        loop = sch.Loop(policy, budget, cap, ps, n_pages=3000, gamma=15.0, max_prefill_reqs=8)
        for a, p, o in trace:
            loop.submit(a, p, o)
        chunks = {i: [] for i in range(len(trace))}
        ctxs = {i: [] for i in range(len(trace))}
        n_it = 0
        while any(r.finish_time is None for r in loop.reqs):
            it = loop.next(n_it * dt)
            assert sum(n for _, _, n in it.prefill) <= budget and len(it.prefill) <= 8
            assert len(it.decode) <= cap
            assert len({rid for rid, _, _ in it.prefill}) == len(it.prefill)
            held = [p for pages in it.page_tables.values() for p in pages]
            assert len(held) == len(set(held)) and all(0 <= p < 3000 for p in held)      # no page shared
            for rid, prefix, n in it.prefill:
                assert loop.reqs[rid].arrival <= it.now and n >= 1
                chunks[rid].append((prefix, n))
                assert len(it.page_tables[rid]) == sch.pages_for(prefix + n, ps)
            for rid, c in it.decode:
                ctxs[rid].append(c)
                assert len(it.page_tables[rid]) == sch.pages_for(c + 1, ps)
            # work conservation: tokens are left on the table only if no admitted request wants them
            waiting = sum(r.remaining for r in loop.reqs if r.arrival <= it.now and r.admitted)
            if len(it.prefill) < 8:
                assert sum(n for _, _, n in it.prefill) == min(budget, waiting)
            assert it.kv_used_pages == 3000 - len(loop.free)
            loop.commit((n_it + 1) * dt)
            n_it += 1
            assert n_it < 20000
        for i, (a, p, o) in enumerate(trace):
            r = loop.reqs[i]
            pos = 0
            for prefix, n in chunks[i]:
                assert prefix == pos
                pos += n
            assert pos == p
            assert ctxs[i] == list(range(p, p + o - 1))                   # one position per decoded token
            assert r.emitted == o and len(r.tbt) == o - 1
            assert r.first_token_time - a >= dt * -(-p // budget) - 1e-12  # at least ceil(p / B) iterations
            assert all(x >= dt - 1e-12 for x in r.tbt)
        assert loop.prefill_tokens == sum(p for _, p, _ in trace)
        assert loop.decode_tokens == sum(o - 1 for _, _, o in trace)
        assert len(loop.free) == 3000 and sorted(loop.free) == list(range(3000)) and loop.reserved_total == 0


def test_decode_pool_is_first_come_first_served():
    """Pool of one: requests decode in the order their prefill completed, each one only after the previous one
    has finished; the waiting time shows up as that request's first TBT."""
    loop = sch.Loop(sch.FCFS, budget=100, max_decode=1, page_size=16, n_pages=256)
    loop.submit(0.0, 10, 4)
    loop.submit(0.0, 10, 3)
    loop.submit(0.5, 10, 2)
    its = sch.run_virtual(loop, 8, 1.0)
    assert [it.decode for it in its] == [[], [(0, 10)], [(0, 11)], [(0, 12)], [(1, 10)], [(1, 11)], [(2, 10)], []]
    assert [r.tbt for r in loop.reqs] == [[1.0, 1.0, 1.0], [4.0, 1.0], [5.0]]
    assert loop.ttft() == [1.0, 1.0, 1.5]


def test_admission_waits_for_kv_space_without_reordering():
    """16 pages in all.  The first request's lifetime needs 10, the second's 8 (prompt and output together): the second waits until the first
    has finished and released its pages, and the third (which would fit) does not pass it."""
    loop = sch.Loop(sch.FCFS, budget=1000, max_decode=4, page_size=16, n_pages=16)
    loop.submit(0.0, 150, 3)     # 152 tokens -> 10 pages
    loop.submit(0.0, 96, 33)     # 128 tokens over its lifetime -> 8 pages (the prompt alone would need 6 and fit)
    loop.submit(0.0, 10, 1)      # 1 page
    its = sch.run_virtual(loop, 6, 1.0)
    assert [it.prefill for it in its] == [[(0, 0, 150)], [], [], [(1, 0, 96), (2, 0, 10)], [], []]
    assert max(it.kv_used_pages for it in its) <= 16

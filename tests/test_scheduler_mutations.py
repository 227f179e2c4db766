"""Plausible mistakes planted in a copy of the scheduler oracle: every one of them must make a pin fail."""
import os
import sys
import types

import pytest

import tests.test_scheduler_pins as pins

SRC = os.path.join(os.path.dirname(os.path.dirname(__file__)), "oracle", "scheduler.py")

MUTATIONS = [
    ("age raises the score instead of lowering it", "return remaining - gamma * age", "return remaining + gamma * age"),
    ("score uses the prompt length, not what remains", "spf_score(r.remaining, now - r.arrival, gamma)", "spf_score(r.prompt_len, now - r.arrival, gamma)"),
    ("age measured from time zero", "spf_score(r.remaining, now - r.arrival, gamma)", "spf_score(r.remaining, now, gamma)"),
    ("longest first", "return sorted(queue, key=lambda r: (spf_score(r.remaining, now - r.arrival, gamma), r.arrival, r.rid))",
     "return sorted(queue, key=lambda r: (-spf_score(r.remaining, now - r.arrival, gamma), r.arrival, r.rid))"),
    ("fit test strict", "if total + r.remaining <= budget:", "if total + r.remaining < budget:"),
    ("a request that does not fit is skipped instead of ending the batch",
     "                batch.append((r, budget - total))\n            break", "                batch.append((r, budget - total))\n            continue"),
    ("tail chunk ignores what the batch already holds", "batch.append((r, budget - total))", "batch.append((r, min(r.remaining, budget)))"),
    ("future arrivals are visible", "if r.arrival <= now and r.remaining > 0", "if r.remaining > 0"),
    ("decode context off by one", "ctx = r.prompt_len + r.emitted - 1", "ctx = r.prompt_len + r.emitted"),
    ("decode pool unbounded", "if len(self.pool) == self.max_decode:", "if False:"),
    ("pool order by arrival instead of prefill completion", "key=lambda r: (r.ready_time, r.arrival, r.rid))", "key=lambda r: (-r.arrival, r.rid))"),
    ("first token not counted", "r.emitted = 1\n", "r.emitted = 0\n"),
    ("pages never returned", "        self.free.extend(reversed(r.pages))\n", ""),
    ("reservation counts the prompt only", "need = pages_for(r.prompt_len + r.output_len - 1, self.page_size)", "need = pages_for(r.prompt_len, self.page_size)"),
    ("a blocked request lets later ones pass", "if blocked or self.reserved_total + need > self.n_pages:", "if self.reserved_total + need > self.n_pages:"),
    ("TBT measured from arrival", "r.tbt.append(end - r.last_token_time)", "r.tbt.append(end - r.arrival)"),
    ("normalised latency per prompt token", "(r.finish_time - r.arrival) / r.output_len", "(r.finish_time - r.arrival) / r.prompt_len"),
    ("TTFT from the start of the loop", "r.first_token_time - r.arrival for r", "r.first_token_time for r"),
]

PINS = [getattr(pins, n) for n in dir(pins) if n.startswith("test_")]


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_pins_catch(name, old, new, monkeypatch):
    src = open(SRC).read()
    assert src.count(old) == 1, f"mutation site not found exactly once: {old}"
    mod = types.ModuleType("scheduler_mutant")
    sys.modules["scheduler_mutant"] = mod  # dataclasses look the module up by name
    try:
        exec(compile(src.replace(old, new), SRC, "exec"), mod.__dict__)
        monkeypatch.setattr(pins, "sch", mod)
        failed = False
        for fn in PINS:
            try:
                fn()
            except Exception:
                failed = True
                break
        assert failed, f"no pin noticed: {name}"
    finally:
        sys.modules.pop("scheduler_mutant", None)

"""Host-only validation of a step's integer inputs (chunk offsets, lengths, page tables): the check that the debug
mode of the library runs before a step, driven here without a GPU."""
import numpy as np
import pytest
import torch

from paper_2507_06608_amd import synth


@pytest.fixture(scope="module")
def nx():
    from paper_2507_06608_amd import binding, build
    if build.stale():
        build.build()
    binding.lib()
    return binding


def _workload(seed=3):
    return synth.make_workload("v", synth.SHAPES["tiny"], seed, chunk_lens=[37, 1, 130], prefix_lens=[0, 47, 16],
                               decode_ctx=[0, 1, 15, 16, 17, 255, 256, 300, 31], page_slack=4)


def test_generated_workloads_validate(nx):
    wl = synth.config(1)
    nx.validate_batches(wl.n_pages, 16, wl.prefill, wl.decode)
    wl = _workload()
    nx.validate_batches(wl.n_pages, 16, wl.prefill, wl.decode)
    nx.validate_batches(wl.n_pages, 16, wl.prefill, None)
    nx.validate_batches(wl.n_pages, 16, None, wl.decode)
    # looser hints are fine
    nx.validate_batches(wl.n_pages, 16, wl.prefill, wl.decode, hints=dict(max_chunk=500, max_total_len=999, max_ctx=999))


def _mutate(what):
    wl = _workload()
    p, d = wl.prefill, wl.decode
    hints = {}
    if what == "page id past the pool":
        d.page_table[5, 3] = wl.n_pages
    elif what == "negative page id inside a request's range":
        p.page_table[2, 0] = -1
    elif what == "unused table entries may hold anything":
        p.page_table[1, 4:] = 10 ** 6          # request 1 holds 48 positions = 3 pages
        d.page_table[0, 1:] = -7
        return wl, hints, None
    elif what == "negative context length":
        d.ctx_len[2] = -1
    elif what == "negative prefix":
        p.prefix_len[0] = -5
    elif what == "offsets do not start at zero":
        p.cu_chunk[0] = 1
    elif what == "offsets decrease":
        p.cu_chunk[1], p.cu_chunk[2] = 38, 37
    elif what == "offsets do not end at n_tokens":
        hints["n_tokens"] = int(p.cu_chunk[-1]) + 1
    elif what == "chunk longer than the grid hint":
        hints["max_chunk"] = 129
    elif what == "total length beyond the hint":
        hints["max_total_len"] = 145
    elif what == "context beyond the hint":
        hints["max_ctx"] = 300
    elif what == "two requests append into one page":
        d.page_table[3, 1] = d.page_table[4, 1]            # ctx 16 and 17 both write logical page 1
    elif what == "a decode request writes a page a prefill request reads":
        d.page_table[0, 0] = p.page_table[2, 0]            # prefill request 2 reads its page 0 (prefix 16)
    elif what == "a prefill request writes a page a decode request reads":
        p.page_table[0, 1] = d.page_table[6, 2]
    elif what == "row too short for the request":
        keep = p.page_table[:, :5].copy()
        wl.prefill = synth.PrefillBatch(p.x, p.cu_chunk, p.prefix_len, keep)
    else:
        raise AssertionError(what)
    return wl, hints, "error"


CASES = ["page id past the pool", "negative page id inside a request's range", "unused table entries may hold anything",
         "negative context length", "negative prefix", "offsets do not start at zero", "offsets decrease",
         "offsets do not end at n_tokens", "chunk longer than the grid hint", "total length beyond the hint",
         "context beyond the hint", "two requests append into one page", "a decode request writes a page a prefill request reads",
         "a prefill request writes a page a decode request reads", "row too short for the request"]


@pytest.mark.parametrize("what", CASES)
def test_violations_are_named(nx, what):
    wl, hints, expect = _mutate(what)
    if expect is None:
        nx.validate_batches(wl.n_pages, 16, wl.prefill, wl.decode, hints=hints)
        return
    with pytest.raises(nx.NexusError) as e:
        nx.validate_batches(wl.n_pages, 16, wl.prefill, wl.decode, hints=hints)
    msg = str(e.value)
    assert "request" in msg or "cu_chunk" in msg, msg
    print(what, "->", msg)


def test_shared_read_only_prefix_pages_are_allowed(nx):
    """Two requests may read the same pages (a shared prompt prefix) as long as neither writes them."""
    wl = synth.make_workload("shared", synth.SHAPES["tiny"], 4, chunk_lens=[20, 20], prefix_lens=[32, 32], decode_ctx=[40])
    wl.prefill.page_table[1, :2] = wl.prefill.page_table[0, :2]      # both prefixes: the same two full pages
    nx.validate_batches(wl.n_pages, 16, wl.prefill, wl.decode)
    wl.prefill.page_table[1, 2] = wl.prefill.page_table[0, 2]        # but not the page both append to
    with pytest.raises(nx.NexusError, match="written by"):
        nx.validate_batches(wl.n_pages, 16, wl.prefill, wl.decode)

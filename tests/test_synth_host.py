"""Host-side checks of the synthetic input generators used by the trace loop and the fused baseline (no GPU)."""
import numpy as np

from paper_2507_06608_amd import synth


def test_poisson_trace_is_seeded_and_in_range():
    a = synth.poisson_trace(3, rate=8.0, horizon_s=20.0)
    b = synth.poisson_trace(3, rate=8.0, horizon_s=20.0)
    c = synth.poisson_trace(4, rate=8.0, horizon_s=20.0)
    assert a == b and a != c
    t = np.array([x[0] for x in a])
    assert (np.diff(t) > 0).all() and t[0] > 0 and t[-1] < 20.0
    assert 100 < len(a) < 230                                     # 160 expected, Poisson
    prompts = np.array([x[1] for x in a])
    outs = np.array([x[2] for x in a])
    assert prompts.min() >= 1 and prompts.max() <= 8192 and outs.min() >= 1 and outs.max() <= 2048
    assert 700 < np.median(prompts) < 1500 and 170 < np.median(outs) < 380    # medians 1024 and 256
    capped = synth.poisson_trace(3, rate=8.0, horizon_s=20.0, prompt_cap=500, output_cap=64)
    assert max(x[1] for x in capped) == 500 and max(x[2] for x in capped) == 64


def test_fused_single_batch_layout():
    wl = synth.config(1, seed=0)
    f = synth.fused_single_batch(wl)
    p, d = wl.prefill, wl.decode
    assert f.n_reqs == p.n_reqs + d.n_reqs and f.n_tokens == p.n_tokens + d.n_reqs
    assert f.cu_chunk.tolist() == p.cu_chunk.tolist() + [p.n_tokens + 1 + j for j in range(d.n_reqs)]
    assert f.prefix_len.tolist() == p.prefix_len.tolist() + d.ctx_len.tolist()
    assert (f.chunk_len[p.n_reqs:] == 1).all()
    assert (f.x[:p.n_tokens] == p.x).all()
    assert (f.x[p.n_tokens:] == d.x).all()
    w = f.page_table.shape[1]
    for j in range(d.n_reqs):
        row, src = f.page_table[p.n_reqs + j], d.page_table[j]
        assert row[:len(src)].tolist() == src.tolist() and (row[len(src):] == -1).all() and len(row) == w


def test_larger_configurations_have_the_stated_shapes():
    for idx, hidden, hq, hkv, ffn, layers in ((4, 5120, 40, 8, 13824, 48), (5, 8192, 64, 8, 28672, 80)):
        s = synth.SHAPES["qwen25_14b" if idx == 4 else "llama3_70b"]
        assert (s.hidden, s.n_q_heads, s.n_kv_heads, s.ffn, s.n_layers, s.head_dim) == (hidden, hq, hkv, ffn, layers, 128)
    assert synth.weight_std(synth.SHAPES["llama3_8b"]) == 0.02
    assert abs(synth.weight_std(synth.SHAPES["llama3_70b"]) - 0.02 / 2 ** 0.5) < 1e-12


def test_token_rows_of_the_loop_are_a_pure_function_of_request_and_position():
    from paper_2507_06608_amd.serve import ROW_STRIDE, token_rows
    r = token_rows(3, 100, 5, 4096)
    assert r.tolist() == [(3 * ROW_STRIDE + 100 + i) % 4096 for i in range(5)]
    # a chunk boundary does not change which row a position gets
    assert np.array_equal(np.concatenate([token_rows(7, 0, 60, 999), token_rows(7, 60, 40, 999)]), token_rows(7, 0, 100, 999))

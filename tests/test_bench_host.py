"""Host-side checks of bench.py: the one-GPU rule and the algorithmic work figures its rooflines divide by
(hand-computed from the shapes, Eq. 1-4: 2 T N K flops per projection, 4 hd Hq flops per visible (query, key) pair,
every weight byte and every cached K/V byte once per decode step)."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, cwd=ROOT)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stderr + r.stdout)


def test_algorithmic_work_of_the_8b_shaped_step_by_hand():
    import bench
    from paper_2507_06608_amd import synth
    wl = synth.config(2, seed=0)
    w = bench.algorithmic_work(wl, 1)
    T, d, ffn, nqkv, qd = 512, 4096, 14336, 6144, 4096
    assert w["prefill_flops"]["gemm_qkv"] == 2 * T * nqkv * d
    assert w["prefill_flops"]["gemm_o"] == 2 * T * d * qd
    assert w["prefill_flops"]["gemm_gate_up"] == 2 * T * 2 * ffn * d
    assert w["prefill_flops"]["gemm_down"] == 2 * T * d * ffn
    # one 512-token chunk over a 1536-token prefix: 512 * 1536 pairs with the prefix + 512 * 513 / 2 inside the chunk
    pairs = 512 * 1536 + 512 * 513 // 2
    assert w["prefill_flops"]["attn_prefill"] == 4 * 128 * 32 * pairs
    assert w["prefill_layer_flops"] == pytest.approx(238.4e9, rel=2e-3)
    params = nqkv * d + d * qd + 2 * ffn * d + d * ffn
    kv_tokens = int(sum(int(c) + 1 for c in wl.decode.ctx_len))
    assert w["decode_layer_bytes"] == 2 * params + kv_tokens * 2 * 8 * 128 * 2
    assert w["decode_bytes"]["attn_decode"] == kv_tokens * 4096
    assert w["tokens"] == 512 + 64


def test_algorithmic_work_of_the_70b_shaped_step_by_hand():
    import bench
    from paper_2507_06608_amd import synth
    wl = synth.config(5, seed=0)
    w = bench.algorithmic_work(wl, 80)
    T, d, ffn = 2048, 8192, 28672
    assert w["prefill_flops"]["gemm_gate_up"] == 2 * T * 2 * ffn * d == 1924145348608
    assert w["prefill_flops"]["gemm_down"] == 2 * T * d * ffn
    assert w["prefill_flops"]["gemm_qkv"] == 2 * T * (64 + 2 * 8) * 128 * d
    pairs = 2048 * 2048 + 2048 * 2049 // 2
    assert w["prefill_flops"]["attn_prefill"] == 4 * 128 * 64 * pairs
    assert w["prefill_layer_flops"] == pytest.approx(3.71e12, rel=3e-3)
    assert w["decode_bytes"]["gemm_gate_up"] == 2 * 2 * ffn * d

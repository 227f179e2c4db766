"""What the storage format of the KV cache alone costs at the 70B-shaped configuration with N(0, 0.02) weights.

The path stores keys and values as bf16 (8 significant bits).  This test takes the CPU oracle, changes NOTHING but
that one fact -- the K/V a chunk appends are rounded to bf16 when stored, every other operation stays the oracle's
fp64 arithmetic -- and measures the layer output against the unrounded oracle with the bar the GPU tests use
(|err| <= 2e-2 + 2e-2 |ref|).  At hidden 8192 / FFN 28672 with N(0, 0.02) weights every projection amplifies
(gain 0.02 sqrt(fan-in) = 1.8 for the four 8192-wide ones, 3.4 for the down projection) and the layer output has an
rms of ~7, so the absolute term of the bar is 0.3 % of the output scale: the 2^-9 relative rounding of the cached
keys and values, carried through the softmax, the output projection and the feed-forward block, already exceeds it.
No kernel that keeps a bf16 KV cache can therefore meet the elementwise bar on this recipe, whatever its own
arithmetic; the relative L2 error stays far inside its bar.  With the weight variance following the fan-in
(0.02 sqrt(4096 / 8192)) the same rounding stays inside the bar, which is the recipe the GPU parity case of this
configuration is gated on; the GPU test reports both."""
import numpy as np
import torch

from paper_2507_06608_amd import synth
from tests.parity_util import ATOL, RTOL, oracle_model


def _bf16(a):
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(torch.bfloat16).float().numpy()


def _layer_by_steps(o, m, w, x, prefix, table, kp, vp, store):
    """The chunked-prefill layer composed from the oracle's own primitives in the order of its layer function;
    `store` is applied to a token's rotated K and its V before they are written to the cache."""
    T = x.shape[0]
    qd, kvd = m.n_q_heads * m.head_dim, m.n_kv_heads * m.head_dim
    qkv = o.linear(o.rmsnorm(x, w["attn_norm_g"], m.rms_eps), w["w_qkv"])
    q = np.empty((T, m.n_q_heads, m.head_dim), np.float32)
    for t in range(T):
        q[t] = o.rope(qkv[t, :qd].reshape(m.n_q_heads, m.head_dim), prefix + t, m.rope_theta)
        k = o.rope(qkv[t, qd:qd + kvd].reshape(m.n_kv_heads, m.head_dim), prefix + t, m.rope_theta)
        v = qkv[t, qd + kvd:].reshape(m.n_kv_heads, m.head_dim)
        o.kv_append(m, kp, vp, table, prefix + t, store(k), store(v))
    a = np.stack([o.attention_paged(m, q[t], prefix + t, kp, vp, table).reshape(-1) for t in range(T)])
    x1 = (x.astype(np.float64) + o.linear(a, w["w_o"])).astype(np.float32)
    act = o.swiglu(o.linear(o.rmsnorm(x1, w["ffn_norm_g"], m.rms_eps), w["w_gate_up"]), m.ffn)
    return (x1.astype(np.float64) + o.linear(act, w["w_down"])).astype(np.float32)


def _worst_and_fraction(y, ref):
    err, bound = np.abs(y.astype(np.float64) - ref), ATOL + RTOL * np.abs(ref)
    rel = np.linalg.norm(y - ref) / np.linalg.norm(ref)
    return float((err / bound).max()), float((err > bound).mean()), float(rel)


def test_bf16_kv_storage_alone_misses_the_elementwise_bar_at_70b_width_with_std_002(oracle):
    sh = synth.SHAPES["llama3_70b"]
    m = oracle_model(oracle, sh)
    T, prefix = 12, 52
    rng = np.random.default_rng(5)
    x = _bf16(rng.standard_normal((T, sh.hidden), dtype=np.float32))
    n_pages = (prefix + T + sh.page_size - 1) // sh.page_size
    table = rng.permutation(n_pages).astype(np.int32)
    pool = (n_pages, sh.n_kv_heads, sh.page_size, sh.head_dim)
    k0, v0 = _bf16(rng.standard_normal(pool, dtype=np.float32)), _bf16(rng.standard_normal(pool, dtype=np.float32))
    results = {}
    for tag, std in (("N(0, 0.02)", 0.02), ("fan-in", None)):
        w = {k: v.float().numpy() for k, v in synth.make_weights(sh, 0, 79, std=std).items()}
        kp, vp = k0.copy(), v0.copy()
        ref = oracle.layer_prefill(m, w, x, [0, T], [prefix], table[None], kp, vp)
        if std is not None:
            # the composition is the oracle's layer, step for step
            kp, vp = k0.copy(), v0.copy()
            same = _layer_by_steps(oracle, m, w, x, prefix, table, kp, vp, lambda t: t)
            assert np.array_equal(same, ref)
        kp, vp = k0.copy(), v0.copy()
        y = _layer_by_steps(oracle, m, w, x, prefix, table, kp, vp, _bf16)
        if std is not None:
            # the storage switch of the row-subset entry is this composition: torch's bf16 rounding, bit for bit
            kp2, vp2 = k0.copy(), v0.copy()
            y2 = oracle.layer_prefill_rows(m, w, x, [0, T], [prefix], table[None], kp2, vp2, np.arange(T), kv_store_bf16=True)
            assert np.array_equal(y2, y) and np.array_equal(kp2, kp) and np.array_equal(vp2, vp)
        results[tag] = _worst_and_fraction(y, ref)
        print(f"[kv storage floor] 70B width, weights {tag}: output rms {ref.std():.2f}, bf16 K/V storage alone -> worst "
              f"err/bound {results[tag][0]:.2f}, {100 * results[tag][1]:.2f} % of outputs outside the bar, rel L2 {results[tag][2]:.2e}", flush=True)
        del w
    worst, frac, rel = results["N(0, 0.02)"]
    assert worst > 1.5 and frac > 1e-3, "the storage rounding alone was expected to break the elementwise bar here"
    assert rel < 1e-2
    worst, frac, rel = results["fan-in"]
    assert worst < 0.6 and frac == 0.0 and rel < 1e-2

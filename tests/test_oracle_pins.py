"""Pins of the CPU oracle against facts fixed by the mathematics, not by the oracle itself.

The paper prints no worked numeric example of a layer output, so the pins are
closed forms, invariants, special cases that reduce to library routines
(numpy fp64 matmul, scipy softmax, complex multiplication) and brute force on
tiny shapes written in a different formulation (dense masked matrices).
"""
import math

import numpy as np
import pytest
from scipy.special import softmax

rng = np.random.default_rng(1234)


def _model(o, **kw):
    base = dict(hidden=32, n_q_heads=4, n_kv_heads=2, head_dim=8, ffn=24, page_size=4, rms_eps=1e-5,
                rope_theta=10000.0)
    base.update(kw)
    return o.Model(**base)


def _weights(m, scale=0.2, r=rng):
    d, F = m.hidden, m.ffn
    qd, kvd = m.n_q_heads * m.head_dim, m.n_kv_heads * m.head_dim
    f = lambda *s: (r.standard_normal(s) * scale).astype(np.float32)
    return {"attn_norm_g": (1 + f(d)).astype(np.float32), "w_qkv": f(qd + 2 * kvd, d), "b_qkv": None,
            "w_o": f(d, qd), "ffn_norm_g": (1 + f(d)).astype(np.float32), "w_gate_up": f(2 * F, d),
            "w_down": f(d, F)}


# ---------------------------------------------------------------- RMSNorm
def test_rmsnorm_scale_invariant_and_unit_rms(oracle):
    x = rng.standard_normal((5, 64)).astype(np.float32)
    g = np.ones(64, np.float32)
    a = oracle.rmsnorm(x, g, 0.0)
    b = oracle.rmsnorm(4.0 * x, g, 0.0)           # power-of-two scale: exact in fp32
    np.testing.assert_allclose(a, b, rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(np.sqrt((a.astype(np.float64) ** 2).mean(1)), 1.0, rtol=1e-6)


def test_rmsnorm_constant_vector_closed_form(oracle):
    d, c, eps = 48, -3.0, 0.25
    g = rng.standard_normal(d).astype(np.float32)
    out = oracle.rmsnorm(np.full((1, d), c, np.float32), g, eps)
    expect = g.astype(np.float64) * c / math.sqrt(c * c + eps)
    np.testing.assert_allclose(out[0], expect, rtol=1e-6)


def test_rmsnorm_gain_is_applied_per_feature(oracle):
    x = rng.standard_normal((3, 16)).astype(np.float32)
    g = np.zeros(16, np.float32)
    g[5] = 2.0
    out = oracle.rmsnorm(x, g, 1e-5)
    assert np.all(out[:, np.arange(16) != 5] == 0)
    expect = 2.0 * x[:, 5] / np.sqrt((x.astype(np.float64) ** 2).mean(1) + 1e-5)
    np.testing.assert_allclose(out[:, 5], expect, rtol=1e-6)


# ---------------------------------------------------------------- linear
def test_linear_matches_fp64_matmul_nonsquare(oracle):
    x = rng.standard_normal((7, 19)).astype(np.float32)
    W = rng.standard_normal((11, 19)).astype(np.float32)
    b = rng.standard_normal(11).astype(np.float32)
    np.testing.assert_allclose(oracle.linear(x, W), x.astype(np.float64) @ W.astype(np.float64).T, rtol=1e-6,
                               atol=1e-6)
    np.testing.assert_allclose(oracle.linear(x, W, b), x.astype(np.float64) @ W.astype(np.float64).T + b,
                               rtol=1e-6, atol=1e-6)


def test_linear_one_hot_selects_weight_column(oracle):
    W = rng.standard_normal((6, 9)).astype(np.float32)
    x = np.zeros((1, 9), np.float32)
    x[0, 4] = 1.0
    assert np.array_equal(oracle.linear(x, W)[0], W[:, 4])


# ---------------------------------------------------------------- RoPE
def test_rope_hand_values_hd4(oracle):
    # head_dim 4, theta 10000, pos 1: angles are 1 and 10000^(-1/2) = 0.01; pairs (0,2) and (1,3).
    u = np.array([[1.0, 2.0, 3.0, 4.0]], np.float32)
    out = oracle.rope(u, 1, 10000.0)[0]
    c1, s1, c2, s2 = math.cos(1.0), math.sin(1.0), math.cos(0.01), math.sin(0.01)
    expect = [1 * c1 - 3 * s1, 2 * c2 - 4 * s2, 3 * c1 + 1 * s1, 4 * c2 + 2 * s2]
    np.testing.assert_allclose(out, expect, rtol=1e-6)
    # independently typed decimal values of the same four numbers
    np.testing.assert_allclose(out, [-1.9841106, 1.9599007, 2.4623780, 4.0197997], atol=2e-6)


def test_rope_is_complex_rotation(oracle):
    hd, theta, pos = 16, 500000.0, 37
    u = rng.standard_normal((3, hd)).astype(np.float32)
    out = oracle.rope(u, pos, theta)
    z = u[:, :hd // 2].astype(np.float64) + 1j * u[:, hd // 2:].astype(np.float64)
    ang = pos * theta ** (-np.arange(hd // 2) * 2.0 / hd)
    zr = z * np.exp(1j * ang)
    np.testing.assert_allclose(out[:, :hd // 2], zr.real, rtol=1e-5, atol=1e-6)
    np.testing.assert_allclose(out[:, hd // 2:], zr.imag, rtol=1e-5, atol=1e-6)


def test_rope_pos0_identity_norms_and_relative_property(oracle):
    hd, theta = 32, 10000.0
    q = rng.standard_normal((1, hd)).astype(np.float32)
    k = rng.standard_normal((1, hd)).astype(np.float32)
    assert np.array_equal(oracle.rope(q, 0, theta), q)
    r = oracle.rope(q, 911, theta)
    half = hd // 2
    np.testing.assert_allclose(r[0, :half] ** 2 + r[0, half:] ** 2, q[0, :half] ** 2 + q[0, half:] ** 2, rtol=1e-5)
    dots = [float(oracle.rope(q, m, theta)[0].astype(np.float64) @ oracle.rope(k, n, theta)[0].astype(np.float64))
            for m, n in ((5, 2), (105, 102), (1003, 1000))]
    np.testing.assert_allclose(dots, dots[0], rtol=1e-4, atol=1e-5)
    other = float(oracle.rope(q, 5, theta)[0].astype(np.float64) @ oracle.rope(k, 3, theta)[0].astype(np.float64))
    assert abs(other - dots[0]) > 1e-3          # and it does depend on the offset


# ---------------------------------------------------------------- paging
def test_kv_slot_hand_table(oracle):
    # 3 logical pages of 4 tokens mapped to physical pages 7, 2, 5
    row = [7, 2, 5]
    expect = [(7, 0), (7, 1), (7, 2), (7, 3), (2, 0), (2, 1), (2, 2), (2, 3), (5, 0), (5, 1), (5, 2), (5, 3)]
    assert [oracle.kv_slot(row, p, 4) for p in range(12)] == expect


def test_kv_append_writes_exactly_one_slot_per_head(oracle):
    m = _model(oracle)
    shape = (6, m.n_kv_heads, m.page_size, m.head_dim)
    kp = np.full(shape, -7.0, np.float32)
    vp = np.full(shape, -9.0, np.float32)
    k = rng.standard_normal((m.n_kv_heads, m.head_dim)).astype(np.float32)
    v = rng.standard_normal((m.n_kv_heads, m.head_dim)).astype(np.float32)
    oracle.kv_append(m, kp, vp, [4, 1, 3], 6, k, v)      # pos 6 -> logical page 1 (physical 1), slot 2
    touched = np.zeros(shape[:3], bool)
    touched[1, :, 2] = True
    assert np.array_equal(kp[1, :, 2], k) and np.array_equal(vp[1, :, 2], v)
    assert np.all(kp[~touched] == -7.0) and np.all(vp[~touched] == -9.0)


def _paged_from_contig(m, K, V, perm_seed):
    L = K.shape[0]
    n_log = (L + m.page_size - 1) // m.page_size
    n_pages = n_log + 3
    r = np.random.default_rng(perm_seed)
    row = r.permutation(n_pages)[:n_log].astype(np.int32)
    kp = r.standard_normal((n_pages, m.n_kv_heads, m.page_size, m.head_dim)).astype(np.float32)
    vp = r.standard_normal((n_pages, m.n_kv_heads, m.page_size, m.head_dim)).astype(np.float32)
    for u in range(L):
        kp[row[u // m.page_size], :, u % m.page_size] = K[u]
        vp[row[u // m.page_size], :, u % m.page_size] = V[u]
    return kp, vp, row


def test_paged_attention_equals_contiguous_bit_exact_and_page_permutation_invariant(oracle):
    m = _model(oracle)
    L = 23
    K = rng.standard_normal((L, m.n_kv_heads, m.head_dim)).astype(np.float32)
    V = rng.standard_normal((L, m.n_kv_heads, m.head_dim)).astype(np.float32)
    q = rng.standard_normal((m.n_q_heads, m.head_dim)).astype(np.float32)
    ref = oracle.attention_contig(m, q, L - 1, K, V)
    for s in (1, 2):
        kp, vp, row = _paged_from_contig(m, K, V, s)
        assert np.array_equal(oracle.attention_paged(m, q, L - 1, kp, vp, row), ref)
        kg, vg = oracle.kv_gather(m, kp, vp, row, L)
        assert np.array_equal(kg, K) and np.array_equal(vg, V)


# ---------------------------------------------------------------- attention
def _brute_attention(m, q, pos, K, V):
    """fp64, dense formulation with explicitly repeated KV heads and scipy softmax."""
    G = m.n_q_heads // m.n_kv_heads
    Kr = np.repeat(K[:pos + 1].astype(np.float64), G, axis=1)      # [n, Hq, hd]
    Vr = np.repeat(V[:pos + 1].astype(np.float64), G, axis=1)
    s = np.einsum("hd,nhd->hn", q.astype(np.float64), Kr) / math.sqrt(m.head_dim)
    p = softmax(s, axis=1)
    return np.einsum("hn,nhd->hd", p, Vr), p


@pytest.mark.parametrize("Hq,Hkv,hd,L", [(1, 1, 4, 1), (2, 1, 4, 5), (4, 2, 8, 8), (6, 2, 2, 7), (4, 4, 4, 6)])
def test_attention_brute_force_tiny(oracle, Hq, Hkv, hd, L):
    m = _model(oracle, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=hd)
    K = rng.standard_normal((L, Hkv, hd)).astype(np.float32) * 2
    V = rng.standard_normal((L, Hkv, hd)).astype(np.float32)
    q = rng.standard_normal((Hq, hd)).astype(np.float32) * 2
    for pos in (0, L // 2, L - 1):
        a, p = oracle.attention_contig(m, q, pos, K, V, want_p=True)
        ea, ep = _brute_attention(m, q, pos, K, V)
        np.testing.assert_allclose(a, ea, rtol=2e-6, atol=2e-7)
        np.testing.assert_allclose(p, ep, rtol=2e-6, atol=1e-8)
        np.testing.assert_allclose(p.astype(np.float64).sum(1), 1.0, atol=1e-6)


def test_attention_special_cases(oracle):
    m = _model(oracle, n_q_heads=4, n_kv_heads=2, head_dim=8)
    L = 9
    K = rng.standard_normal((L, 2, 8)).astype(np.float32)
    V = rng.standard_normal((L, 2, 8)).astype(np.float32)
    q = rng.standard_normal((4, 8)).astype(np.float32)
    # one visible key: output is that key's V row of the right kv head (q head h -> kv head h // 2)
    a0 = oracle.attention_contig(m, q, 0, K, V)
    assert np.array_equal(a0, V[0][[0, 0, 1, 1]])
    # all V rows equal: output is that row
    Vc = np.broadcast_to(V[3], V.shape).copy()
    np.testing.assert_allclose(oracle.attention_contig(m, q, L - 1, K, Vc), V[3][[0, 0, 1, 1]], rtol=1e-6)
    # all keys equal: uniform weights, output is the mean of the visible V rows
    Kc = np.broadcast_to(K[2], K.shape).copy()
    np.testing.assert_allclose(oracle.attention_contig(m, q, 5, Kc, V),
                               V[:6].astype(np.float64).mean(0)[[0, 0, 1, 1]], rtol=1e-5, atol=1e-6)
    # a large score gap: softmax saturates on the matching key (catches a missing 1/sqrt(hd) only weakly,
    # the brute-force test above is the scale pin)
    Kbig = np.zeros_like(K)
    Kbig[4, :, 0] = 100.0
    qbig = np.zeros_like(q)
    qbig[:, 0] = 100.0
    np.testing.assert_allclose(oracle.attention_contig(m, qbig, L - 1, Kbig, V), V[4][[0, 0, 1, 1]], atol=1e-6)


def test_attention_causal_future_is_never_read(oracle):
    m = _model(oracle)
    L, pos = 12, 6
    K = rng.standard_normal((L, m.n_kv_heads, m.head_dim)).astype(np.float32)
    V = rng.standard_normal((L, m.n_kv_heads, m.head_dim)).astype(np.float32)
    q = rng.standard_normal((m.n_q_heads, m.head_dim)).astype(np.float32)
    a = oracle.attention_contig(m, q, pos, K, V)
    K2, V2 = K.copy(), V.copy()
    K2[pos + 1:] = np.nan
    V2[pos + 1:] = np.nan
    assert np.array_equal(oracle.attention_contig(m, q, pos, K2, V2), a)
    # ...and position pos itself is read
    K3 = K.copy()
    K3[pos] += 1.0
    assert not np.array_equal(oracle.attention_contig(m, q, pos, K3, V), a)


def test_gqa_equals_mha_on_repeated_kv_heads(oracle):
    m = _model(oracle, n_q_heads=6, n_kv_heads=2, head_dim=4)
    mm = _model(oracle, n_q_heads=6, n_kv_heads=6, head_dim=4)
    L = 10
    K = rng.standard_normal((L, 2, 4)).astype(np.float32)
    V = rng.standard_normal((L, 2, 4)).astype(np.float32)
    q = rng.standard_normal((6, 4)).astype(np.float32)
    a = oracle.attention_contig(m, q, L - 1, K, V)
    b = oracle.attention_contig(mm, q, L - 1, np.repeat(K, 3, 1), np.repeat(V, 3, 1))
    assert np.array_equal(a, b)


# ---------------------------------------------------------------- SwiGLU
def test_swiglu_values(oracle):
    gu = np.array([[0.0, 1.0, -2.0, 5.0, 3.0, 0.5]], np.float32)      # F = 3: gate then up
    out = oracle.swiglu(gu, 3)[0]
    sig = lambda z: 1.0 / (1.0 + math.exp(-z))
    np.testing.assert_allclose(out, [0.0, 1.0 * sig(1.0) * 3.0, -2.0 * sig(-2.0) * 0.5], rtol=1e-6)
    assert out[0] == 0.0


# ---------------------------------------------------------------- whole layer
def _numpy_layer(m, w, x, pos, Kprev, Vprev):
    """Independent fp64 formulation of the layer for one request: tokens x at
    consecutive positions pos[0].., previous keys/values Kprev/Vprev [p, Hkv, hd]
    (already rotated).  Dense masked attention, complex-number RoPE."""
    f8 = lambda a: np.asarray(a, np.float64)
    d, hd, Hq, Hkv = m.hidden, m.head_dim, m.n_q_heads, m.n_kv_heads
    G = Hq // Hkv
    x = f8(x)

    def rms(v, g):
        return v / np.sqrt((v ** 2).mean(-1, keepdims=True) + m.rms_eps) * f8(g)

    def rot(u, positions):                       # u [T, H, hd]
        z = u[..., :hd // 2] + 1j * u[..., hd // 2:]
        ang = np.asarray(positions, np.float64)[:, None, None] * m.rope_theta ** (-np.arange(hd // 2) * 2.0 / hd)
        z = z * np.exp(1j * ang)
        return np.concatenate([z.real, z.imag], -1)

    h = rms(x, w["attn_norm_g"])
    qkv = h @ f8(w["w_qkv"]).T
    T = x.shape[0]
    q = rot(qkv[:, :Hq * hd].reshape(T, Hq, hd), pos)
    k = rot(qkv[:, Hq * hd:(Hq + Hkv) * hd].reshape(T, Hkv, hd), pos)
    v = qkv[:, (Hq + Hkv) * hd:].reshape(T, Hkv, hd)
    Kall = np.concatenate([f8(Kprev), k], 0)
    Vall = np.concatenate([f8(Vprev), v], 0)
    Kr, Vr = np.repeat(Kall, G, 1), np.repeat(Vall, G, 1)
    s = np.einsum("thd,nhd->htn", q, Kr) / math.sqrt(hd)
    key_pos = np.arange(Kall.shape[0])[None, None, :]
    s = np.where(key_pos <= np.asarray(pos)[None, :, None], s, -np.inf)
    a = np.einsum("htn,nhd->thd", softmax(s, axis=2), Vr).reshape(T, Hq * hd)
    x1 = x + a @ f8(w["w_o"]).T
    h2 = rms(x1, w["ffn_norm_g"])
    gu = h2 @ f8(w["w_gate_up"]).T
    g_, u_ = gu[:, :m.ffn], gu[:, m.ffn:]
    y = x1 + (g_ / (1 + np.exp(-g_)) * u_) @ f8(w["w_down"]).T
    return y, k, v, q.reshape(T, Hq * hd), a, x1


def _empty_pools(m, n_pages, fill=np.nan):
    shape = (n_pages, m.n_kv_heads, m.page_size, m.head_dim)
    return np.full(shape, fill, np.float32), np.full(shape, fill, np.float32)


def test_layer_prefill_matches_independent_numpy_formulation(oracle):
    m = _model(oracle)
    w = _weights(m)
    T = 11
    x = rng.standard_normal((T, m.hidden)).astype(np.float32)
    kp, vp = _empty_pools(m, 5)
    row = np.array([[3, 0, 4]], np.int32)
    y, dbg = oracle.layer_prefill(m, w, x, [0, T], [0], row, kp, vp, debug=True)
    ey, ek, ev, eq, ea, ex1 = _numpy_layer(m, w, x, np.arange(T), np.zeros((0, 2, 8)), np.zeros((0, 2, 8)))
    np.testing.assert_allclose(dbg["q"], eq, rtol=1e-4, atol=1e-5)
    np.testing.assert_allclose(dbg["attn"], ea, rtol=1e-4, atol=1e-5)
    np.testing.assert_allclose(dbg["x1"], ex1, rtol=1e-4, atol=1e-5)
    np.testing.assert_allclose(y, ey, rtol=1e-4, atol=1e-5)
    kg, vg = oracle.kv_gather(m, kp, vp, row[0], T)
    np.testing.assert_allclose(kg, ek, rtol=1e-4, atol=1e-5)
    np.testing.assert_allclose(vg, ev, rtol=1e-4, atol=1e-5)
    # pages not in the table, and slots past the chunk, were never written
    assert np.isnan(kp[[1, 2]]).all() and np.isnan(kp[4, :, T - 8:]).all()


def test_layer_prefill_with_prefix_and_two_requests(oracle):
    m = _model(oracle)
    w = _weights(m)
    p0, n0, n1 = 6, 5, 7
    x = rng.standard_normal((n0 + n1, m.hidden)).astype(np.float32)
    kp, vp = _empty_pools(m, 8)
    pt = np.array([[5, 1, 7], [2, 6, -1]], np.int32)
    Kprev = rng.standard_normal((p0, 2, 8)).astype(np.float32)
    Vprev = rng.standard_normal((p0, 2, 8)).astype(np.float32)
    for u in range(p0):
        kp[pt[0, u // 4], :, u % 4] = Kprev[u]
        vp[pt[0, u // 4], :, u % 4] = Vprev[u]
    y = oracle.layer_prefill(m, w, x, [0, n0, n0 + n1], [p0, 0], pt, kp, vp)
    e0 = _numpy_layer(m, w, x[:n0], p0 + np.arange(n0), Kprev, Vprev)[0]
    e1 = _numpy_layer(m, w, x[n0:], np.arange(n1), np.zeros((0, 2, 8)), np.zeros((0, 2, 8)))[0]
    np.testing.assert_allclose(y[:n0], e0, rtol=1e-4, atol=1e-5)
    np.testing.assert_allclose(y[n0:], e1, rtol=1e-4, atol=1e-5)


def test_layer_prefill_rows_equals_the_full_layer_on_those_rows(oracle):
    """The row-subset entry point (what the full-size GPU tests call for the last strips of long chunks) against
    the pinned whole-batch function: same rows bit for bit, in the order asked for, and the same pools -- with two
    requests, a cached prefix, a QKV bias, rows out of order, and against the independent numpy formulation."""
    m = _model(oracle)
    w = _weights(m)
    qd, kvd = m.n_q_heads * m.head_dim, m.n_kv_heads * m.head_dim
    w["b_qkv"] = (rng.standard_normal(qd + 2 * kvd) * 0.3).astype(np.float32)
    p0, n0, n1 = 6, 5, 7
    x = rng.standard_normal((n0 + n1, m.hidden)).astype(np.float32)
    pt = np.array([[5, 1, 7], [2, 6, -1]], np.int32)
    kp, vp = _empty_pools(m, 8)
    for u in range(p0):
        kp[pt[0, u // 4], :, u % 4] = rng.standard_normal((2, 8)).astype(np.float32)
        vp[pt[0, u // 4], :, u % 4] = rng.standard_normal((2, 8)).astype(np.float32)
    kp2, vp2 = kp.copy(), vp.copy()
    full = oracle.layer_prefill(m, w, x, [0, n0, n0 + n1], [p0, 0], pt, kp, vp)
    rows = [n0 + n1 - 1, 0, n0 - 1, n0, 7]
    part = oracle.layer_prefill_rows(m, w, x, [0, n0, n0 + n1], [p0, 0], pt, kp2, vp2, rows)
    assert part.shape == (len(rows), m.hidden)
    assert np.array_equal(part, full[rows])
    assert np.array_equal(kp, kp2, equal_nan=True) and np.array_equal(vp, vp2, equal_nan=True)
    # and directly against the numpy formulation (which knows no bias: fold it out by a second run without one)
    w["b_qkv"] = None
    kp3, vp3 = _empty_pools(m, 8)
    part = oracle.layer_prefill_rows(m, w, x[n0:], [0, n1], [0], pt[1:], kp3, vp3, [n1 - 1, 2])
    e1 = _numpy_layer(m, w, x[n0:], np.arange(n1), np.zeros((0, 2, 8)), np.zeros((0, 2, 8)))[0]
    np.testing.assert_allclose(part, e1[[n1 - 1, 2]], rtol=1e-4, atol=1e-5)


def test_chunked_prefill_equals_one_shot(oracle):
    m = _model(oracle)
    w = _weights(m)
    T = 19
    x = rng.standard_normal((T, m.hidden)).astype(np.float32)
    row = np.array([[2, 0, 4, 1, 3]], np.int32)
    kp, vp = _empty_pools(m, 5)
    y_one = oracle.layer_prefill(m, w, x, [0, T], [0], row, kp, vp)
    for cuts in ([5], [1], [8, 12], [16]):
        kq, vq = _empty_pools(m, 5)
        edges = [0] + cuts + [T]
        ys = [oracle.layer_prefill(m, w, x[a:b], [0, b - a], [a], row, kq, vq) for a, b in zip(edges, edges[1:])]
        assert np.array_equal(np.concatenate(ys, 0), y_one)
        assert np.array_equal(kq[~np.isnan(kq)], kp[~np.isnan(kp)])


def test_decode_equals_last_row_of_prefill(oracle):
    m = _model(oracle)
    w = _weights(m)
    L = 13
    x = rng.standard_normal((L + 1, m.hidden)).astype(np.float32)
    row = np.array([[1, 3, 0, 2]], np.int32)
    kp, vp = _empty_pools(m, 4)
    y_all = oracle.layer_prefill(m, w, x, [0, L + 1], [0], row, kp, vp)
    kq, vq = _empty_pools(m, 4)
    oracle.layer_prefill(m, w, x[:L], [0, L], [0], row, kq, vq)
    y_dec = oracle.layer_decode(m, w, x[L:], [L], row, kq, vq)
    assert np.array_equal(y_dec[0], y_all[L])
    assert np.array_equal(kq[~np.isnan(kq)], kp[~np.isnan(kp)])


def test_decode_batch_matches_numpy_and_requests_are_independent(oracle):
    m = _model(oracle)
    w = _weights(m)
    ctx = [5, 9, 4]
    pt = np.array([[6, 2, -1], [0, 5, 3], [1, 4, -1]], np.int32)
    kp = rng.standard_normal((7, 2, 4, 8)).astype(np.float32)
    vp = rng.standard_normal((7, 2, 4, 8)).astype(np.float32)
    x = rng.standard_normal((3, m.hidden)).astype(np.float32)
    k0, v0 = kp.copy(), vp.copy()
    y = oracle.layer_decode(m, w, x, ctx, pt, kp, vp)
    for j, c in enumerate(ctx):
        Kprev, Vprev = oracle.kv_gather(m, k0, v0, pt[j], c)
        ey = _numpy_layer(m, w, x[j:j + 1], np.array([c]), Kprev, Vprev)[0]
        np.testing.assert_allclose(y[j], ey[0], rtol=1e-4, atol=1e-5)
    # exactly one slot per request and kv head changed
    changed = (kp != k0).any(-1)
    expect = np.zeros_like(changed)
    for j, c in enumerate(ctx):
        expect[pt[j, c // 4], :, c % 4] = True
    assert np.array_equal(changed, expect)


def test_residual_identities(oracle):
    m = _model(oracle)
    w = _weights(m)
    x = rng.standard_normal((6, m.hidden)).astype(np.float32)
    row = np.array([[0, 1]], np.int32)
    wz = dict(w, w_o=np.zeros_like(w["w_o"]), w_down=np.zeros_like(w["w_down"]))
    kp, vp = _empty_pools(m, 2, 0.0)
    assert np.array_equal(oracle.layer_prefill(m, wz, x, [0, 6], [0], row, kp, vp), x)
    wg = dict(w, w_gate_up=np.concatenate([np.zeros((m.ffn, m.hidden), np.float32), w["w_gate_up"][m.ffn:]]))
    kp, vp = _empty_pools(m, 2, 0.0)
    y, dbg = oracle.layer_prefill(m, wg, x, [0, 6], [0], row, kp, vp, debug=True)
    assert np.array_equal(y, dbg["x1"])


def test_qkv_bias_is_added_before_rotation(oracle):
    m = _model(oracle)
    w = _weights(m)
    nq = (m.n_q_heads + 2 * m.n_kv_heads) * m.head_dim
    b = rng.standard_normal(nq).astype(np.float32)
    x = rng.standard_normal((4, m.hidden)).astype(np.float32)
    row = np.array([[0]], np.int32)
    kp, vp = _empty_pools(m, 1, 0.0)
    _, dbg = oracle.layer_prefill(m, dict(w, b_qkv=b), x, [0, 4], [0], row, kp, vp, debug=True)
    h = oracle.rmsnorm(x, w["attn_norm_g"], m.rms_eps)
    q = oracle.linear(h, w["w_qkv"], b)[:, :m.n_q_heads * m.head_dim]
    expect = np.stack([oracle.rope(q[t].reshape(m.n_q_heads, m.head_dim), t, m.rope_theta).ravel() for t in range(4)])
    np.testing.assert_allclose(dbg["q"], expect, rtol=1e-6, atol=1e-6)


# ---------------------------------------------------------------- split selection
def test_choose_split_equals_exhaustive_scan(oracle):
    r = np.random.default_rng(5)
    for trial in range(50):
        n = int(r.integers(2, 9))
        share = np.sort(r.choice(np.arange(1, 16), n, replace=False)) / 16.0
        t_p = (1.0 / share + r.random(n) * 0.05).astype(np.float32)            # falls with the prefill share
        t_d = (1.0 + 0.3 / (1 - share) + r.random(n) * 0.05).astype(np.float32)  # rises with it
        t_s = np.maximum(t_p, t_d) * (1 + r.random(n).astype(np.float32) * 0.1)
        tpm, tdm = float(t_p.min() * 0.9), float(t_d.min() * 0.95)
        for pol, a, b in ((0, 1.3, 1.1), (1, 1.3, 1.1), (2, 1.3, 1.1), (0, 1.3, 1.0), (1, 1.0, 1.1)):
            got = oracle.choose_split(t_p, t_d, t_s, tpm, tdm, pol, a, b)
            if pol == 2:
                want = int(np.argmin(t_s))
            else:
                obj, con, bound = (t_p, t_d, np.float64(np.float32(b)) * np.float32(tdm)) if pol == 0 else \
                                  (t_d, t_p, np.float64(np.float32(a)) * np.float32(tpm))
                ok = [i for i in range(n) if con[i] <= bound]
                want = min(ok, key=lambda i: (obj[i], i)) if ok else min(range(n), key=lambda i: (con[i], i))
            assert got == want

"""CPU oracle of the decoder layer evaluated by the partitioned prefill/decode step.

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import this package; the product path never does.
The arithmetic lives in ``nexus_oracle.c`` (plain C, fp32 storage, fp64
reductions); this module compiles it with gcc and exposes it through ctypes
with numpy arrays.  Nothing here is shared with the HIP path.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nexus_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None
# The mutation tests point this at a deliberately broken build to show that the pins notice.
_LIB_OVERRIDE = os.environ.get("NEXUS_ORACLE_LIB_OVERRIDE")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over tokens/heads)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-fvisibility=hidden",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Model(C.Structure):
    _fields_ = [("hidden", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("ffn", C.c_int32), ("page_size", C.c_int32),
                ("rms_eps", C.c_float), ("rope_theta", C.c_float)]


class _Weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("attn_norm_g", "w_qkv", "b_qkv", "w_o", "ffn_norm_g", "w_gate_up", "w_down")]


@dataclass
class Model:
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    page_size: int = 16
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0

    def c(self) -> _Model:
        return _Model(self.hidden, self.n_q_heads, self.n_kv_heads, self.head_dim, self.ffn,
                      self.page_size, self.rms_eps, self.rope_theta)


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_LIB_OVERRIDE) if _LIB_OVERRIDE else C.CDLL(build())
        _lib.oracle_num_threads.restype = C.c_int
        _lib.oracle_choose_split.restype = C.c_int
    return _lib


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def num_threads() -> int:
    return lib().oracle_num_threads()


def set_num_threads(n: int) -> None:
    lib().oracle_set_num_threads(C.c_int(n))


def rmsnorm(x, g, eps: float) -> np.ndarray:
    x, g = _f32(x), _f32(g)
    T, d = x.shape
    out = np.empty_like(x)
    lib().oracle_rmsnorm(_p(x), _p(g), C.c_int(T), C.c_int(d), C.c_float(eps), _p(out))
    return out


def linear(x, W, b=None) -> np.ndarray:
    x, W = _f32(x), _f32(W)
    b = None if b is None else _f32(b)
    T, n_in = x.shape
    n_out = W.shape[0]
    assert W.shape[1] == n_in
    y = np.empty((T, n_out), np.float32)
    lib().oracle_linear(_p(x), _p(W), _p(b), C.c_int(T), C.c_int(n_in), C.c_int(n_out), _p(y))
    return y


def rope(u, pos: int, theta: float) -> np.ndarray:
    """u: [n_heads, hd]; returns the rotated copy."""
    u = _f32(u).copy()
    n_heads, hd = u.shape
    lib().oracle_rope(_p(u), C.c_int(n_heads), C.c_int(hd), C.c_int(pos), C.c_float(theta))
    return u


def kv_slot(page_table_row, pos: int, page_size: int):
    row = _i32(page_table_row)
    page, slot = C.c_int32(), C.c_int32()
    lib().oracle_kv_slot(_p(row), C.c_int(pos), C.c_int(page_size), C.byref(page), C.byref(slot))
    return page.value, slot.value


def kv_append(m: Model, k_pool, v_pool, page_table_row, pos: int, k, v) -> None:
    """k_pool/v_pool: float32 [n_pages, Hkv, page_size, hd], modified in place."""
    assert k_pool.dtype == np.float32 and k_pool.flags.c_contiguous
    assert v_pool.dtype == np.float32 and v_pool.flags.c_contiguous
    row, k, v = _i32(page_table_row), _f32(k), _f32(v)
    cm = m.c()
    lib().oracle_kv_append(C.byref(cm), _p(k_pool), _p(v_pool), _p(row), C.c_int(pos), _p(k), _p(v))


def kv_gather(m: Model, k_pool, v_pool, page_table_row, length: int):
    row = _i32(page_table_row)
    k = np.empty((length, m.n_kv_heads, m.head_dim), np.float32)
    v = np.empty_like(k)
    cm = m.c()
    lib().oracle_kv_gather(C.byref(cm), _p(_f32(k_pool)), _p(_f32(v_pool)), _p(row), C.c_int(length), _p(k), _p(v))
    return k, v


def attention_contig(m: Model, q, pos: int, K, V, want_p: bool = False):
    """q: [Hq, hd]; K, V: [>= pos+1, Hkv, hd]."""
    q, K, V = _f32(q), _f32(K), _f32(V)
    a = np.empty((m.n_q_heads, m.head_dim), np.float32)
    p = np.empty((m.n_q_heads, pos + 1), np.float32) if want_p else None
    cm = m.c()
    lib().oracle_attention_contig(C.byref(cm), _p(q), C.c_int(pos), _p(K), _p(V), _p(a), _p(p))
    return (a, p) if want_p else a


def attention_paged(m: Model, q, pos: int, k_pool, v_pool, page_table_row, want_p: bool = False):
    q, k_pool, v_pool, row = _f32(q), _f32(k_pool), _f32(v_pool), _i32(page_table_row)
    a = np.empty((m.n_q_heads, m.head_dim), np.float32)
    p = np.empty((m.n_q_heads, pos + 1), np.float32) if want_p else None
    cm = m.c()
    lib().oracle_attention_paged(C.byref(cm), _p(q), C.c_int(pos), _p(k_pool), _p(v_pool), _p(row), _p(a), _p(p))
    return (a, p) if want_p else a


def swiglu(gu, F: int) -> np.ndarray:
    gu = _f32(gu)
    T = gu.shape[0]
    act = np.empty((T, F), np.float32)
    lib().oracle_swiglu(_p(gu), C.c_int(T), C.c_int(F), _p(act))
    return act


def _weights(w: dict):
    keep = {k: (None if w.get(k) is None else _f32(w[k])) for k in
            ("attn_norm_g", "w_qkv", "b_qkv", "w_o", "ffn_norm_g", "w_gate_up", "w_down")}
    cw = _Weights(*[None if keep[k] is None else keep[k].ctypes.data for k in
                    ("attn_norm_g", "w_qkv", "b_qkv", "w_o", "ffn_norm_g", "w_gate_up", "w_down")])
    return cw, keep


def layer_prefill(m: Model, w: dict, x, cu_chunk, prefix_len, page_table, k_pool, v_pool, debug: bool = False):
    """One layer over a chunked-prefill sub-batch.  Pools (float32, canonical layout) are updated in place.

    Returns y [T, hidden]; with debug=True also a dict with q (rotated), attn and x1.
    """
    assert k_pool.dtype == np.float32 and k_pool.flags.c_contiguous
    assert v_pool.dtype == np.float32 and v_pool.flags.c_contiguous
    x, cu, pl, pt = _f32(x), _i32(cu_chunk), _i32(prefix_len), _i32(page_table)
    n_reqs = len(pl)
    T = int(cu[n_reqs])
    assert x.shape == (T, m.hidden)
    qd = m.n_q_heads * m.head_dim
    y = np.empty((T, m.hidden), np.float32)
    dbg = {"q": np.empty((T, qd), np.float32), "attn": np.empty((T, qd), np.float32),
           "x1": np.empty((T, m.hidden), np.float32)} if debug else {}
    cw, keep = _weights(w)
    cm = m.c()
    lib().oracle_layer_prefill(C.byref(cm), C.byref(cw), _p(x), C.c_int(n_reqs), _p(cu), _p(pl), _p(pt),
                               C.c_int(pt.shape[1]), _p(k_pool), _p(v_pool), _p(y),
                               _p(dbg.get("q")), _p(dbg.get("attn")), _p(dbg.get("x1")))
    del keep
    return (y, dbg) if debug else y


def layer_prefill_rows(m: Model, w: dict, x, cu_chunk, prefix_len, page_table, k_pool, v_pool, rows,
                       kv_store_bf16: bool = False):
    """The chunked-prefill phase for the listed batch rows only: every token's K/V is appended (pools updated in
    place), then the query projection, the attention and the rest of the layer run for `rows`.  Returns
    [len(rows), hidden], row i being row rows[i] of layer_prefill's result.  kv_store_bf16 rounds the appended K/V
    to bf16 as a bf16 cache would (a measurement of that format's cost; parity gates use the exact default)."""
    assert k_pool.dtype == np.float32 and k_pool.flags.c_contiguous
    assert v_pool.dtype == np.float32 and v_pool.flags.c_contiguous
    x, cu, pl, pt, rows = _f32(x), _i32(cu_chunk), _i32(prefix_len), _i32(page_table), _i32(rows)
    n_reqs = len(pl)
    T = int(cu[n_reqs])
    assert x.shape == (T, m.hidden)
    assert rows.ndim == 1 and (rows >= 0).all() and (rows < T).all()
    y = np.empty((len(rows), m.hidden), np.float32)
    cw, keep = _weights(w)
    cm = m.c()
    lib().oracle_layer_prefill_rows(C.byref(cm), C.byref(cw), _p(x), C.c_int(n_reqs), _p(cu), _p(pl), _p(pt),
                                    C.c_int(pt.shape[1]), _p(k_pool), _p(v_pool), C.c_int(len(rows)), _p(rows),
                                    C.c_int(int(kv_store_bf16)), _p(y))
    del keep
    return y


def layer_decode(m: Model, w: dict, x, ctx_len, page_table, k_pool, v_pool, debug: bool = False):
    """One layer over a decode sub-batch: request j's new token sits at position ctx_len[j]."""
    assert k_pool.dtype == np.float32 and k_pool.flags.c_contiguous
    assert v_pool.dtype == np.float32 and v_pool.flags.c_contiguous
    x, cl, pt = _f32(x), _i32(ctx_len), _i32(page_table)
    n = len(cl)
    assert x.shape == (n, m.hidden)
    qd = m.n_q_heads * m.head_dim
    y = np.empty((n, m.hidden), np.float32)
    dbg = {"q": np.empty((n, qd), np.float32), "attn": np.empty((n, qd), np.float32),
           "x1": np.empty((n, m.hidden), np.float32)} if debug else {}
    cw, keep = _weights(w)
    cm = m.c()
    lib().oracle_layer_decode(C.byref(cm), C.byref(cw), _p(x), C.c_int(n), _p(cl), _p(pt), C.c_int(pt.shape[1]),
                              _p(k_pool), _p(v_pool), _p(y), _p(dbg.get("q")), _p(dbg.get("attn")),
                              _p(dbg.get("x1")))
    del keep
    return (y, dbg) if debug else y


def choose_split(t_p, t_d, t_step, t_p_min: float, t_d_min: float, policy: int, alpha: float, beta: float) -> int:
    t_p, t_d, t_step = _f32(t_p), _f32(t_d), _f32(t_step)
    return lib().oracle_choose_split(C.c_int(len(t_p)), _p(t_p), _p(t_d), _p(t_step), C.c_float(t_p_min),
                                     C.c_float(t_d_min), C.c_int(policy), C.c_float(alpha), C.c_float(beta))

"""Helpers shared by the GPU parity tests: run a workload through the CPU oracle and through the HIP library, and
compare to the stated bar (|gpu - ref| <= 2e-2 + 2e-2 |ref| elementwise, relative L2 <= 1e-2 per layer output;
integer / index work bit-exact)."""
from __future__ import annotations

import numpy as np
import torch

ATOL, RTOL, REL_L2 = 2e-2, 2e-2, 1e-2


def f32(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy()


def oracle_model(oracle, shape):
    return oracle.Model(hidden=shape.hidden, n_q_heads=shape.n_q_heads, n_kv_heads=shape.n_kv_heads,
                        head_dim=shape.head_dim, ffn=shape.ffn, page_size=shape.page_size, rms_eps=shape.rms_eps,
                        rope_theta=shape.rope_theta)


def oracle_weights(w):
    return {k: (None if v is None else f32(v)) for k, v in w.items()}


def run_oracle(oracle, wl, weights, do_prefill=True, do_decode=True, debug=False):
    """Both sub-batches of one layer on the CPU oracle; returns outputs and the updated canonical pools (fp32)."""
    m = oracle_model(oracle, wl.shape)
    ow = oracle_weights(weights)
    kp, vp = f32(wl.k_pool).copy(), f32(wl.v_pool).copy()
    out = {}
    if do_prefill and wl.prefill is not None:
        p = wl.prefill
        r = oracle.layer_prefill(m, ow, f32(p.x), p.cu_chunk, p.prefix_len, p.page_table, kp, vp, debug=debug)
        out["y_p"], out["dbg_p"] = (r if debug else (r, None))
    if do_decode and wl.decode is not None:
        d = wl.decode
        r = oracle.layer_decode(m, ow, f32(d.x), d.ctx_len, d.page_table, kp, vp, debug=debug)
        out["y_d"], out["dbg_d"] = (r if debug else (r, None))
    out["k_pool"], out["v_pool"] = kp, vp
    return out


def expected_touched(wl, do_prefill=True, do_decode=True) -> np.ndarray:
    """Boolean [n_pages, page_size]: the (page, slot) pairs the step must write -- pure integer paging arithmetic."""
    ps = wl.shape.page_size
    t = np.zeros((wl.n_pages, ps), bool)
    if do_prefill and wl.prefill is not None:
        p = wl.prefill
        for r in range(p.n_reqs):
            for pos in range(int(p.prefix_len[r]), int(p.prefix_len[r] + p.chunk_len[r])):
                t[p.page_table[r, pos // ps], pos % ps] = True
    if do_decode and wl.decode is not None:
        d = wl.decode
        for j in range(d.n_reqs):
            c = int(d.ctx_len[j])
            t[d.page_table[j, c // ps], c % ps] = True
    return t


def assert_close(name, got: np.ndarray, ref: np.ndarray):
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, f"{name}: shape {got.shape} vs {ref.shape}"
    assert np.isfinite(got).all(), f"{name}: non-finite values in the GPU result"
    err = np.abs(got - ref)
    bound = ATOL + RTOL * np.abs(ref)
    worst = np.unravel_index(np.argmax(err - bound), err.shape)
    assert (err <= bound).all(), (f"{name}: elementwise bar exceeded at {worst}: gpu {got[worst]:.6f} ref {ref[worst]:.6f} "
                                  f"(err {err[worst]:.4g} > {bound[worst]:.4g}); {int((err > bound).sum())} of {err.size} fail")
    rel = np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-30)
    assert rel <= REL_L2, f"{name}: relative L2 {rel:.4g} > {REL_L2}"
    print(f"[parity] {name}: worst err/bound {float((err / bound).max()):.3f}, rel L2 {rel:.2e}, n {err.size}", flush=True)
    return rel


def check_pools(name, wl, kv_gpu, ref, touched, before):
    """kv_gpu: (k, v) canonical bf16 tensors exported from the GPU after the step.
    Slots outside `touched` must be bit-identical to `before`; slots inside must match the oracle's values."""
    for which, g, r, b in (("K", kv_gpu[0], ref["k_pool"], before[0]), ("V", kv_gpu[1], ref["v_pool"], before[1])):
        gbits = g.cpu().view(torch.int16).numpy()
        bbits = b.cpu().view(torch.int16).numpy()
        changed = (gbits != bbits).any(axis=(1, 3))          # [pages, slots]
        # index work is exact: nothing outside the expected slots may change
        assert not (changed & ~touched).any(), f"{name}: {which} pool modified outside the appended slots"
        same = np.broadcast_to((~touched)[:, None, :, None], gbits.shape)
        assert np.array_equal(gbits[same], bbits[same]), f"{name}: {which} untouched slots not bit-identical"
        sel = np.broadcast_to(touched[:, None, :, None], gbits.shape)
        if sel.any():
            assert_close(f"{name} {which} appended", f32(g)[sel], r[sel])
            # every expected slot was really written (random N(0,1) contents cannot coincide on a whole slot)
            assert (changed | ~touched).all(), f"{name}: {which} an expected slot was not written"

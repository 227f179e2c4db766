"""Sec. 3.3 (Fig. 5) on this chip: the latency of an identical decode batch on a fixed partition while the chunk that
prefills next to it attends to more and more cached keys.  The decode phase runs as its own loop (Sec. 5), step after
step, for as long as the chunk is in flight; the mean latency of those steps is the figure.  The same points go
through the calibrated latency model (Eq. 5-9), whose decode-side contention term is what Sec. 3.3 motivates.
The paper measures +36 % from 2000 to 10000 keys on its GPU; what this chip does is measured, printed and compared
with the model's direction rather than assumed."""
import numpy as np
import pytest
import torch

from paper_2507_06608_amd import synth

pytestmark = pytest.mark.gpu

SPLIT = (128, 128)
KV_LENGTHS = (2000, 4000, 6000, 8000, 10000)     # keys the 512-token chunk attends to (prefix + chunk)
CHUNK = 512


@pytest.fixture(scope="module")
def nx():
    from paper_2507_06608_amd import binding
    binding.lib()
    assert torch.cuda.is_available()
    return binding


def test_decode_latency_against_kv_length_of_the_co_running_prefill(nx):
    print("[case] decode latency vs KV length of the co-running prefill, split %d/%d" % SPLIT, flush=True)
    sh = synth.SHAPES["llama3_8b"]
    rng = np.random.default_rng(33)
    ctxs = rng.integers(512, 4097, size=64).tolist()
    wl = synth.make_workload("contention", sh, 33, chunk_lens=[CHUNK], prefix_lens=[KV_LENGTHS[-1] - CHUNK], decode_ctx=ctxs,
                             kv_device="cuda:0")
    ctx = nx.context_for(wl)
    ctx.load_layer(0, synth.make_weights(sh, 33))
    kv = ctx.make_kv(wl.k_pool, wl.v_pool)
    db = nx.DevDecode(wl.decode, ctx.device)
    p = wl.prefill
    batches = {L: nx.DevPrefill(synth.PrefillBatch(p.x, p.cu_chunk, np.array([L - CHUNK], np.int32), p.page_table), ctx.device)
               for L in KV_LENGTHS}
    ctx.set_cu_split(*SPLIT)

    def decode_alone(n=30):
        out = []
        for _ in range(n):
            ctx.decode_step(db, kv)
            out.append(ctx.phase_wait(nx.PHASE_DECODE))
        return float(np.median(out[5:]))

    def decode_next_to(pb, chunks=12):
        lat, per_chunk, t_chunk = [], [], []
        for c in range(chunks):
            ctx.prefill_chunk(pb, kv)
            n = 0
            while not ctx.phase_done(nx.PHASE_PREFILL):
                ctx.decode_step(db, kv)
                ms = ctx.phase_wait(nx.PHASE_DECODE)
                if not ctx.phase_done(nx.PHASE_PREFILL) and c >= 2:       # steps that ran wholly inside the chunk
                    lat.append(ms)
                n += 1
            t_chunk.append(ctx.phase_wait(nx.PHASE_PREFILL))
            per_chunk.append(n)
        return float(np.mean(lat)), float(np.median(t_chunk[2:])), float(np.mean(per_chunk[2:])), len(lat)

    base = decode_alone()
    print(f"[contention] decode step alone on {SPLIT[1]} CUs: {base:.3f} ms", flush=True)
    rows = []
    for L in KV_LENGTHS:
        lat, t_chunk, steps, n = decode_next_to(batches[L])
        rows.append((L, lat, t_chunk, steps))
        print(f"[contention] chunk attends to {L:5d} keys: decode step {lat:.3f} ms ({lat / base:.3f} of alone, {n} steps timed), "
              f"chunk {t_chunk:.3f} ms, {steps:.1f} decode steps per chunk", flush=True)
    lat = [r[1] for r in rows]
    print(f"[contention] decode latency at {KV_LENGTHS[-1]} keys / at {KV_LENGTHS[0]} keys: {lat[-1] / lat[0]:.3f} "
          f"(the paper's GPU: 1.36)", flush=True)
    # A decode step next to prefill is never faster than alone (margin for run-to-run noise), and the interference is
    # a two-digit percentage.  WHICH WAY it moves with the chunk's KV length is a property of the chip, reported here
    # and compared with the model below: on the paper's GPU the chunk's attention is the memory-hungry part and a
    # longer KV slows decode (+36 %); on MI355X the chunk's attention runs out of L2 (8-41 MB of K/V, re-read by every
    # query strip) while its GEMMs stream 436 MB of weights, so the more of the chunk is attention, the LESS it takes
    # from the decode stream -- m_p1 < m_p2 in Eq. 9.
    assert min(lat) > 0.97 * base
    assert max(lat) > 1.05 * base, "no interference measured at all: the phases did not overlap?"
    assert max(lat) < 1.6 * base
    measured_trend = lat[-1] / lat[0]

    # the same points through the latency model calibrated on this machine (phases alone at 8 shares)
    from paper_2507_06608_amd.calibrate import calibrate
    d = wl.decode
    kv_d = float((d.ctx_len + 1).sum())
    mid = KV_LENGTHS[len(KV_LENGTHS) // 2]

    def describe(L):
        pairs = float(CHUNK * (L - CHUNK) + CHUNK * (CHUNK + 1) // 2)
        return nx.cost_describe(sh, 1, CHUNK, pairs, float(L), d.n_reqs, kv_d)
    alg_p, alg_d = describe(mid)
    cal = calibrate(ctx, kv, batches[mid], db, alg_p, alg_d)
    ctx.set_cu_split(*SPLIT)
    share = SPLIT[1] // 8
    model_ms = []
    for L in KV_LENGTHS:
        a_p, a_d = describe(L)
        model_ms.append(cal.model(a_p, a_d).latency(nx.PHASE_DECODE, share, 32) * 1e3)
    print("[contention] keys:             " + " ".join(f"{L:7d}" for L in KV_LENGTHS))
    print("[contention] measured ms:      " + " ".join(f"{t:7.3f}" for t in lat))
    print("[contention] modelled ms:      " + " ".join(f"{t:7.3f}" for t in model_ms), flush=True)
    for L, a, b in zip(KV_LENGTHS, model_ms, lat):
        assert a == pytest.approx(b, rel=0.25), ("modelled decode latency", L)
    model_trend = model_ms[-1] / model_ms[0]
    print(f"[contention] trend {KV_LENGTHS[0]} -> {KV_LENGTHS[-1]} keys: measured {measured_trend:.3f}, modelled {model_trend:.3f}", flush=True)
    # Eq. 8-9 with this chip's byte counts move the same way as the measurement (or both are flat within 3 %)
    assert (measured_trend - 1.0) * (model_trend - 1.0) > 0 or (abs(measured_trend - 1.0) < 0.03 and abs(model_trend - 1.0) < 0.03) \
        or abs(measured_trend - model_trend) < 0.08, (measured_trend, model_trend)
    ctx.close()

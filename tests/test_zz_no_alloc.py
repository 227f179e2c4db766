"""The decode step that allocates nothing (its workspace is a static device array of the library), through the C
ABI, against the ordinary decode step: identical bits, on two calls in a row, the second with a smaller batch;
plus the size limit."""
import numpy as np
import pytest
import torch

from paper_2507_06608_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def nx():
    from paper_2507_06608_amd import binding
    binding.lib()
    assert torch.cuda.is_available()
    return binding


def _bits(t):
    return t.view(torch.int16)


@pytest.mark.parametrize("shape,ctx_lens,seed", [("tiny", [200, 17, 64, 255, 256, 0, 31, 100], 21),
                                                 ("llama3_8b", [3000, 512, 4095, 17, 1024, 2047, 2048, 100, 999, 1, 4000, 77], 22)],
                         ids=["tiny", "8B-shaped"])
def test_noalloc_decode_step_equals_decode_step_twice_in_a_row(nx, shape, ctx_lens, seed):
    print(f"[case] no-alloc decode step, {shape}", flush=True)
    sh = synth.SHAPES[shape]
    wl = synth.make_workload("noalloc", sh, seed, chunk_lens=[], prefix_lens=[], decode_ctx=ctx_lens, kv_device="cuda:0")
    w = synth.make_weights(sh, seed)
    ctx = nx.context_for(wl)
    ctx.load_layer(0, w)
    small = synth.DecodeBatch(wl.decode.x[2:5], wl.decode.ctx_len[2:5], wl.decode.page_table[2:5])
    for batch in (wl.decode, small):                      # second call: smaller input, same static array
        outs = []
        for call in (ctx.decode_step, ctx.decode_step_noalloc):
            kv = ctx.make_kv(wl.k_pool, wl.v_pool)
            db = nx.DevDecode(batch, ctx.device)
            db.y.fill_(float("nan"))
            torch.cuda.synchronize()
            call(db, kv)
            ctx.sync()
            outs.append((db.y.clone(), ctx.kv_export(kv)))
        (y0, kv0), (y1, kv1) = outs
        assert torch.isfinite(y1.float()).all()
        assert torch.equal(_bits(y0), _bits(y1)), f"{batch.n_reqs} requests: outputs differ"
        for a, b in zip(kv0, kv1):
            assert torch.equal(_bits(a), _bits(b)), f"{batch.n_reqs} requests: caches differ"
    # back to back without a sync in between, alternating with the ordinary call on the same stream
    kv = ctx.make_kv(wl.k_pool, wl.v_pool)
    db, ds = nx.DevDecode(wl.decode, ctx.device), nx.DevDecode(small, ctx.device)
    ctx.decode_step_noalloc(db, kv)
    ctx.decode_step_noalloc(ds, kv)
    ctx.decode_step(db, kv)
    ctx.decode_step_noalloc(db, kv)
    ctx.sync()
    assert torch.equal(_bits(db.y), _bits(y_full(ctx, nx, wl)))
    ctx.close()


def y_full(ctx, nx, wl):
    kv = ctx.make_kv(wl.k_pool, wl.v_pool)
    db = nx.DevDecode(wl.decode, ctx.device)
    ctx.decode_step(db, kv)
    ctx.sync()
    return db.y.clone()


def test_noalloc_decode_step_two_layers_and_a_partitioned_layout(nx):
    print("[case] no-alloc decode step, two layers on a 64-CU share", flush=True)
    sh = synth.SHAPES["tiny"]
    wl = synth.make_workload("noalloc2", sh, 23, chunk_lens=[], prefix_lens=[], decode_ctx=[50, 20, 129], kv_device="cuda:0")
    ctx = nx.context_for(wl, n_layers=2)
    for l in range(2):
        ctx.load_layer(l, synth.make_weights(sh, 23, layer=l))
    ctx.set_cu_split(192, 64)
    outs = []
    for call in (ctx.decode_step, ctx.decode_step_noalloc):
        kv = ctx.make_kv(wl.k_pool, wl.v_pool, layers=2)
        db = nx.DevDecode(wl.decode, ctx.device)
        call(db, kv, layers=(0, 2))
        ctx.sync()
        outs.append((db.y.clone(), ctx.kv_export(kv, 1)))
    assert torch.equal(_bits(outs[0][0]), _bits(outs[1][0]))
    for a, b in zip(outs[0][1], outs[1][1]):
        assert torch.equal(_bits(a), _bits(b))
    ctx.close()


def test_noalloc_decode_step_rejects_what_does_not_fit(nx):
    print("[case] no-alloc decode step, size limit", flush=True)
    sh = synth.SHAPES["llama3_8b"]
    n, c = 256, 8191
    wl = synth.make_workload("too big", sh, 24, chunk_lens=[], prefix_lens=[], decode_ctx=[c] * n, kv_device="cuda:0")
    ctx = nx.context_for(wl)
    ctx.load_layer(0, synth.make_weights(sh, 24))
    kv = ctx.make_kv(wl.k_pool, wl.v_pool)
    db = nx.DevDecode(wl.decode, ctx.device)
    db.y.zero_()
    torch.cuda.synchronize()
    with pytest.raises(nx.NexusError, match="static scratch array"):
        ctx.decode_step_noalloc(db, kv)
    ctx.sync()
    assert not db.y.any(), "a rejected call must launch nothing"
    ctx.decode_step(db, kv)          # the ordinary call takes the same batch
    ctx.sync()
    assert torch.isfinite(db.y.float()).all()
    ctx.close()

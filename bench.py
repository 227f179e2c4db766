#!/usr/bin/env python3
"""Benchmark of the partitioned prefill/decode step on one MI355X.

A "step" is one pass of the whole hot path over one batch: a chunked-prefill sub-batch and a decode sub-batch through
every layer of the stack, run concurrently on disjoint CU partitions (or back to back for the serialized baseline).

Headline workload (the largest single-GPU configuration): the Llama-3-70B-shaped stack at full depth, 80 layers
resident (~137 GB of packed weights drawn on the device + ~55 GB of KV), a 2048-token chunk over a 2048-token prefix
next to 64 decode requests with contexts uniform in [1024, 4096]; seeded, synthetic, resident in HBM before the timed
region.  The 8B-shaped single-layer configurations (512-token chunk + 64 decodes; 4 x 2048-token chunks + 256 decodes)
ride along as `secondary` objects of the same JSON line.

Prints ONE JSON line: mixed-step tokens/s at the chosen CU split, the sweep over splits with decode-step latency,
the serialized baseline, the roofline of the dominant kernel and the CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_TFLOPS = 2500.0   # MI355X dense fp16 / bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E
# what actually runs: storage and arithmetic types of the path
DTYPE = "bf16 storage (x, y, KV cache, queries); fp16 GEMM operands; bf16 attention MFMA; fp32 accumulate"


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_work(wl, layers):
    """Flops / bytes the method itself must do per launch of each kernel family (one layer), and per step."""
    s = wl.shape
    p, d = wl.prefill, wl.decode
    T, B = p.n_tokens, d.n_reqs
    kv_tok_bytes = 2 * s.n_kv_heads * s.head_dim * 2
    pairs = sum(int(n) * int(pre) + int(n) * (int(n) + 1) // 2 for n, pre in zip(p.chunk_len, p.prefix_len))
    w = {
        "gemm_qkv": 2.0 * T * s.n_qkv * s.hidden,
        "gemm_o": 2.0 * T * s.hidden * s.q_dim,
        "gemm_gate_up": 2.0 * T * 2 * s.ffn * s.hidden,
        "gemm_down": 2.0 * T * s.hidden * s.ffn,
        "attn_prefill": 4.0 * s.head_dim * s.n_q_heads * pairs,
    }
    decode_kv_bytes = float(sum(int(c) + 1 for c in d.ctx_len)) * kv_tok_bytes
    weight_bytes = 2.0 * s.params_per_layer
    decode_bytes = {
        "attn_decode": decode_kv_bytes,
        "gemm_qkv": 2.0 * s.n_qkv * s.hidden, "gemm_o": 2.0 * s.hidden * s.q_dim,
        "gemm_gate_up": 2.0 * 2 * s.ffn * s.hidden, "gemm_down": 2.0 * s.hidden * s.ffn,
    }
    # operand bytes of the prefill kernels (weights once + activations in + result out), for the traffic ratio only
    prefill_bytes = {
        "gemm_qkv": 2.0 * s.n_qkv * s.hidden + 2.0 * T * (s.hidden + s.n_qkv),
        "gemm_o": 2.0 * s.hidden * s.q_dim + 2.0 * T * s.q_dim + 4.0 * T * s.hidden,
        "gemm_gate_up": 2.0 * 2 * s.ffn * s.hidden + 2.0 * T * (s.hidden + s.ffn),
        "gemm_down": 2.0 * s.hidden * s.ffn + 2.0 * T * (s.ffn + s.hidden),
        "attn_prefill": float(sum(int(n) + int(pre) for n, pre in zip(p.chunk_len, p.prefix_len))) * kv_tok_bytes
                        + 2.0 * 2 * T * s.q_dim,
    }
    return {"prefill_flops": w, "prefill_layer_flops": sum(w.values()), "decode_bytes": decode_bytes, "prefill_bytes": prefill_bytes,
            "decode_layer_bytes": decode_kv_bytes + weight_bytes, "tokens": T + B, "layers": layers}


def cpu_baseline(wl, weights, layers, n_prefill_tokens, n_decode, reps):
    """The oracle as it stands, on the host cores, on a bounded sample of the same workload: the first tokens of the
    first chunk (they see the whole cached prefix) and the first decode requests, ONE layer; the rate is then divided
    by the number of layers of the stack, which the oracle would run one after the other."""
    import numpy as np

    import oracle
    from paper_2507_06608_amd import synth
    p = wl.prefill
    sub = synth.subset_for_oracle(wl, [0], list(range(min(n_decode, wl.decode.n_reqs))))
    n = min(n_prefill_tokens, int(p.chunk_len[0]))
    sp = sub.prefill
    sp = synth.PrefillBatch(sp.x[:n], np.array([0, n], np.int32), sp.prefix_len[:1], sp.page_table[:1])
    m = oracle.Model(hidden=wl.shape.hidden, n_q_heads=wl.shape.n_q_heads, n_kv_heads=wl.shape.n_kv_heads,
                     head_dim=wl.shape.head_dim, ffn=wl.shape.ffn, page_size=wl.shape.page_size,
                     rms_eps=wl.shape.rms_eps, rope_theta=wl.shape.rope_theta)
    ow = {k: v.float().cpu().numpy() for k, v in weights.items()}
    kp, vp = sub.k_pool.float().numpy().copy(), sub.v_pool.float().numpy().copy()
    oracle.lib()
    t0 = time.perf_counter()
    for _ in range(reps):
        oracle.layer_prefill(m, ow, sp.x.float().numpy(), sp.cu_chunk, sp.prefix_len, sp.page_table, kp, vp)
        oracle.layer_decode(m, ow, sub.decode.x.float().numpy(), sub.decode.ctx_len, sub.decode.page_table, kp, vp)
    dt = time.perf_counter() - t0
    toks = reps * (n + sub.decode.n_reqs)
    return {"value": toks / dt / layers, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"{n} of {p.n_tokens} prefill tokens (over the full {int(p.prefix_len[0])}-token prefix) + "
                      f"{sub.decode.n_reqs} of {wl.decode.n_reqs} decode requests through ONE layer, {reps} pass(es), {dt:.1f} s of "
                      f"CPU work; tokens/s of that layer divided by the {layers} layers of the stack"}


def device_layer_weights(shape, layer, std):
    """One layer's bf16 weights drawn on the GPU (a host copy of the 70B-shaped stack's 137 GB is avoided)."""
    import torch
    g = torch.Generator(device="cuda:0")
    g.manual_seed(1000 + layer)

    def mat(r, c):
        return (torch.randn((r, c), generator=g, device="cuda:0") * std).to(torch.bfloat16)

    def gain():
        return (1.0 + torch.randn(shape.hidden, generator=g, device="cuda:0") * 0.02).to(torch.bfloat16)
    return {"attn_norm_g": gain(), "w_qkv": mat(shape.n_qkv, shape.hidden), "w_o": mat(shape.hidden, shape.q_dim),
            "ffn_norm_g": gain(), "w_gate_up": mat(2 * shape.ffn, shape.hidden), "w_down": mat(shape.hidden, shape.ffn)}


def load_traffic(name):
    """HBM bytes per launch from the committed rocprofv3 FETCH_SIZE / WRITE_SIZE summaries (scaled by a copy of known
    size; see the files): bench.py cannot run the profiler on itself, so it reports what those runs measured."""
    traffic = {}
    prof_dir = os.path.join(ROOT, "profiles")
    if os.path.isdir(prof_dir):
        for fn in sorted(os.listdir(prof_dir)):
            if fn.startswith("hbm_traffic_"):
                for line in open(os.path.join(prof_dir, fn)):
                    f = line.split()
                    if len(f) == 4 and f[0] == "traffic_bytes_per_launch" and f[1] == name:
                        traffic[f[2]] = {"bytes_per_launch": float(f[3]), "source": "profiles/" + fn}
    return traffic


def continuous_decode(ctx, binding, wl, pb, db, kv, layers, split, n_chunks=3):
    """The two phases as independent loops (Sec. 5): prefill chunks back to back on the prefill share while decode steps
    run back to back on the decode share; and, on all CUs, the temporal schedule that reaches the same time between
    decode steps by slicing the chunk (a decode step, then k layers of the chunk, and so on).  Tokens per second of
    each over the time the chunks take."""
    import copy

    import torch
    L = (0, layers)
    tokens_p, tokens_d = wl.prefill.n_tokens, wl.decode.n_reqs
    ctx.set_cu_split(*split)
    ctx.mixed_step(pb, db, kv, layers=L)
    ctx.sync()
    t0 = time.perf_counter()
    for _ in range(n_chunks):
        ctx.prefill_chunk(pb, kv, layers=L)
    steps, t_steps = 0, []
    while not ctx.phase_done(binding.PHASE_PREFILL):
        ctx.decode_step(db, kv, layers=L)
        t_steps.append(ctx.phase_wait(binding.PHASE_DECODE))
        steps += 1
    ctx.sync()
    window = time.perf_counter() - t0
    tbt = window / steps * 1e3
    spatial = {"cu_split": f"{split[0]}/{split[1]}", "prefill_chunks": n_chunks, "decode_steps": steps, "window_ms": window * 1e3,
               "time_between_decode_steps_ms": tbt, "decode_step_ms": float(sum(t_steps) / len(t_steps)),
               "tokens_per_s": (n_chunks * tokens_p + steps * tokens_d) / window}
    # temporal schedule on all CUs at (about) the same time between decode steps
    ctx.set_cu_split(binding.CUS_ALL, binding.CUS_ALL)
    ctx.decode_step(db, kv, layers=L)
    t_dec = ctx.phase_wait(binding.PHASE_DECODE)
    ctx.prefill_chunk(pb, kv, layers=L)
    t_layer = ctx.phase_wait(binding.PHASE_PREFILL) / layers
    k = max(1, min(layers, int(round((tbt - t_dec) / t_layer))))
    bufs = [torch.empty_like(pb.y), torch.empty_like(pb.y)]
    ctx.sync()
    t0 = time.perf_counter()
    steps_t = 0
    for _ in range(n_chunks):
        src = pb.x
        for i, a in enumerate(range(0, layers, k)):
            b = min(layers, a + k)
            ctx.decode_step(db, kv, layers=L)
            steps_t += 1
            part = copy.copy(pb)
            part.c = binding.PrefillBatchC.from_buffer_copy(pb.c)
            dst = pb.y if b == layers else bufs[i & 1]
            part.c.x, part.c.y = src.data_ptr(), dst.data_ptr()
            ctx.prefill_chunk(part, kv, layers=(a, b))
            src = dst
    ctx.sync()
    window_t = time.perf_counter() - t0
    temporal = {"layers_per_slice": k, "prefill_chunks": n_chunks, "decode_steps": steps_t, "window_ms": window_t * 1e3,
                "time_between_decode_steps_ms": window_t / steps_t * 1e3,
                "tokens_per_s": (n_chunks * tokens_p + steps_t * tokens_d) / window_t}
    return {"independent_loops": spatial, "temporal_slices_all_cus": temporal,
            "tokens_per_s_ratio": spatial["tokens_per_s"] / temporal["tokens_per_s"]}


def measure(idx, layers, steps, warmup, args, headline):
    """One configuration: serialized baseline, sweep of the split, timed steps at the chosen split, rooflines."""
    import numpy as np
    import torch

    from paper_2507_06608_amd import binding, synth
    dev = "cuda:0"
    t0 = time.time()
    wl = synth.config(idx, seed=0, kv_device=dev)
    s = wl.shape
    ctx = binding.context_for(wl, n_layers=layers)
    if layers == 1:
        first = synth.make_weights(s, 0)
        ctx.load_layer(0, first)
    else:
        first = None
        for l in range(layers):
            w = device_layer_weights(s, l, synth.weight_std(s))
            if l == 0:
                first = {k: v.clone() for k, v in w.items()}
            ctx.load_layer(l, w)
            del w
            if l % 20 == 19:
                log(f"[bench] {wl.name}: {l + 1} of {layers} layers packed")
    kv = ctx.make_kv(wl.k_pool, wl.v_pool, layers=layers)
    pb, db = binding.DevPrefill(wl.prefill, ctx.device), binding.DevDecode(wl.decode, ctx.device)
    work = algorithmic_work(wl, layers)
    n_cus = ctx.cu_count
    L = (0, layers)
    log(f"[bench] workload {wl.name} x {layers} layer(s): resident after {time.time() - t0:.1f} s")
    # No caller stream: the inputs are resident and complete before the loop starts, and the library itself orders
    # each step after both phases of the previous one, so steps do not overlap each other.

    hand = [None]    # handover layer of the prefill phase inside the step (None: the split is held to the end of the step)

    def one_step(timing=False):
        if hand[0] is None:
            return ctx.mixed_step(pb, db, kv, layers=L, timing=timing)
        return ctx.mixed_step_handover(pb, db, kv, hand[0], layers=L, timing=timing)

    def run_steps(n):
        for _ in range(n):
            one_step()

    def timed(n):
        torch.cuda.synchronize()
        t = time.perf_counter()
        run_steps(n)
        torch.cuda.synchronize()
        return (time.perf_counter() - t) / n * 1e3

    # ---- serialized baseline (one unmasked stream, prefill then decode)
    ctx.set_cu_split(binding.CUS_ALL, binding.CUS_ALL)
    run_steps(warmup)
    serial_ms = timed(max(3, steps // 4))
    tm = [ctx.mixed_step(pb, db, kv, layers=L, timing=True) for _ in range(3)][-1]
    serial = {"ms_per_step": serial_ms, "tokens_per_s": work["tokens"] / serial_ms * 1e3,
              "t_prefill_ms": tm.t_prefill_ms, "decode_latency_ms": tm.t_decode_ms}
    # the same two phases in the other order (decode step first, then the chunk; all CUs, one stream): the purely
    # temporal schedule with the short decode latency, for comparison with what the partition buys
    def decode_first():
        ctx.decode_step(db, kv, layers=L)
        ctx.prefill_chunk(pb, kv, layers=L)
    decode_first()
    torch.cuda.synchronize()
    n_df = max(3, steps // 4)
    t = time.perf_counter()
    for _ in range(n_df):
        decode_first()
    torch.cuda.synchronize()
    df_ms = (time.perf_counter() - t) / n_df * 1e3
    ctx.decode_step(db, kv, layers=L)
    serial["decode_first"] = {"ms_per_step": df_ms, "tokens_per_s": work["tokens"] / df_ms * 1e3,
                              "decode_latency_ms": ctx.phase_wait(binding.PHASE_DECODE)}
    log(f"[bench] {wl.name} serialized: {serial}")

    # ---- the engine without phase separation (the chunked-prefill engines the paper measures against): ONE batch,
    # every projection once over all rows (weights read once), chunk rows through the chunked-prefill attention,
    # decode rows through the decode attention; all CUs, one stream.  Single-layer configurations only: the fused
    # batch needs a context (and a packed weight copy) of its own.
    fused_res = None
    if layers == 1 and not args.no_fused:
        fused = synth.fused_single_batch(wl)
        fctx = binding.Nexus(s, max_prefill_tokens=fused.n_tokens, max_prefill_reqs=fused.n_reqs,
                             max_decode_reqs=wl.decode.n_reqs, max_positions=int((fused.prefix_len + fused.chunk_len).max()), n_layers=1)
        fctx.load_layer(0, first)
        fb = binding.DevPrefill(fused, fctx.device)
        max_ctx = int(wl.decode.ctx_len.max()) + 1
        for _ in range(warmup):
            fctx.fused_step(fb, wl.decode.n_reqs, max_ctx, kv)
        torch.cuda.synchronize()
        t = time.perf_counter()
        n_f = max(3, steps // 4)
        for _ in range(n_f):
            fctx.fused_step(fb, wl.decode.n_reqs, max_ctx, kv)
        torch.cuda.synchronize()
        fused_ms = (time.perf_counter() - t) / n_f * 1e3
        fused_res = {"ms_per_step": fused_ms, "tokens_per_s": work["tokens"] / fused_ms * 1e3, "decode_latency_ms": fused_ms}
        log(f"[bench] {wl.name} fused single batch: {fused_res}")
        fctx.close()
        del fb, fctx

    # ---- sweep of the CU split (steps of 32 CUs: shares in between leave a shader engine of every XCD a CU short and
    # run at the speed of the next lower multiple of 32)
    sweep, alone = [], {}
    if args.split == "auto":
        cands = [c for c in range(32, n_cus, 32)]
        prof = ctx.profile_split(pb, db, kv, cands, binding.POLICY_MIN_STEP, repeats=5 if layers == 1 else 3, layers=L)
        for i, c in enumerate(cands):
            sweep.append({"prefill_cus": c, "decode_cus": n_cus - c, "t_prefill_alone_ms": prof["t_prefill_ms"][i],
                          "t_decode_alone_ms": prof["t_decode_ms"][i], "t_step_ms": prof["t_step_ms"][i],
                          "tokens_per_s": work["tokens"] / prof["t_step_ms"][i] * 1e3})
        chosen = prof["chosen_prefill_cus"]
        alone = {"t_prefill_all_cus_ms": prof["t_prefill_all_ms"], "t_decode_all_cus_ms": prof["t_decode_all_ms"]}
        # the paper's two objectives on the same measured curves, for the record
        for name, pol in (("prefill_prioritized", binding.POLICY_PREFILL_PRIORITIZED),
                          ("decode_prioritized", binding.POLICY_DECODE_PRIORITIZED)):
            i = binding.choose_split(prof["t_prefill_ms"], prof["t_decode_ms"], prof["t_step_ms"],
                                     prof["t_prefill_all_ms"], prof["t_decode_all_ms"], pol, 1.3, 1.1)
            alone[name + "_prefill_cus"] = cands[i]
        best_ms = min(e["t_step_ms"] for e in sweep)
        if layers > 1 and not args.no_handover:
            # Sec. 4.2 inside a step: at each split, hand the decode share back to the prefill phase at the first layer
            # boundary after the decode step has ended (measured next to the prefill phase), and time that step too
            for e in sweep:
                ctx.set_cu_split(e["prefill_cus"], e["decode_cus"])
                t = ctx.mixed_step(pb, db, kv, layers=L, timing=True)
                h = min(layers, max(1, int(np.ceil(t.t_decode_ms / (t.t_prefill_ms / layers)))))
                ts = [ctx.mixed_step_handover(pb, db, kv, h, layers=L, timing=True) for _ in range(3)]
                e["handover_layer"] = h
                e["t_step_handover_ms"] = float(np.median([x.t_step_ms for x in ts]))
                e["decode_latency_handover_ms"] = float(np.median([x.t_decode_ms for x in ts]))
            # the shortest step wins; among steps within 1 % of it, the one with the shortest decode step
            t_min = min(best_ms, min(e["t_step_handover_ms"] for e in sweep))
            near = [e for e in sweep if e["t_step_handover_ms"] <= 1.01 * t_min]
            if near and t_min < best_ms:
                e = min(near, key=lambda e: e["decode_latency_handover_ms"])
                best_ms, chosen, hand[0] = e["t_step_handover_ms"], e["prefill_cus"], e["handover_layer"]
        log(f"[bench] {wl.name} sweep: {json.dumps(sweep)}")
        log(f"[bench] {wl.name} alone on all CUs: {alone}; chosen prefill CUs (min step): {chosen}" +
            (f", decode share handed to prefill at layer {hand[0]}" if hand[0] is not None else ""))
    else:
        a, b = (int(v) for v in args.split.split("/"))
        if a + b > n_cus:
            sys.exit(f"bench.py: split {a}/{b} exceeds the device's {n_cus} CUs")
        chosen = a
        if args.handover == "auto":
            # the library's own choice: its first step on a layout measures the two phases, the next ones use that
            ctx.set_cu_split(a, b)
            for _ in range(3):
                ctx.mixed_step_handover(pb, db, kv, binding.HANDOVER_AUTO, layers=L)
                ctx.sync()
            hand[0] = ctx.last_handover_layer()
            log(f"[bench] {wl.name} split {a}/{b}: the library hands the decode share over at layer {hand[0]}")
        elif args.handover != "":
            hand[0] = min(layers, max(0, int(args.handover)))
    d_cus = n_cus - chosen if args.split == "auto" else int(args.split.split("/")[1])
    ctx.set_cu_split(chosen, d_cus)
    # the sweep left a stream pair per split alive; queues beyond the GPU's hardware queues are time-multiplexed, and
    # with all of them alive back-to-back steps run 2-3 % slower: keep the chosen pair only
    ctx.retire_cu_splits()

    # ---- kernel times at this split (short traced passes), to find the dominant kernel of the step
    run_steps(max(1, warmup // 2))
    kt = {}
    traced = (("prefill", binding.PHASE_PREFILL, ("gemm_qkv", "attn_prefill", "gemm_o", "gemm_gate_up", "gemm_down")),
              ("decode", binding.PHASE_DECODE, ("gemm_qkv", "attn_decode", "gemm_o", "gemm_gate_up", "gemm_down")))
    n_tr = 3 if layers == 1 else 1
    for pname, phase, names in traced:
        for k in names:
            ctx.trace_begin(phase, k)
            run_steps(n_tr)
            ms, n = ctx.trace_read()
            kt[(pname, k)] = (ms, n / float(n_tr))
    log(f"[bench] {wl.name} kernel times at {chosen}/{d_cus} (ms per launch, launches per step): " +
        json.dumps({f"{a}.{b}": (round(v[0], 4), v[1]) for (a, b), v in kt.items()}))
    dom = max(kt, key=lambda k: kt[k][0] * kt[k][1])     # most time per step

    # ---- timed region: exactly `steps` steps, the dominant kernel bracketed by HIP events on its own stream
    ctx.trace_begin(binding.PHASE_PREFILL if dom[0] == "prefill" else binding.PHASE_DECODE, dom[1])
    ms_per_step = timed(steps)
    dom_ms, dom_n = ctx.trace_read()
    tms = [one_step(timing=True) for _ in range(5 if layers == 1 else 3)]
    if layers > 1:
        # the serialized baseline once more, after the timed region: clocks drift over a minute of sustained load
        ctx.set_cu_split(binding.CUS_ALL, binding.CUS_ALL)
        keep, hand[0] = hand[0], None
        run_steps(1)
        serial["ms_per_step_after_timed_region"] = timed(max(3, steps // 4))
        hand[0] = keep
        ctx.set_cu_split(chosen, d_cus)
    dec_lat = float(np.median([t.t_decode_ms for t in tms]))
    pre_lat = float(np.median([t.t_prefill_ms for t in tms]))

    traffic = load_traffic(wl.name)
    eff_cus = chosen if hand[0] is None else (hand[0] * chosen + (layers - hand[0]) * n_cus) / layers

    def roof(phase, k, ms):
        if phase == "prefill":
            fl = work["prefill_flops"][k]
            ach = fl / (ms * 1e-3) / 1e12
            r = {"kernel": f"{phase}.{k}", "bound": "mfma", "achieved": ach, "peak": PEAK_MFMA_TFLOPS,
                 "unit": "TFLOP/s", "frac": ach / PEAK_MFMA_TFLOPS, "traffic": None, "ms_per_launch": ms,
                 "flops_per_launch": fl, "cus": chosen, "frac_of_cu_share": ach / (PEAK_MFMA_TFLOPS * eff_cus / n_cus)}
            if hand[0] is not None:
                r["cus"] = f"{chosen} for layers < {hand[0]}, {n_cus} from there on (launch-weighted mean {eff_cus:.0f})"
        else:
            by = work["decode_bytes"][k]
            ach = by / (ms * 1e-3) / 1e9
            r = {"kernel": f"{phase}.{k}", "bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                 "frac": ach / PEAK_HBM_GBS, "traffic": None, "ms_per_launch": ms, "bytes_per_launch": by, "cus": d_cus}
        t = traffic.get(f"{phase}.{k}")
        if t:
            r["traffic"] = t["bytes_per_launch"]
            r["traffic_source"] = t["source"]
            alg = work["decode_bytes"][k] if phase == "decode" else work["prefill_bytes"].get(k)
            if alg:
                r["traffic_over_operand_bytes"] = t["bytes_per_launch"] / alg
        return r

    roofline = roof(dom[0], dom[1], dom_ms)
    roofline["launches_timed"] = dom_n
    others = {f"{a}.{b}": roof(a, b, kt[(a, b)][0]) for (a, b) in (("prefill", "gemm_gate_up"), ("prefill", "attn_prefill"),
                                                                   ("decode", "attn_decode"), ("decode", "gemm_gate_up")) if (a, b) != dom}
    pf, dbytes = work["prefill_layer_flops"] * layers, work["decode_layer_bytes"] * layers
    phase_roof = {
        "prefill_phase_tflops": pf / (pre_lat * 1e-3) / 1e12,
        "prefill_phase_frac_of_mfma_peak": pf / (pre_lat * 1e-3) / 1e12 / PEAK_MFMA_TFLOPS,
        "decode_phase_gbs": dbytes / (dec_lat * 1e-3) / 1e9,
        "decode_phase_frac_of_hbm_peak": dbytes / (dec_lat * 1e-3) / 1e9 / PEAK_HBM_GBS,
    }
    if alone:
        phase_roof["prefill_alone_all_cus_frac_of_mfma_peak"] = pf / (alone["t_prefill_all_cus_ms"] * 1e-3) / 1e12 / PEAK_MFMA_TFLOPS
        phase_roof["decode_alone_all_cus_frac_of_hbm_peak"] = dbytes / (alone["t_decode_all_cus_ms"] * 1e-3) / 1e9 / PEAK_HBM_GBS
    res = {
        "value": work["tokens"] / ms_per_step * 1e3, "ms_per_step": ms_per_step, "steps": steps,
        "config": {"workload": wl.name, "layers": layers, "prefill_tokens": wl.prefill.n_tokens,
                   "decode_requests": wl.decode.n_reqs,
                   "cu_split": f"{chosen}/{d_cus}" + (f", prefill on all {n_cus} CUs from layer {hand[0]}" if hand[0] is not None else ""),
                   "split_policy": ("min measured step time over the sweep of 32-CU splits" +
                                    (", each held to the end of the step or handed to the prefill phase when the decode step has ended" if layers > 1 and not args.no_handover else ""))
                   if args.split == "auto" else "given"},
        "decode_step_latency_ms": dec_lat, "prefill_phase_latency_ms": pre_lat,
        "serialized": serial, "speedup_vs_serialized": serial_ms / ms_per_step,
        "fused_single_batch": fused_res, "speedup_vs_fused_single_batch": (fused_res["ms_per_step"] / ms_per_step) if fused_res else None,
        "alone": alone, "sweep": sweep, "roofline": roofline, "roofline_other": others, "phase_roofline": phase_roof,
    }
    if headline and layers > 1 and not args.no_continuous:
        # steady state with decoding never paused (the serving case): the decode share that keeps a decode step within
        # alpha = 1.3 of its best (the decode-prioritised choice of the sweep, Sec. 4.1.2), against temporal slicing
        cd_splits = sorted({alone.get("decode_prioritized_prefill_cus", chosen) if alone else chosen, chosen, n_cus // 2}, reverse=True)
        res["continuous_decode"] = [continuous_decode(ctx, binding, wl, pb, db, kv, layers, (c, n_cus - c)) for c in cd_splits]
        ctx.set_cu_split(chosen, d_cus)
        log(f"[bench] {wl.name} continuous decode: {json.dumps(res['continuous_decode'])}")
    if headline and not args.no_cpu_baseline:
        big = s.hidden >= 8192
        res["cpu_baseline"] = cpu_baseline(wl, first, layers, 160 if big else 512, 32 if big else 64, 1 if big else 2)
    ctx.close()
    del ctx, kv, pb, db, wl
    torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed steps of the headline workload (default 20 at full depth, 200 for one layer)")
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--config", type=int, default=5, help="headline configuration (1..5)")
    ap.add_argument("--layers", type=int, default=0, help="layers of the headline stack (0 = the configuration's own depth)")
    ap.add_argument("--split", default="auto", help="'auto' (profile and choose) or PREFILL_CUS/DECODE_CUS")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-secondary", action="store_true", help="skip the 8B-shaped single-layer configurations")
    ap.add_argument("--no-fused", action="store_true", help="skip the fused single-batch step of the single-layer configurations")
    ap.add_argument("--trace", action="store_true", help="also run the trace-driven serving legs (48-layer 14B-shaped stack, about a minute)")
    ap.add_argument("--handover", default="", help="with --split: layer from which the prefill phase runs on all CUs, or 'auto' for the library's choice from its own phase timings")
    ap.add_argument("--no-handover", action="store_true", help="keep every split to the end of the step")
    ap.add_argument("--no-continuous", action="store_true", help="skip the continuous-decode leg of a multi-layer headline")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (known traffic) to calibrate rocprofv3 byte counters")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (the partitioned step is an intra-GPU method); --gpus must be 1")

    import torch

    from paper_2507_06608_amd import synth
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.config not in (1, 2, 3, 4, 5):
        sys.exit("bench.py: --config must be 1..5")
    depth = args.layers or {1: 1, 2: 1, 3: 1, 4: synth.SHAPES["qwen25_14b"].n_layers, 5: synth.SHAPES["llama3_70b"].n_layers}[args.config]
    steps = args.steps if args.steps is not None else (20 if depth > 8 else 200)
    warmup = args.warmup if args.warmup is not None else (3 if depth > 8 else 20)

    if args.calib_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    head = measure(args.config, depth, steps, warmup, args, headline=True)
    out = {
        "metric": "mixed-step tokens/s + decode-step latency vs CU split; MFMA %, HBM GB/s",
        "value": head.pop("value"), "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": head.pop("ms_per_step"), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": DTYPE, "data": "synthetic",
    }
    head.pop("steps")
    out.update(head)
    if not args.no_secondary:
        out["secondary"] = {}
        for idx in (2, 3):
            if idx == args.config and depth == 1:
                continue
            r = measure(idx, 1, 100 if idx == 2 else 30, 10 if idx == 2 else 5, args, headline=False)
            r["tokens_per_s"] = r.pop("value")
            out["secondary"][r["config"]["workload"]] = r
    if args.trace:
        try:
            out["serving_trace"] = serving_trace(log)
        except Exception as e:  # the headline above does not depend on this leg
            out["serving_trace"] = {"error": f"{type(e).__name__}: {e}"}
    print(json.dumps(out), flush=True)


def serving_trace(log):
    """The trace-driven configuration (14B-shaped stack of 48 layers, Poisson arrivals, lognormal prompt and
    output lengths, 1024-token chunks, SPF prefill queue, FCFS decode pool of 128) on the measured clock until every
    request has finished: coupled iterations on the unpartitioned GPU (prefill then decode, or both as one fused
    batch) against independent phase loops on a 160/96 split.  Latencies in milliseconds on the loop's own clock."""
    import torch

    from paper_2507_06608_amd import binding, synth
    from paper_2507_06608_amd.serve import DecoupledRunner, TraceRunner
    shape = synth.SHAPES["qwen25_14b"]
    rate, horizon = 12.0, 3.0
    trace = synth.poisson_trace(1, rate=rate, horizon_s=horizon, output_cap=384)
    arrivals = [a for a, _, _ in trace]

    def weights(l):
        return device_layer_weights(shape, l, synth.weight_std(shape))

    common = dict(policy=binding.PREFILL_SPF, token_budget=1024, max_decode_reqs=128, n_pages=12288, gamma=15.0,
                  max_prefill_reqs=8, seed=2)
    res = {"workload": f"qwen25_14b x {shape.n_layers} layers, Poisson {rate}/s for {horizon} s ({len(trace)} requests), "
                       "prompts lognormal(median 1024, sigma 0.8) <= 8192, outputs lognormal(median 256, sigma 0.7) <= 384",
           "unit": "ms"}
    for name, cls, split, fused in (("coupled_unpartitioned", TraceRunner, None, False), ("coupled_fused_single_batch", TraceRunner, None, True),
                                    ("independent_loops_160_96", DecoupledRunner, (160, 96), False)):
        run = cls(shape, shape.n_layers, weights, split=split, fused=fused, **common)
        run.submit(trace)
        if cls is DecoupledRunner:
            run.run_decoupled(arrivals, max_wall_s=150.0)
            rep = run.report_decoupled()
        else:
            run.run_until_done(arrivals)
            rep = run.report()
        res[name] = {"ttft_mean": rep["ttft_mean"] * 1e3, "ttft_p95": rep["ttft_p95"] * 1e3, "tbt_mean": rep["tbt_mean"] * 1e3,
                     "tbt_p95": rep["tbt_p95"] * 1e3, "tbt_p99": rep["tbt_p99"] * 1e3,
                     "normalized_latency_mean": rep["norm_latency_mean"] * 1e3, "tokens": rep["tokens"],
                     "tokens_per_s_of_gpu_busy_time": rep["tokens_per_s"], "finished": rep["n_finished"]}
        log(f"[bench] serving trace, {name}: {res[name]}")
        run.close()
        del run
        torch.cuda.empty_cache()
    return res


if __name__ == "__main__":
    main()

"""ctypes binding of libnexus.so (the C ABI of include/nexus.h).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  torch is used for device memory (tensors whose data_ptr() is handed
over) and for the caller's stream.  There is no CPU fallback: if the library
is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Dict, Optional, Sequence

import numpy as np
import torch

from .synth import DecodeBatch, ModelShape, PrefillBatch, Workload

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libnexus.so")

CUS_ALL = -1
PHASE_PREFILL, PHASE_DECODE = 0, 1
POLICY_PREFILL_PRIORITIZED, POLICY_DECODE_PRIORITIZED, POLICY_MIN_STEP = 0, 1, 2
HANDOVER_AUTO = -1
KERNELS = ("rmsnorm", "gemm_qkv", "rope_append", "attn_prefill", "gemm_o", "gemm_gate_up", "gemm_down",
           "attn_decode", "attn_merge", "splitk_reduce")
BUF_NORM1, BUF_Q, BUF_ATTN, BUF_X1, BUF_ACT = range(5)

EXPORTS = ("nexus_create", "nexus_destroy", "nexus_load_layer", "nexus_sync", "nexus_last_error", "nexus_cu_count",
           "nexus_kv_import", "nexus_kv_export", "nexus_set_cu_split",
           "nexus_prefill_chunk", "nexus_decode_step", "nexus_mixed_step", "nexus_mixed_step_handover", "nexus_last_handover_layer", "nexus_profile_split",
           "nexus_choose_split", "nexus_trace_begin", "nexus_trace_read", "nexus_debug_fetch",
           "nexus_debug_cu_probe", "nexus_debug_token_order", "nexus_cost_latency", "nexus_adjust_partition", "nexus_partition_controller",
           "nexus_cost_fit", "nexus_cost_describe",
           "nexus_sched_create", "nexus_sched_destroy", "nexus_sched_submit", "nexus_sched_next", "nexus_sched_commit",
           "nexus_sched_request", "nexus_sched_summarize", "nexus_sched_samples", "nexus_sched_next_phase",
           "nexus_sched_commit_phase", "nexus_phase_query", "nexus_phase_wait", "nexus_fused_step",
           "nexus_prepare_cu_splits", "nexus_retire_cu_splits", "nexus_set_debug_checks", "nexus_validate_batches", "nexus_decode_step_noalloc")


class NexusError(RuntimeError):
    pass


class ModelDesc(C.Structure):
    _fields_ = [("hidden", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("ffn", C.c_int32), ("n_layers", C.c_int32), ("page_size", C.c_int32),
                ("rms_eps", C.c_float), ("rope_theta", C.c_float)]


class Limits(C.Structure):
    _fields_ = [("max_prefill_tokens", C.c_int32), ("max_prefill_reqs", C.c_int32),
                ("max_decode_reqs", C.c_int32), ("max_positions", C.c_int32)]


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("attn_norm_g", "w_qkv", "b_qkv", "w_o", "ffn_norm_g", "w_gate_up", "w_down")]


class KVCache(C.Structure):
    _fields_ = [("k_pool", C.c_void_p), ("v_pool", C.c_void_p), ("layer_stride_bytes", C.c_int64),
                ("n_pages", C.c_int32)]


class PrefillBatchC(C.Structure):
    _fields_ = [("n_reqs", C.c_int32), ("n_tokens", C.c_int32), ("x", C.c_void_p), ("y", C.c_void_p),
                ("cu_chunk", C.c_void_p), ("prefix_len", C.c_void_p), ("page_table", C.c_void_p),
                ("max_pages", C.c_int32), ("max_chunk", C.c_int32), ("max_total_len", C.c_int32)]


class DecodeBatchC(C.Structure):
    _fields_ = [("n_reqs", C.c_int32), ("x", C.c_void_p), ("y", C.c_void_p), ("ctx_len", C.c_void_p),
                ("page_table", C.c_void_p), ("max_pages", C.c_int32), ("max_ctx", C.c_int32)]


class CostOp(C.Structure):
    _fields_ = [("flops", C.c_double), ("bytes", C.c_double), ("r_sat", C.c_double), ("lam", C.c_double),
                ("kind", C.c_int32), ("reserved", C.c_int32)]


class CostModelC(C.Structure):
    _fields_ = [("peak_flops", C.c_double), ("peak_bytes_per_s", C.c_double), ("n_prefill_ops", C.c_int32),
                ("n_decode_ops", C.c_int32), ("prefill_ops", C.POINTER(CostOp)), ("decode_ops", C.POINTER(CostOp))]


class StepTiming(C.Structure):
    _fields_ = [("t_prefill_ms", C.c_float), ("t_decode_ms", C.c_float), ("t_step_ms", C.c_float)]


_lib = None


def lib():
    """Loads libnexus.so; raises if it has not been built (see build.py / __graft_entry__.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise NexusError(f"{LIB_PATH} not found: build it with `python -m paper_2507_06608_amd.build`")
        _lib = C.CDLL(LIB_PATH)
        _lib.nexus_last_error.restype = C.c_char_p
        for name in EXPORTS:
            if name not in ("nexus_last_error", "nexus_destroy", "nexus_sched_destroy"):
                getattr(_lib, name).restype = C.c_int
        _lib.nexus_destroy.restype = None
        _lib.nexus_sched_destroy.restype = None
        _lib.nexus_choose_split.argtypes = [C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_float, C.c_float,
                                            C.c_int, C.c_float, C.c_float]
    return _lib


def _check(rc: int) -> int:
    if rc < 0:
        raise NexusError(f"nexus error {rc}: {lib().nexus_last_error().decode()}")
    return rc


def choose_split(t_p, t_d, t_step, t_p_all: float, t_d_all: float, policy: int, alpha: float, beta: float) -> int:
    """Host-only selection rule on measured curves (no GPU needed)."""
    a, b, s = (np.ascontiguousarray(v, np.float32) for v in (t_p, t_d, t_step))
    return _check(lib().nexus_choose_split(len(a), a.ctypes.data, b.ctypes.data, s.ctypes.data, t_p_all, t_d_all,
                                           policy, alpha, beta))


def validate_batches(n_pages: int, page_size: int, prefill: Optional[PrefillBatch] = None, decode: Optional[DecodeBatch] = None,
                     hints: Optional[dict] = None) -> None:
    """Host-only validation of a step's integer inputs (numpy arrays); raises NexusError on the first violation.
    hints may override max_chunk / max_total_len / max_ctx (default: the tightest values)."""
    hints = hints or {}
    i32 = lambda a: np.ascontiguousarray(a, np.int32)
    args = [n_pages, page_size]
    keep = []
    if prefill is not None and prefill.n_reqs:
        cu, pre, pt = i32(prefill.cu_chunk), i32(prefill.prefix_len), i32(prefill.page_table)
        keep += [cu, pre, pt]
        chunk = np.diff(cu)
        args += [len(pre), hints.get("n_tokens", int(cu[-1])), cu.ctypes.data_as(C.c_void_p), pre.ctypes.data_as(C.c_void_p),
                 pt.ctypes.data_as(C.c_void_p), pt.shape[1], hints.get("max_chunk", int(chunk.max())),
                 hints.get("max_total_len", int((pre + chunk).max()))]
    else:
        args += [0, 0, None, None, None, 0, 0, 0]
    if decode is not None and decode.n_reqs:
        ctx, pt = i32(decode.ctx_len), i32(decode.page_table)
        keep += [ctx, pt]
        args += [len(ctx), ctx.ctypes.data_as(C.c_void_p), pt.ctypes.data_as(C.c_void_p), pt.shape[1],
                 hints.get("max_ctx", int(ctx.max()) + 1)]
    else:
        args += [0, None, None, 0, 0]
    _check(lib().nexus_validate_batches(*args))


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


class DevPrefill:
    """A prefill sub-batch resident on the GPU; keeps the tensors alive and builds the C descriptor."""

    def __init__(self, b: PrefillBatch, device):
        self.host = b
        self.x = b.x.to(device).contiguous()
        self.y = torch.empty_like(self.x)
        self.cu = torch.from_numpy(b.cu_chunk.astype(np.int32)).to(device)
        self.prefix = torch.from_numpy(b.prefix_len.astype(np.int32)).to(device)
        self.pt = torch.from_numpy(np.ascontiguousarray(b.page_table, np.int32)).to(device)
        total = b.prefix_len + b.chunk_len
        self.c = PrefillBatchC(b.n_reqs, b.n_tokens, self.x.data_ptr(), self.y.data_ptr(), self.cu.data_ptr(),
                               self.prefix.data_ptr(), self.pt.data_ptr(), b.page_table.shape[1],
                               int(b.chunk_len.max()), int(total.max()))


class DevDecode:
    def __init__(self, b: DecodeBatch, device):
        self.host = b
        self.x = b.x.to(device).contiguous()
        self.y = torch.empty_like(self.x)
        self.ctx = torch.from_numpy(b.ctx_len.astype(np.int32)).to(device)
        self.pt = torch.from_numpy(np.ascontiguousarray(b.page_table, np.int32)).to(device)
        self.c = DecodeBatchC(b.n_reqs, self.x.data_ptr(), self.y.data_ptr(), self.ctx.data_ptr(),
                              self.pt.data_ptr(), b.page_table.shape[1], int(b.ctx_len.max()) + 1)


class Nexus:
    """One context: model shape, workspace limits, packed weights, CU layouts."""

    def __init__(self, shape: ModelShape, *, max_prefill_tokens: int, max_prefill_reqs: int, max_decode_reqs: int,
                 max_positions: int, device: int = 0, n_layers: Optional[int] = None):
        self.shape = shape
        self.device = torch.device("cuda", device)
        self.n_layers = n_layers or shape.n_layers
        desc = ModelDesc(shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.ffn, self.n_layers,
                         shape.page_size, shape.rms_eps, shape.rope_theta)
        lim = Limits(max_prefill_tokens, max_prefill_reqs, max_decode_reqs, max_positions)
        self._ctx = C.c_void_p()
        torch.cuda.init()
        _check(lib().nexus_create(C.byref(desc), C.byref(lim), device, C.byref(self._ctx)))

    # -- lifetime
    def close(self):
        if self._ctx:
            lib().nexus_destroy(self._ctx)
            self._ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def sync(self):
        _check(lib().nexus_sync(self._ctx))

    @property
    def cu_count(self) -> int:
        return _check(lib().nexus_cu_count(self._ctx))

    # -- weights
    def load_layer(self, layer: int, w: Dict[str, torch.Tensor]):
        dev = {k: (None if v is None else v.to(self.device, torch.bfloat16).contiguous()) for k, v in w.items()}
        cw = LayerWeights(*[None if dev.get(k) is None else dev[k].data_ptr() for k in
                            ("attn_norm_g", "w_qkv", "b_qkv", "w_o", "ffn_norm_g", "w_gate_up", "w_down")])
        torch.cuda.synchronize(self.device)   # the library's stream does not wait for torch's: sources must be complete
        _check(lib().nexus_load_layer(self._ctx, layer, C.byref(cw)))

    # -- KV cache
    def make_kv(self, k_canon: torch.Tensor, v_canon: torch.Tensor, layers: int = 1):
        """Allocates private pools for `layers` layers and imports the canonical pools
        [n_pages, Hkv, page, hd] (bf16, any device) into every layer."""
        s = self.shape
        n_pages = k_canon.shape[0]
        assert tuple(k_canon.shape) == (n_pages, s.n_kv_heads, s.page_size, s.head_dim)
        per_layer = n_pages * s.n_kv_heads * s.page_size * s.head_dim
        kp = torch.empty(layers * per_layer, dtype=torch.bfloat16, device=self.device)
        vp = torch.empty(layers * per_layer, dtype=torch.bfloat16, device=self.device)
        kv = KVCache(kp.data_ptr(), vp.data_ptr(), per_layer * 2, n_pages)
        kc = k_canon.to(self.device).contiguous()
        vc = v_canon.to(self.device).contiguous()
        torch.cuda.synchronize(self.device)
        for l in range(layers):
            _check(lib().nexus_kv_import(self._ctx, C.byref(kv), l, _ptr(kc), _ptr(vc), 0, n_pages))
        kv.pools = (kp, vp)      # the descriptor owns its tensors: it stays valid as long as the caller holds it
        return kv

    def alloc_kv(self, n_pages: int, layers: int):
        """Zero-filled pools of `n_pages` pages for `layers` layers (all zeros is the same in either page layout)."""
        s = self.shape
        per_layer = n_pages * s.n_kv_heads * s.page_size * s.head_dim
        kp = torch.zeros(layers * per_layer, dtype=torch.bfloat16, device=self.device)
        vp = torch.zeros(layers * per_layer, dtype=torch.bfloat16, device=self.device)
        torch.cuda.synchronize(self.device)
        kv = KVCache(kp.data_ptr(), vp.data_ptr(), per_layer * 2, n_pages)
        kv.pools = (kp, vp)
        return kv

    def kv_export(self, kv: KVCache, layer: int = 0):
        s = self.shape
        shape = (kv.n_pages, s.n_kv_heads, s.page_size, s.head_dim)
        kc = torch.empty(shape, dtype=torch.bfloat16, device=self.device)
        vc = torch.empty(shape, dtype=torch.bfloat16, device=self.device)
        _check(lib().nexus_kv_export(self._ctx, C.byref(kv), layer, _ptr(kc), _ptr(vc), 0, kv.n_pages))
        return kc, vc

    # -- partitioning
    def set_cu_split(self, prefill_cus: int, decode_cus: int):
        _check(lib().nexus_set_cu_split(self._ctx, prefill_cus, decode_cus))

    def prepare_cu_splits(self, splits: Sequence[tuple]):
        """Creates the stream pairs of the given (prefill_cus, decode_cus) splits ahead of use."""
        n = len(splits)
        p, d = (C.c_int32 * n)(*[s[0] for s in splits]), (C.c_int32 * n)(*[s[1] for s in splits])
        _check(lib().nexus_prepare_cu_splits(self._ctx, n, p, d))

    def retire_cu_splits(self):
        _check(lib().nexus_retire_cu_splits(self._ctx))

    def set_debug_checks(self, on: bool):
        _check(lib().nexus_set_debug_checks(self._ctx, int(on)))

    # -- steps
    def prefill_chunk(self, pb: DevPrefill, kv: KVCache, layers=(0, 1)):
        _check(lib().nexus_prefill_chunk(self._ctx, layers[0], layers[1], C.byref(pb.c), C.byref(kv)))

    def decode_step(self, db: DevDecode, kv: KVCache, layers=(0, 1)):
        _check(lib().nexus_decode_step(self._ctx, layers[0], layers[1], C.byref(db.c), C.byref(kv)))

    def decode_step_noalloc(self, db: DevDecode, kv: KVCache, layers=(0, 1)):
        _check(lib().nexus_decode_step_noalloc(self._ctx, layers[0], layers[1], C.byref(db.c), C.byref(kv)))

    def fused_step(self, batch: DevPrefill, n_decode_reqs: int, max_decode_ctx: int, kv: KVCache, layers=(0, 1)):
        """One batch, the last n_decode_reqs requests being decode requests written as one-token chunks."""
        _check(lib().nexus_fused_step(self._ctx, layers[0], layers[1], C.byref(batch.c), n_decode_reqs, max_decode_ctx,
                                      C.byref(kv)))

    def mixed_step(self, pb: DevPrefill, db: DevDecode, kv: KVCache, layers=(0, 1), stream=None, timing=False):
        tm = StepTiming() if timing else None
        sp = C.c_void_p(stream.cuda_stream) if stream is not None else None
        _check(lib().nexus_mixed_step(self._ctx, layers[0], layers[1], C.byref(pb.c), C.byref(db.c), C.byref(kv), sp,
                                      C.byref(tm) if timing else None))
        return tm

    def mixed_step_handover(self, pb: DevPrefill, db: DevDecode, kv: KVCache, handover_layer: int, layers=(0, 1), stream=None,
                            timing=False):
        tm = StepTiming() if timing else None
        sp = C.c_void_p(stream.cuda_stream) if stream is not None else None
        _check(lib().nexus_mixed_step_handover(self._ctx, layers[0], layers[1], handover_layer, C.byref(pb.c), C.byref(db.c),
                                               C.byref(kv), sp, C.byref(tm) if timing else None))
        return tm

    def last_handover_layer(self) -> int:
        return _check(lib().nexus_last_handover_layer(self._ctx))

    def phase_done(self, phase: int) -> bool:
        return bool(_check(lib().nexus_phase_query(self._ctx, phase)))

    def phase_wait(self, phase: int) -> float:
        ms = C.c_float()
        _check(lib().nexus_phase_wait(self._ctx, phase, C.byref(ms)))
        return ms.value

    def profile_split(self, pb: DevPrefill, db: DevDecode, kv: KVCache, cand_prefill_cus: Sequence[int], policy: int,
                      alpha: float = 1.3, beta: float = 1.1, repeats: int = 5, layers=(0, 1)):
        n = len(cand_prefill_cus)
        cand = (C.c_int32 * n)(*cand_prefill_cus)
        tp, td, ts = (C.c_float * n)(), (C.c_float * n)(), (C.c_float * n)()
        tall = (C.c_float * 2)()
        chosen = C.c_int32()
        _check(lib().nexus_profile_split(self._ctx, layers[0], layers[1], C.byref(pb.c), C.byref(db.c), C.byref(kv),
                                         cand, n, policy, C.c_float(alpha), C.c_float(beta), repeats, tp, td, ts, tall,
                                         C.byref(chosen)))
        return {"cand_prefill_cus": list(cand_prefill_cus), "t_prefill_ms": list(tp), "t_decode_ms": list(td),
                "t_step_ms": list(ts), "t_prefill_all_ms": tall[0], "t_decode_all_ms": tall[1],
                "chosen_prefill_cus": chosen.value}

    # -- measurement / debug
    def trace_begin(self, phase: int, kernel: str):
        _check(lib().nexus_trace_begin(self._ctx, phase, KERNELS.index(kernel)))

    def trace_read(self):
        ms, n = C.c_float(), C.c_int32()
        _check(lib().nexus_trace_read(self._ctx, C.byref(ms), C.byref(n)))
        return ms.value, n.value

    def debug_fetch(self, phase: int, which: int, n_tokens: int) -> torch.Tensor:
        s = self.shape
        width = {BUF_Q: s.q_dim, BUF_ATTN: s.q_dim, BUF_X1: s.hidden, BUF_ACT: s.ffn}[which]
        out = torch.empty((n_tokens, width), dtype=torch.float32, device=self.device)
        _check(lib().nexus_debug_fetch(self._ctx, phase, which, n_tokens, _ptr(out)))
        return out

    def cu_probe(self, phase: int, n_blocks: int = 8192) -> np.ndarray:
        out = np.zeros(8 * 128, np.int32)
        _check(lib().nexus_debug_cu_probe(self._ctx, phase, n_blocks, out.ctypes.data_as(C.c_void_p)))
        return out.reshape(8, 8, 16)


OP_DENSE, OP_ATTENTION = 0, 1


class CostModel:
    """Host-side latency model of the two phases (marshalling only; the arithmetic is in the library).
    ops: sequences of (flops, bytes, r_sat, lambda, kind)."""

    def __init__(self, peak_flops: float, peak_bytes_per_s: float, prefill_ops, decode_ops):
        self._p = (CostOp * max(len(prefill_ops), 1))(*[CostOp(*o, 0) for o in prefill_ops])
        self._d = (CostOp * max(len(decode_ops), 1))(*[CostOp(*o, 0) for o in decode_ops])
        self.c = CostModelC(peak_flops, peak_bytes_per_s, len(prefill_ops), len(decode_ops), self._p, self._d)

    def latency(self, phase: int, share: int, total: int) -> float:
        out = C.c_double()
        _check(lib().nexus_cost_latency(C.byref(self.c), phase, share, total, C.byref(out)))
        return out.value

    def adjust_partition(self, target_phase: int, cur_prefill_share: int, total: int, alpha: float, beta: float):
        new, ev = C.c_int32(), C.c_int32()
        _check(lib().nexus_adjust_partition(C.byref(self.c), target_phase, cur_prefill_share, total, C.c_double(alpha),
                                            C.c_double(beta), C.byref(new), C.byref(ev)))
        return new.value, ev.value

    def partition_controller(self, kv_usage: float, kv_switch: float, cur_prefill_share: int, total: int, alpha: float,
                             beta: float, delta: int) -> int:
        new = C.c_int32()
        _check(lib().nexus_partition_controller(C.byref(self.c), C.c_double(kv_usage), C.c_double(kv_switch),
                                                cur_prefill_share, total, C.c_double(alpha), C.c_double(beta), delta,
                                                C.byref(new)))
        return new.value


def cost_fit(shares, seconds, peak_flops: float):
    n = len(shares)
    a, b = (C.c_double * n)(*shares), (C.c_double * n)(*seconds)
    f, r, l = C.c_double(), C.c_double(), C.c_double()
    _check(lib().nexus_cost_fit(n, a, b, C.c_double(peak_flops), C.byref(f), C.byref(r), C.byref(l)))
    return f.value, r.value, l.value


def cost_describe(shape, layers: int, prefill_tokens: float, prefill_pairs: float, prefill_kv_tokens: float,
                  decode_reqs: float, decode_kv_tokens: float):
    """Algorithmic (flops, bytes, 1.0, 0.0, kind) of QKV, attention, O, gate/up, down for each phase."""
    md = ModelDesc(shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.ffn, layers, shape.page_size,
                   shape.rms_eps, shape.rope_theta)
    p, d = (CostOp * 5)(), (CostOp * 5)()
    _check(lib().nexus_cost_describe(C.byref(md), layers, C.c_double(prefill_tokens), C.c_double(prefill_pairs),
                                     C.c_double(prefill_kv_tokens), C.c_double(decode_reqs), C.c_double(decode_kv_tokens), p, d))
    unpack = lambda ops: [(o.flops, o.bytes, o.r_sat, o.lam, o.kind) for o in ops]
    return unpack(p), unpack(d)


def context_for(w: Workload, device: int = 0, n_layers: int = 1) -> Nexus:
    """A context sized for one workload."""
    p, d = w.prefill, w.decode
    max_pos = 1
    if p is not None:
        max_pos = max(max_pos, int((p.prefix_len + p.chunk_len).max()))
    if d is not None:
        max_pos = max(max_pos, int(d.ctx_len.max()) + 1)
    return Nexus(w.shape, max_prefill_tokens=p.n_tokens if p else 1, max_prefill_reqs=p.n_reqs if p else 1,
                 max_decode_reqs=d.n_reqs if d else 1, max_positions=max_pos, device=device, n_layers=n_layers)


# ---- phase-specific schedulers (host only) ------------------------------------------------------------------------
PREFILL_FCFS, PREFILL_SPF = 0, 1
_I32P = C.POINTER(C.c_int32)


class SchedConfigC(C.Structure):
    _fields_ = [("prefill_policy", C.c_int32), ("token_budget", C.c_int32), ("max_prefill_reqs", C.c_int32),
                ("max_decode_reqs", C.c_int32), ("page_size", C.c_int32), ("n_pages", C.c_int32),
                ("chunk_tail", C.c_int32), ("reserved", C.c_int32), ("gamma", C.c_double), ("page_order", _I32P)]


class SchedBatchC(C.Structure):
    _fields_ = [("n_prefill", C.c_int32), ("prefill_tokens", C.c_int32), ("prefill_req", _I32P),
                ("prefill_prefix", _I32P), ("prefill_chunk", _I32P), ("prefill_cu_chunk", _I32P),
                ("prefill_page_table", _I32P), ("prefill_max_pages", C.c_int32), ("prefill_max_chunk", C.c_int32),
                ("prefill_max_total_len", C.c_int32), ("n_decode", C.c_int32), ("decode_req", _I32P),
                ("decode_ctx", _I32P), ("decode_page_table", _I32P), ("decode_max_pages", C.c_int32),
                ("decode_max_ctx", C.c_int32), ("kv_used_pages", C.c_int32), ("kv_total_pages", C.c_int32)]


class SchedRequestInfo(C.Structure):
    _fields_ = [("arrival_s", C.c_double), ("first_token_s", C.c_double), ("finish_s", C.c_double),
                ("prompt_len", C.c_int32), ("output_len", C.c_int32), ("prefilled", C.c_int32), ("emitted", C.c_int32),
                ("n_pages", C.c_int32), ("state", C.c_int32)]


class SchedSummary(C.Structure):
    _fields_ = [("n_submitted", C.c_int32), ("n_first_token", C.c_int32), ("n_finished", C.c_int32), ("reserved", C.c_int32),
                ("prefill_tokens", C.c_int64), ("decode_tokens", C.c_int64)] + \
               [(k, C.c_double) for k in ("ttft_mean", "ttft_p50", "ttft_p95", "ttft_p99", "ttft_max", "tbt_mean", "tbt_p50",
                                          "tbt_p95", "tbt_p99", "tbt_max", "norm_latency_mean", "norm_latency_p95")]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_ if k != "reserved"}


def _arr(ptr, n) -> np.ndarray:
    return np.ctypeslib.as_array(ptr, shape=(n,)).copy() if n else np.zeros(0, np.int32)


@dataclass
class SchedIteration:
    """Host copies of one iteration's batches (the scheduler's own arrays are only valid until its next call)."""
    prefill_req: np.ndarray
    prefill_prefix: np.ndarray
    prefill_chunk: np.ndarray
    prefill_cu_chunk: np.ndarray
    prefill_page_table: np.ndarray   # [n_prefill, max_pages]
    prefill_max_chunk: int
    prefill_max_total_len: int
    decode_req: np.ndarray
    decode_ctx: np.ndarray
    decode_page_table: np.ndarray    # [n_decode, max_pages]
    decode_max_ctx: int
    kv_used_pages: int
    kv_total_pages: int


class Scheduler:
    """Marshalling around nexus_sched_*; every decision is taken in the library."""

    def __init__(self, policy: int, token_budget: int, max_decode_reqs: int, page_size: int, n_pages: int,
                 gamma: float = 15.0, chunk_tail: bool = True, max_prefill_reqs: int = 0, page_order=None):
        order = None if page_order is None else np.ascontiguousarray(page_order, np.int32)
        cfg = SchedConfigC(policy, token_budget, max_prefill_reqs, max_decode_reqs, page_size, n_pages, int(chunk_tail), 0,
                           gamma, None if order is None else order.ctypes.data_as(_I32P))
        self._s = C.c_void_p()
        _check(lib().nexus_sched_create(C.byref(cfg), C.byref(self._s)))

    def close(self):
        if self._s:
            lib().nexus_sched_destroy(self._s)
            self._s = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def submit(self, arrival_s: float, prompt_len: int, output_len: int) -> int:
        rid = C.c_int32()
        _check(lib().nexus_sched_submit(self._s, C.c_double(arrival_s), prompt_len, output_len, C.byref(rid)))
        return rid.value

    def next(self, now_s: float) -> SchedIteration:
        b = SchedBatchC()
        _check(lib().nexus_sched_next(self._s, C.c_double(now_s), C.byref(b)))
        return self._iteration(b)

    def _iteration(self, b: SchedBatchC) -> SchedIteration:
        npf, nd = b.n_prefill, b.n_decode
        return SchedIteration(
            _arr(b.prefill_req, npf), _arr(b.prefill_prefix, npf), _arr(b.prefill_chunk, npf), _arr(b.prefill_cu_chunk, npf + 1 if b.prefill_cu_chunk else 0),
            _arr(b.prefill_page_table, npf * b.prefill_max_pages).reshape(npf, max(b.prefill_max_pages, 1)), b.prefill_max_chunk,
            b.prefill_max_total_len, _arr(b.decode_req, nd), _arr(b.decode_ctx, nd),
            _arr(b.decode_page_table, nd * b.decode_max_pages).reshape(nd, max(b.decode_max_pages, 1)), b.decode_max_ctx,
            b.kv_used_pages, b.kv_total_pages)

    def next_phase(self, phase: int, now_s: float) -> SchedIteration:
        """One phase's tick; the other phase's arrays come back empty."""
        b = SchedBatchC()
        _check(lib().nexus_sched_next_phase(self._s, phase, C.c_double(now_s), C.byref(b)))
        return self._iteration(b)

    def commit_phase(self, phase: int, end_s: float):
        _check(lib().nexus_sched_commit_phase(self._s, phase, C.c_double(end_s)))

    def commit(self, end_s: float):
        _check(lib().nexus_sched_commit(self._s, C.c_double(end_s)))

    def request(self, rid: int) -> SchedRequestInfo:
        info = SchedRequestInfo()
        _check(lib().nexus_sched_request(self._s, rid, C.byref(info)))
        return info

    def summary(self) -> dict:
        out = SchedSummary()
        _check(lib().nexus_sched_summarize(self._s, C.byref(out)))
        return out.as_dict()

    def samples(self, kind: int) -> np.ndarray:
        n = C.c_int32()
        _check(lib().nexus_sched_samples(self._s, kind, None, 0, C.byref(n)))
        out = np.zeros(n.value, np.float64)
        if n.value:
            _check(lib().nexus_sched_samples(self._s, kind, out.ctypes.data_as(C.POINTER(C.c_double)), n.value, C.byref(n)))
        return out

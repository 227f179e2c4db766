"""Seeded synthetic inputs shaped like the paper's serving workloads.

This module holds none of the method's arithmetic: it only draws random
numbers, rounds them to bf16 and lays out batch descriptors (chunk offsets,
prefix/context lengths, page tables).  Both the HIP path and the CPU oracle
consume the arrays produced here, so the generator itself is not part of any
parity claim.

Stand-ins: the paper evaluates on Long Data Collections, ArXiv Summarization
and a ShareGPT mix (Sec. 6.1, Table 1: inputs of a few hundred to ~10K tokens,
outputs of a few hundred).  Those datasets are not available here; the
workloads below bracket the same lengths with uniform / fixed draws.

Value recipe: weight matrices N(0, 0.02); RMSNorm gains 1 + N(0, 0.02);
activations N(0, 1); pre-existing KV-cache contents N(0, 1); everything rounded
to bf16 (round-to-nearest-even).  Page tables are a random permutation of a
pool holding exactly the pages the batch needs.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np
import torch

PAGE_SIZE = 16


@dataclass(frozen=True)
class ModelShape:
    name: str
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    rope_theta: float
    rms_eps: float = 1e-5
    page_size: int = PAGE_SIZE
    n_layers: int = 1

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    @property
    def n_qkv(self) -> int:
        return self.q_dim + 2 * self.kv_dim

    @property
    def params_per_layer(self) -> int:
        return self.hidden * (self.n_qkv + self.q_dim + 3 * self.ffn)


SHAPES: Dict[str, ModelShape] = {
    "tiny": ModelShape("tiny", 512, 8, 8, 64, 1376, 10000.0),
    "llama3_8b": ModelShape("llama3_8b", 4096, 32, 8, 128, 14336, 500000.0),
    "qwen25_14b": ModelShape("qwen25_14b", 5120, 40, 8, 128, 13824, 1000000.0, n_layers=48),
    "llama3_70b": ModelShape("llama3_70b", 8192, 64, 8, 128, 28672, 500000.0, n_layers=80),
}


def _bf16(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16)


def weight_std(shape: ModelShape) -> float:
    """Standard deviation of the weight matrices: 0.02 as the configurations state it, except for the 70B shape,
    whose configuration names no distribution: there the variance follows the fan-in (0.02 at hidden 4096, so
    0.02 / sqrt(2) at 8192), which keeps a layer's output at the scale of its input instead of 7 times larger."""
    return 0.02 * (4096.0 / shape.hidden) ** 0.5 if shape.name == "llama3_70b" else 0.02


def make_weights(shape: ModelShape, seed: int, layer: int = 0, std: Optional[float] = None) -> Dict[str, torch.Tensor]:
    """bf16 CPU tensors of one layer, in the [out_features, in_features] orientation."""
    rng = np.random.default_rng([seed, 1000 + layer])
    d, F = shape.hidden, shape.ffn
    std = np.float32(weight_std(shape) if std is None else std)

    def mat(r, c):
        return _bf16(rng.standard_normal((r, c), dtype=np.float32) * std)

    def gain():
        return _bf16(1.0 + rng.standard_normal(d, dtype=np.float32) * np.float32(0.02))

    return {
        "attn_norm_g": gain(),
        "w_qkv": mat(shape.n_qkv, d),
        "w_o": mat(d, shape.q_dim),
        "ffn_norm_g": gain(),
        "w_gate_up": mat(2 * F, d),
        "w_down": mat(d, F),
    }


@dataclass
class PrefillBatch:
    x: torch.Tensor            # [T, hidden] bf16
    cu_chunk: np.ndarray       # [n_reqs + 1] int32
    prefix_len: np.ndarray     # [n_reqs] int32
    page_table: np.ndarray     # [n_reqs, max_pages] int32

    @property
    def n_reqs(self) -> int:
        return len(self.prefix_len)

    @property
    def n_tokens(self) -> int:
        return int(self.cu_chunk[-1])

    @property
    def chunk_len(self) -> np.ndarray:
        return np.diff(self.cu_chunk)


@dataclass
class DecodeBatch:
    x: torch.Tensor            # [n_reqs, hidden] bf16
    ctx_len: np.ndarray        # [n_reqs] int32, tokens cached before this step
    page_table: np.ndarray     # [n_reqs, max_pages] int32

    @property
    def n_reqs(self) -> int:
        return len(self.ctx_len)


@dataclass
class Workload:
    name: str
    shape: ModelShape
    seed: int
    n_pages: int
    prefill: Optional[PrefillBatch]
    decode: Optional[DecodeBatch]
    k_pool: torch.Tensor       # canonical [n_pages, Hkv, page_size, hd] bf16
    v_pool: torch.Tensor
    notes: dict = field(default_factory=dict)


def _pages_for(n_tokens: int, page_size: int) -> int:
    return (n_tokens + page_size - 1) // page_size


def make_workload(name: str, shape: ModelShape, seed: int, *, chunk_lens: List[int], prefix_lens: List[int],
                  decode_ctx: List[int], kv_device: str = "cpu", page_slack: int = 0) -> Workload:
    """Build both sub-batches over one shared page pool.

    chunk_lens / prefix_lens: per prefill request; decode_ctx: per decode request
    (tokens cached before the step).  Each request gets the pages covering all
    positions it will hold after the step; `page_slack` unused pages are added
    to the pool.  Page ids are a random permutation of the pool, so no two
    requests share a page.  Pool contents are N(0, 1) everywhere (slots past a
    request's length hold values that must never be read).
    """
    assert len(chunk_lens) == len(prefix_lens)
    rng = np.random.default_rng([seed, 7])
    ps = shape.page_size
    need_p = [_pages_for(p + n, ps) for p, n in zip(prefix_lens, chunk_lens)]
    need_d = [_pages_for(c + 1, ps) for c in decode_ctx]
    n_pages = int(sum(need_p) + sum(need_d) + page_slack)
    n_pages = max(n_pages, 1)
    perm = rng.permutation(n_pages).astype(np.int32)
    cursor = 0

    def table(needs):
        nonlocal cursor
        width = max(needs) if needs else 1
        # Entries past a request's own pages are set to -1 and must never be dereferenced.
        t = np.full((len(needs), width), -1, np.int32)
        for r, k in enumerate(needs):
            t[r, :k] = perm[cursor:cursor + k]
            cursor += k
        return t

    pt_p = table(need_p)
    pt_d = table(need_d)

    prefill = None
    if chunk_lens:
        cu = np.zeros(len(chunk_lens) + 1, np.int32)
        cu[1:] = np.cumsum(chunk_lens)
        xp = _bf16(rng.standard_normal((int(cu[-1]), shape.hidden), dtype=np.float32))
        prefill = PrefillBatch(xp, cu, np.asarray(prefix_lens, np.int32), pt_p)
    decode = None
    if decode_ctx:
        xd = _bf16(rng.standard_normal((len(decode_ctx), shape.hidden), dtype=np.float32))
        decode = DecodeBatch(xd, np.asarray(decode_ctx, np.int32), pt_d)

    pool_shape = (n_pages, shape.n_kv_heads, ps, shape.head_dim)
    if kv_device == "cpu":
        k_pool = _bf16(rng.standard_normal(pool_shape, dtype=np.float32))
        v_pool = _bf16(rng.standard_normal(pool_shape, dtype=np.float32))
    else:
        g = torch.Generator(device=kv_device)
        g.manual_seed(seed * 7919 + 13)
        k_pool = torch.randn(pool_shape, generator=g, device=kv_device, dtype=torch.float32).to(torch.bfloat16)
        v_pool = torch.randn(pool_shape, generator=g, device=kv_device, dtype=torch.float32).to(torch.bfloat16)
    return Workload(name, shape, seed, n_pages, prefill, decode, k_pool, v_pool)


def config(idx: int, seed: int = 0, kv_device: str = "cpu") -> Workload:
    """The benchmark configurations, by their 1-based index."""
    rng = np.random.default_rng([seed, 99, idx])
    if idx == 1:
        ctx = rng.integers(64, 257, size=8).tolist()
        return make_workload("cfg1_tiny", SHAPES["tiny"], seed, chunk_lens=[128], prefix_lens=[0],
                             decode_ctx=ctx, kv_device=kv_device)
    if idx == 2:
        ctx = rng.integers(512, 4097, size=64).tolist()
        return make_workload("cfg2_llama3_8b_512over1536_64dec", SHAPES["llama3_8b"], seed, chunk_lens=[512],
                             prefix_lens=[1536], decode_ctx=ctx, kv_device=kv_device)
    if idx == 3:
        ctx = rng.integers(1024, 8193, size=256).tolist()
        pre = rng.integers(0, 6145, size=4).tolist()
        return make_workload("cfg3_llama3_8b_heavy", SHAPES["llama3_8b"], seed, chunk_lens=[2048] * 4,
                             prefix_lens=pre, decode_ctx=ctx, kv_device=kv_device)
    if idx == 4:
        # One iteration of the trace-driven configuration at its caps: a full 1024-token chunk in the middle of a
        # long prompt next to a full decode pool (output positions on top of lognormal-like prompt lengths).
        ctx = np.minimum(8192 + 1024, rng.lognormal(np.log(1024.0), 0.8, size=128) + rng.lognormal(np.log(256.0), 0.7, size=128))
        return make_workload("cfg4_qwen25_14b_iteration", SHAPES["qwen25_14b"], seed, chunk_lens=[1024],
                             prefix_lens=[3072], decode_ctx=[int(c) for c in ctx], kv_device=kv_device)
    if idx == 5:
        ctx = rng.integers(1024, 4097, size=64).tolist()
        return make_workload("cfg5_llama3_70b_2048over2048_64dec", SHAPES["llama3_70b"], seed, chunk_lens=[2048],
                             prefix_lens=[2048], decode_ctx=ctx, kv_device=kv_device)
    raise ValueError(f"no configuration {idx}")


def fused_single_batch(w: Workload) -> PrefillBatch:
    """The two sub-batches as ONE chunked-prefill batch, the way an engine without phase separation runs them
    (Sec. 2.4): every decode request becomes a one-token chunk over a prefix of its context length, appended after
    the prefill requests.  Rows of the result: the prefill tokens, then one row per decode request."""
    p, d = w.prefill, w.decode
    width = max(p.page_table.shape[1], d.page_table.shape[1])

    def pad(t):
        out = np.full((t.shape[0], width), -1, np.int32)
        out[:, :t.shape[1]] = t
        return out
    cu = np.concatenate([p.cu_chunk, p.cu_chunk[-1] + 1 + np.arange(d.n_reqs, dtype=np.int32)]).astype(np.int32)
    return PrefillBatch(torch.cat([p.x, d.x], 0), cu, np.concatenate([p.prefix_len, d.ctx_len]).astype(np.int32),
                        np.concatenate([pad(p.page_table), pad(d.page_table)], 0))


def subset_for_oracle(w: Workload, prefill_reqs: List[int], decode_reqs: List[int]):
    """Cut a workload down to some of its requests, with page ids renumbered
    into a small pool, so that the oracle can evaluate sampled requests of a
    large configuration.  Returns a Workload whose pools are CPU tensors."""
    ps = w.shape.page_size
    pages: List[int] = []
    pt_p = pt_d = None
    prefill = decode = None

    def remap(table, needs):
        out = np.full((len(needs), max(needs) if needs else 1), -1, np.int32)
        for i, (row, k) in enumerate(zip(table, needs)):
            for c in range(k):
                out[i, c] = len(pages)
                pages.append(int(row[c]))
        return out

    if w.prefill is not None and prefill_reqs:
        p = w.prefill
        needs = [_pages_for(int(p.prefix_len[r] + p.chunk_len[r]), ps) for r in prefill_reqs]
        pt_p = remap([p.page_table[r] for r in prefill_reqs], needs)
        xs = [p.x[int(p.cu_chunk[r]):int(p.cu_chunk[r + 1])] for r in prefill_reqs]
        cu = np.zeros(len(prefill_reqs) + 1, np.int32)
        cu[1:] = np.cumsum([len(t) for t in xs])
        prefill = PrefillBatch(torch.cat(xs, 0), cu, p.prefix_len[prefill_reqs].astype(np.int32), pt_p)
    if w.decode is not None and decode_reqs:
        dd = w.decode
        needs = [_pages_for(int(dd.ctx_len[j]) + 1, ps) for j in decode_reqs]
        pt_d = remap([dd.page_table[j] for j in decode_reqs], needs)
        decode = DecodeBatch(dd.x[decode_reqs], dd.ctx_len[decode_reqs].astype(np.int32), pt_d)
    idx = torch.as_tensor(pages, dtype=torch.long, device=w.k_pool.device)
    k_pool = w.k_pool.index_select(0, idx).cpu()
    v_pool = w.v_pool.index_select(0, idx).cpu()
    return Workload(w.name + "_subset", w.shape, w.seed, len(pages), prefill, decode, k_pool, v_pool,
                    notes={"pages": pages})


def poisson_trace(seed: int, rate: float, horizon_s: float, prompt_median: float = 1024.0, prompt_sigma: float = 0.8,
                  prompt_cap: int = 8192, output_median: float = 256.0, output_sigma: float = 0.7,
                  output_cap: int = 2048) -> List[tuple]:
    """Requests of the trace-driven configuration: Poisson arrivals at `rate` per second over `horizon_s`, prompt
    lengths lognormal(median, sigma) capped, output lengths lognormal(median, sigma) capped.  Returns
    (arrival_s, prompt_len, output_len) tuples in arrival order."""
    rng = np.random.default_rng([seed, 4242])
    out, t = [], 0.0
    while True:
        t += float(rng.exponential(1.0 / rate))
        if t >= horizon_s:
            return out
        prompt = int(min(prompt_cap, max(1.0, rng.lognormal(np.log(prompt_median), prompt_sigma))))
        output = int(min(output_cap, max(1.0, rng.lognormal(np.log(output_median), output_sigma))))
        out.append((t, prompt, output))

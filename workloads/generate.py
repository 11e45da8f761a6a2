"""Synthetic workloads shaped like the paper's serving scenarios.

Everything here is seeded random-number drawing and byte movement.  The five
named configurations mirror the shapes the paper measures on (Llama-3-8B style
GQA 32/8 heads of width 128, Llama-2-7B style MHA 32/32, half of the KV heads
streaming, 64-token physical pages made of 16-token logical pages, a constant
4096-token page budget, selector reuse interval 4, contexts from 32K to 256K
tokens).  They stand in for the prompts of the long-context suites and for the
Q/K/V a trained model would produce, neither of which is available.

No function in this module computes statistics, scores, softmax or attention.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import List, Optional, Sequence

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int = 128
    dtype: str = "fp16"  # "fp16" | "bf16"
    page_size: int = 64  # N_P
    logical_page_size: int = 16  # N_L
    streaming_kv_heads: Sequence[int] = ()  # indices of streaming KV heads
    sink_tokens: int = 128
    local_tokens: int = 512
    budget_tokens: int = 4096
    reuse_interval: int = 4  # C
    decode_steps: int = 16
    context: int = 0  # prompt length of every sequence (0: use lengths)
    lengths: Optional[Sequence[int]] = None  # explicit per-sequence prompt lengths
    length_range: Optional[Sequence[int]] = None  # log-uniform [lo, hi]
    prefill_tokens: int = 0  # tokens per sequence for the prefill part
    needles_per_seq: int = 0
    k_channel_scale: Optional[Sequence[float]] = None  # U(lo, hi) per (kv head, channel)
    seed: int = 1000
    pool_slack: float = 0.03

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float16 if self.dtype == "fp16" else torch.bfloat16

    @property
    def group(self) -> int:
        return self.num_q_heads // self.num_kv_heads

    def streaming_flags(self) -> List[int]:
        return [1 if h in set(self.streaming_kv_heads) else 0 for h in range(self.num_kv_heads)]


CONFIGS = {
    # One layer, prefill of 2048 tokens then one decode step; full oracle comparison.
    "cfg1": Workload(
        name="cfg1", batch=1, num_q_heads=8, num_kv_heads=2, dtype="fp16",
        streaming_kv_heads=(0,), sink_tokens=64, local_tokens=256, budget_tokens=512,
        reuse_interval=1, decode_steps=1, context=2048, prefill_tokens=2048, seed=1001,
        pool_slack=0.25,
    ),
    # Decode only, Llama-3-8B shaped, batch 16 at 32K context.
    "cfg2": Workload(
        name="cfg2", batch=16, num_q_heads=32, num_kv_heads=8, dtype="fp16",
        streaming_kv_heads=(0, 1, 2, 3), sink_tokens=128, local_tokens=512, budget_tokens=4096,
        reuse_interval=4, decode_steps=16, context=32768, seed=1002,
    ),
    # Prefill only, 64K tokens, bf16.
    "cfg3": Workload(
        name="cfg3", batch=1, num_q_heads=32, num_kv_heads=8, dtype="bf16",
        streaming_kv_heads=(0, 1, 2, 3), sink_tokens=128, local_tokens=512, budget_tokens=4096,
        decode_steps=0, context=0, prefill_tokens=65536, seed=1003,
    ),
    # Long-context decode with planted needles.
    "cfg4": Workload(
        name="cfg4", batch=4, num_q_heads=32, num_kv_heads=8, dtype="fp16",
        streaming_kv_heads=(0, 1, 2, 3), sink_tokens=128, local_tokens=512, budget_tokens=4096,
        reuse_interval=4, decode_steps=16, context=262144, needles_per_seq=8, seed=1004,
    ),
    # Ragged MHA decode batch with outlier channels on K.
    "cfg5": Workload(
        name="cfg5", batch=32, num_q_heads=32, num_kv_heads=32, dtype="fp16",
        streaming_kv_heads=tuple(range(16)), sink_tokens=128, local_tokens=512, budget_tokens=2048,
        reuse_interval=4, decode_steps=16, length_range=(4096, 131072),
        k_channel_scale=(0.5, 4.0), seed=1005,
    ),
}


def get_config(name: str, **overrides) -> Workload:
    """Return a named configuration, optionally shrunk (e.g. context=4096) for tests."""
    return replace(CONFIGS[name], **overrides)


@dataclass
class DecodeInputs:
    workload: Workload
    k_pool: torch.Tensor  # [num_pages, Hkv, N_P, D]
    v_pool: torch.Tensor  # [num_pages, Hkv, N_P, D]
    page_table: torch.Tensor  # [B, max_pages_per_seq] int32
    prompt_lens: torch.Tensor  # [B] int32, KV length before the first decode step
    q: torch.Tensor  # [steps, B, H, D]
    needle_pos: Optional[torch.Tensor] = None  # [B, needles] int64 token positions
    k_scale: Optional[torch.Tensor] = None  # [Hkv, D] fp32

    @property
    def num_pages(self) -> int:
        return self.k_pool.shape[0]

    @property
    def max_pages_per_seq(self) -> int:
        return self.page_table.shape[1]

    def seq_lens_at(self, step: int) -> torch.Tensor:
        """KV length seen by decode step `step` (the step's own token is already in the pool)."""
        return (self.prompt_lens + (step + 1)).to(torch.int32)


@dataclass
class PrefillInputs:
    workload: Workload
    q: torch.Tensor  # [total, H, D]
    k: torch.Tensor  # [total, Hkv, D]
    v: torch.Tensor  # [total, Hkv, D]
    cu_seqlens: torch.Tensor  # [B + 1] int32


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _randn_into(out: torch.Tensor, gen: torch.Generator, scale: Optional[torch.Tensor] = None,
                chunk_elems: int = 1 << 26) -> None:
    """Fill `out` (fp16/bf16, first dim = pages or tokens) with N(0,1) rounded to its dtype."""
    rows = out.shape[0]
    per_row = out[0].numel() if rows else 1
    step = max(1, chunk_elems // max(1, per_row))
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        x = torch.randn((r1 - r0,) + tuple(out.shape[1:]), generator=gen, device=out.device,
                        dtype=torch.float32)
        if scale is not None:
            x = x * scale
        out[r0:r1] = x.to(out.dtype)


def _prompt_lengths(w: Workload, gen_cpu: torch.Generator) -> List[int]:
    if w.lengths is not None:
        return [int(x) for x in w.lengths]
    if w.length_range is not None:
        lo, hi = w.length_range
        u = torch.rand(w.batch, generator=gen_cpu, dtype=torch.float64)
        return [int(round(math.exp(math.log(lo) + float(x) * (math.log(hi) - math.log(lo))))) for x in u]
    return [int(w.context)] * w.batch


def make_decode_inputs(w: Workload, device="cpu") -> DecodeInputs:
    """Paged KV pool, page table and per-step queries for a decode workload.

    The pool already holds the K/V of the `decode_steps` tokens that the steps
    will append; a step only sees them once the sequence length covers them.
    Page tables are one random permutation of the shared pool; entries past a
    sequence's last page hold valid but unrelated page ids.
    """
    dev = torch.device(device)
    gen_cpu = _gen(w.seed, "cpu")
    gen = gen_cpu if dev.type == "cpu" else _gen(w.seed, dev)
    lens = _prompt_lengths(w, gen_cpu)
    steps = max(1, w.decode_steps)
    np_ = w.page_size
    pages_per_seq = [(l + steps + np_ - 1) // np_ for l in lens]
    max_pages = max(pages_per_seq)
    used = sum(pages_per_seq)
    num_pages = used + max(2, int(math.ceil(used * w.pool_slack)))

    perm = torch.randperm(num_pages, generator=gen_cpu, dtype=torch.int64)
    page_table = torch.randint(0, num_pages, (w.batch, max_pages), generator=gen_cpu, dtype=torch.int64)
    off = 0
    for b, pb in enumerate(pages_per_seq):
        page_table[b, :pb] = perm[off:off + pb]
        off += pb

    k_scale = None
    if w.k_channel_scale is not None:
        lo, hi = w.k_channel_scale
        k_scale = lo + (hi - lo) * torch.rand((w.num_kv_heads, w.head_dim), generator=gen_cpu,
                                              dtype=torch.float32)
    shape = (num_pages, w.num_kv_heads, np_, w.head_dim)
    k_pool = torch.empty(shape, dtype=w.torch_dtype, device=dev)
    v_pool = torch.empty(shape, dtype=w.torch_dtype, device=dev)
    _randn_into(k_pool, gen, None if k_scale is None else k_scale.to(dev)[None, :, None, :])
    _randn_into(v_pool, gen)
    q = torch.empty((steps, w.batch, w.num_q_heads, w.head_dim), dtype=w.torch_dtype, device=dev)
    _randn_into(q, gen)

    needle_pos = None
    if w.needles_per_seq > 0:
        # Needle keys copy 4x the step-0 query of the first head of each group into
        # distinct pages strictly between the sink pages and the local window.
        s_pages = (w.sink_tokens + np_ - 1) // np_
        w_pages = (w.local_tokens + np_ - 1) // np_
        streaming = set(w.streaming_kv_heads)
        needle_pos = torch.empty((w.batch, w.needles_per_seq), dtype=torch.int64)
        for b, l in enumerate(lens):
            lo_page = s_pages
            hi_page = (l + 1 + np_ - 1) // np_ - w_pages  # exclusive
            cand = torch.randperm(hi_page - lo_page, generator=gen_cpu)[: w.needles_per_seq] + lo_page
            slot = torch.randint(0, np_, (w.needles_per_seq,), generator=gen_cpu)
            needle_pos[b] = cand * np_ + slot
            for j in range(w.needles_per_seq):
                pos = int(needle_pos[b, j])
                phys = int(page_table[b, pos // np_])
                for hk in range(w.num_kv_heads):
                    if hk in streaming:
                        continue
                    qv = q[0, b, hk * w.group].to(torch.float32) * 4.0
                    k_pool[phys, hk, pos % np_] = qv.to(w.torch_dtype)

    return DecodeInputs(
        workload=w,
        k_pool=k_pool,
        v_pool=v_pool,
        page_table=page_table.to(torch.int32).to(dev),
        prompt_lens=torch.tensor(lens, dtype=torch.int32, device=dev),
        q=q,
        needle_pos=needle_pos,
        k_scale=k_scale,
    )


def make_prefill_inputs(w: Workload, device="cpu", lengths: Optional[Sequence[int]] = None) -> PrefillInputs:
    """Q/K/V of a (possibly ragged) prefill batch, tokens of all sequences concatenated."""
    dev = torch.device(device)
    gen = _gen(w.seed + 500, "cpu") if dev.type == "cpu" else _gen(w.seed + 500, dev)
    lens = [int(x) for x in lengths] if lengths is not None else [int(w.prefill_tokens)] * w.batch
    total = sum(lens)
    q = torch.empty((total, w.num_q_heads, w.head_dim), dtype=w.torch_dtype, device=dev)
    k = torch.empty((total, w.num_kv_heads, w.head_dim), dtype=w.torch_dtype, device=dev)
    v = torch.empty((total, w.num_kv_heads, w.head_dim), dtype=w.torch_dtype, device=dev)
    _randn_into(q, gen)
    _randn_into(k, gen)
    _randn_into(v, gen)
    cu = [0]
    for l in lens:
        cu.append(cu[-1] + l)
    return PrefillInputs(workload=w, q=q, k=k, v=v,
                         cu_seqlens=torch.tensor(cu, dtype=torch.int32, device=dev))


def scatter_prefill_kv_to_pages(k: torch.Tensor, v: torch.Tensor, cu_seqlens: Sequence[int],
                                k_pool: torch.Tensor, v_pool: torch.Tensor,
                                page_table: torch.Tensor) -> None:
    """Copy contiguous prefill K/V ([total, Hkv, D]) into the paged pool (pure data movement)."""
    np_ = k_pool.shape[2]
    cu = [int(x) for x in cu_seqlens]
    for b in range(len(cu) - 1):
        n = cu[b + 1] - cu[b]
        pos = torch.arange(n, device=k.device)
        phys = page_table[b].to(torch.int64)[pos // np_]
        slot = pos % np_
        k_pool[phys, :, slot] = k[cu[b]:cu[b + 1]]
        v_pool[phys, :, slot] = v[cu[b]:cu[b + 1]]

"""Host-side decode loop with reusable page selection (Sec. 3.5.3).

The selector runs on the first step of every chunk of C decode steps and its index table is
reused for the other C - 1 steps.  The key statistics of the logical pages that received tokens since
the previous run are refreshed by the selector run itself (inside the scoring kernel) or, optionally,
by a separate launch right before it; every step runs the sparse decode kernel.  This class only owns buffers and
calls the C-ABI entry points in that order; all arithmetic happens in the HIP kernels.
"""
from __future__ import annotations

from typing import Optional, Sequence

import torch

from . import binding as B


class DecodeSession:
    def __init__(self, k_pool: torch.Tensor, v_pool: torch.Tensor, page_table: torch.Tensor,
                 num_q_heads: int, streaming_flags: Sequence[int], sink_tokens: int, local_tokens: int,
                 budget_tokens: int, logical_page_size: int = 16, reuse_interval: int = 4,
                 sm_scale: float = 0.0, want_scores: bool = False, want_lse: bool = False,
                 fused_stats: bool = True, k_pool_stream: Optional[torch.Tensor] = None,
                 v_pool_stream: Optional[torch.Tensor] = None, ring_table: Optional[torch.Tensor] = None,
                 kv_bits: int = 16, dtype: Optional[torch.dtype] = None):
        """k_pool / v_pool hold every KV head, or only the non-streaming ones when the streaming heads live in
        the bounded pool k_pool_stream / v_pool_stream behind ring_table (two-way cache).  kv_bits = 8 or 4: the
        pools are uint8 [pages, heads, 64 * 128 * kv_bits / 8 + 256] (quantised pages, written by `append`), `dtype`
        names the 16-bit type of queries, outputs and statistics, and the statistics are kept current by `append`
        alone."""
        dev = k_pool.device
        if kv_bits != 16:
            num_pages, pool_heads, _ = k_pool.shape
            page_size, head_dim = 64, 128
            if dtype is None:
                raise ValueError("a session over quantised pages needs the 16-bit dtype of the layer")
        else:
            num_pages, pool_heads, page_size, head_dim = k_pool.shape
            dtype = k_pool.dtype
        self.kv_bits = kv_bits
        hkv = len(streaming_flags)
        batch, max_pages = page_table.shape
        self.desc = B.AttnDesc(num_q_heads=num_q_heads, num_kv_heads=hkv, streaming_flags=streaming_flags,
                               head_dim=head_dim, page_size=page_size, logical_page_size=logical_page_size,
                               dtype=dtype, sink_tokens=sink_tokens, local_tokens=local_tokens,
                               sm_scale=sm_scale)
        g = page_size // logical_page_size
        self.stats = torch.zeros((num_pages, pool_heads, g, 2, head_dim), dtype=dtype, device=dev)
        self.seq_lens = torch.zeros((batch,), dtype=torch.int32, device=dev)
        self.kv = B.PagedKV(k_pool, v_pool, self.stats, page_table, self.seq_lens,
                            pool_heads=0 if pool_heads == hkv else pool_heads, k_pool_stream=k_pool_stream,
                            v_pool_stream=v_pool_stream, ring_table=ring_table, kv_bits=kv_bits)
        self.budget_tokens = budget_tokens
        self.reuse_interval = max(1, reuse_interval)
        K = budget_tokens // page_size
        self.K = K
        self.sel_pages = torch.full((batch, hkv, K), -1, dtype=torch.int32, device=dev)
        self.sel_count = torch.zeros((batch, hkv), dtype=torch.int32, device=dev)
        self.sel_seq_len = torch.zeros((batch,), dtype=torch.int32, device=dev)
        self.scores = (torch.zeros((batch, hkv, max_pages), dtype=torch.float32, device=dev)
                       if want_scores else None)
        ws_sel = B.lserve_workspace_bytes(B.LSERVE_CALL_SELECT_PAGES, self.desc, batch, max_pages, K, 0)
        ws_dec = B.lserve_workspace_bytes(B.LSERVE_CALL_SPARSE_DECODE, self.desc, batch, max_pages, K, 0)
        self.ws_select = torch.empty((max(ws_sel, 16),), dtype=torch.uint8, device=dev)
        self.ws_decode = torch.zeros((max(ws_dec, 16),), dtype=torch.uint8, device=dev)  # zero once: arrival counters
        self.out = torch.empty((batch, num_q_heads, head_dim), dtype=dtype, device=dev)
        self.lse = torch.empty((batch, num_q_heads), dtype=torch.float32, device=dev) if want_lse else None
        self.steps_since_selection: Optional[int] = None
        # True: the selector rebuilds the stale logical pages itself; False: a separate statistics launch
        self.fused_stats = fused_stats
        # Key statistics are consumed only by the selector, so the logical pages touched since the
        # last selector run are refreshed in one call right before the next run.
        self._stats_from: Optional[torch.Tensor] = None
        self._stats_tokens = 0

    def set_seq_lens(self, seq_lens: torch.Tensor) -> None:
        """Point the session at the caller's current lengths (device int32 [batch], not copied)."""
        self.seq_lens = seq_lens
        self.kv.seq_lens = seq_lens

    def append(self, k_new: torch.Tensor, v_new: torch.Tensor, cu_new: torch.Tensor, start_pos: torch.Tensor,
               max_new_per_seq: int) -> None:
        """Write new tokens' K/V into the pages (quantising them for 8-bit pools) and fold the keys into the
        statistics in the same pass."""
        B.lserve_append_kv(self.desc, self.kv, k_new, v_new, cu_new, start_pos, max_new_per_seq)

    def build_stats_full(self) -> None:
        """Statistics of every logical page below the current lengths (after prefill)."""
        B.lserve_build_page_stats(self.desc, self.kv, None, 0)

    def update_stats_tail(self, prev_seq_lens: torch.Tensor, max_new_tokens: int = 1) -> None:
        """Refresh the logical pages that hold tokens [prev_seq_lens, seq_lens) of every sequence."""
        np_ = self.desc.page_size
        tail_pages = 1 if max_new_tokens == 1 else (max_new_tokens + np_ - 1) // np_ + 1
        B.lserve_build_page_stats(self.desc, self.kv, prev_seq_lens, tail_pages)

    def select(self, q: torch.Tensor, stats_valid_len: Optional[torch.Tensor] = None) -> None:
        """Run the selector.  With `stats_valid_len` (device int32 [batch]) the statistics of the logical
        pages holding tokens at or above it are rebuilt inside the scoring kernel."""
        B.lserve_select_pages(self.desc, self.kv, q, self.budget_tokens, self.sel_pages, self.sel_count,
                              self.sel_seq_len, self.scores, self.ws_select, stats_valid_len=stats_valid_len)
        self.steps_since_selection = 0

    def decode(self, q: torch.Tensor) -> torch.Tensor:
        B.lserve_sparse_decode(self.desc, self.kv, q, self.sel_pages, self.sel_count, self.sel_seq_len,
                               self.out, self.lse, self.ws_decode)
        return self.out

    def step(self, q: torch.Tensor, seq_lens: torch.Tensor, prev_seq_lens: torch.Tensor,
             run_decode: bool = True) -> torch.Tensor:
        """One decode step.

        The new token's K/V are already in the pool; `seq_lens` counts it and `prev_seq_lens` is the
        length before it was appended (both device int32 [batch], 16-byte aligned, not copied, and
        left unchanged by the caller until the next selector run).
        """
        self.set_seq_lens(seq_lens)
        if self._stats_from is None:
            self._stats_from = prev_seq_lens
        self._stats_tokens += 1
        if self.steps_since_selection is None or self.steps_since_selection >= self.reuse_interval:
            if self.kv_bits != 16:
                self.select(q)  # quantised pages: `append` has kept the statistics current
            elif self.fused_stats:
                self.select(q, stats_valid_len=self._stats_from)
            else:
                self.update_stats_tail(self._stats_from, self._stats_tokens)
                self.select(q)
            self._stats_from, self._stats_tokens = seq_lens, 0
        self.steps_since_selection += 1
        return self.decode(q) if run_decode else self.out  # run_decode=False: selector side only (timing)

    def restart(self) -> None:
        """Forget the selection and the pending statistics range (start of a new episode)."""
        self.steps_since_selection = None
        self._stats_from, self._stats_tokens = None, 0

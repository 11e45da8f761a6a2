"""ctypes binding of liblserve.so: argument marshalling only, every step runs in the HIP kernels."""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# LSERVE_LIBRARY points at another build of the same library (e.g. an instrumented one)
_LIB_PATH = os.environ.get("LSERVE_LIBRARY") or os.path.join(_HERE, "liblserve.so")
_lib = None

LSERVE_CALL_BUILD_PAGE_STATS = 0
LSERVE_CALL_SELECT_PAGES = 1
LSERVE_CALL_SPARSE_PREFILL = 2
LSERVE_CALL_SPARSE_DECODE = 3

EXPORTED_SYMBOLS = (
    "lserve_build_page_stats",
    "lserve_select_pages",
    "lserve_sparse_prefill",
    "lserve_sparse_decode",
    "lserve_append_kv",
    "lserve_sparse_prefill_masked",
    "lserve_sparse_prefill_paged",
    "lserve_sparse_prefill_chunk",
    "lserve_paged_prefill_workspace_bytes",
    "lserve_masked_prefill_workspace_bytes",
    "BlockMask",
    "lserve_workspace_bytes",
    "lserve_strerror",
    "lserve_last_hip_error",
    "lserve_init",
    "lserve_sparse_decode_noalloc",
    "lserve_probe_decode_read",
)


class LserveError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where} failed with code {code}: {lserve_strerror(code)}"
                         + (f" (hipError_t {lserve_last_hip_error()})" if code == -4 else ""))


class _CAttnDesc(ctypes.Structure):
    _fields_ = [
        ("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
        ("page_size", ctypes.c_int32), ("logical_page_size", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("sink_tokens", ctypes.c_int32), ("local_tokens", ctypes.c_int32),
        ("kv_head_is_streaming", ctypes.POINTER(ctypes.c_uint8)), ("sm_scale", ctypes.c_float),
    ]


class _CPagedKV(ctypes.Structure):
    _fields_ = [
        ("k_pool", ctypes.c_void_p), ("v_pool", ctypes.c_void_p), ("stats", ctypes.c_void_p),
        ("page_table", ctypes.c_void_p), ("seq_lens", ctypes.c_void_p),
        ("batch", ctypes.c_int32), ("max_pages_per_seq", ctypes.c_int32), ("num_pages", ctypes.c_int32),
        ("pool_heads", ctypes.c_int32),
        ("k_pool_stream", ctypes.c_void_p), ("v_pool_stream", ctypes.c_void_p), ("ring_table", ctypes.c_void_p),
        ("num_pages_stream", ctypes.c_int32), ("kv_bits", ctypes.c_int32),
    ]


class _CBlockMask(ctypes.Structure):
    _fields_ = [
        ("head_mask", ctypes.c_void_p), ("q_tile_start", ctypes.c_void_p), ("row_ptr", ctypes.c_void_p),
        ("cols", ctypes.c_void_p),
        ("num_masks", ctypes.c_int32), ("rows_per_mask", ctypes.c_int32), ("nnz", ctypes.c_int32),
    ]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load liblserve.so; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2502_14866_amd.build` "
                "(or __graft_entry__.build()); there is no CPU fallback")
        lib = ctypes.CDLL(_LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        dp, kp = ctypes.POINTER(_CAttnDesc), ctypes.POINTER(_CPagedKV)
        lib.lserve_build_page_stats.argtypes = [dp, kp, vp, i32, vp]
        lib.lserve_select_pages.argtypes = [dp, kp, vp, i32, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.lserve_sparse_prefill.argtypes = [dp, vp, vp, vp, vp, i32, i32, i32, vp, vp, vp, sz, vp]
        lib.lserve_sparse_decode.argtypes = [dp, kp, vp, vp, vp, vp, i32, vp, vp, vp, sz, vp]
        lib.lserve_append_kv.argtypes = [dp, kp, vp, vp, vp, vp, i32, vp]
        lib.lserve_append_kv.restype = ctypes.c_int
        mp = ctypes.POINTER(_CBlockMask)
        lib.lserve_sparse_prefill_masked.argtypes = [dp, mp, vp, vp, vp, vp, i32, i32, i32, vp, vp, vp, sz, vp]
        lib.lserve_sparse_prefill_masked.restype = ctypes.c_int
        lib.lserve_masked_prefill_workspace_bytes.argtypes = [dp, i32, i32, i32, i32, i32]
        lib.lserve_masked_prefill_workspace_bytes.restype = ctypes.c_size_t
        lib.lserve_sparse_prefill_paged.argtypes = [dp, kp, vp, vp, i32, i32, i32, vp, vp, vp, sz, vp]
        lib.lserve_sparse_prefill_paged.restype = ctypes.c_int
        lib.lserve_sparse_prefill_chunk.argtypes = [dp, kp, vp, vp, vp, vp, i32, i32, vp, vp, vp]
        lib.lserve_sparse_prefill_chunk.restype = ctypes.c_int
        lib.lserve_paged_prefill_workspace_bytes.argtypes = [dp, i32, i32]
        lib.lserve_paged_prefill_workspace_bytes.restype = ctypes.c_size_t
        lib.lserve_workspace_bytes.argtypes = [ctypes.c_int, dp, i32, i32, i32, i32]
        lib.lserve_workspace_bytes.restype = sz
        lib.lserve_strerror.argtypes = [ctypes.c_int]
        lib.lserve_strerror.restype = ctypes.c_char_p
        lib.lserve_last_hip_error.restype = ctypes.c_int
        lib.lserve_sparse_decode_noalloc.argtypes = [dp, kp, vp, vp, vp, vp, i32, vp, vp, vp]
        lib.lserve_sparse_decode_noalloc.restype = ctypes.c_int
        lib.lserve_probe_decode_read.argtypes = [dp, kp, vp, vp, vp, i32, vp]
        lib.lserve_probe_decode_read.restype = ctypes.c_int
        lib.lserve_init.argtypes = []
        lib.lserve_init.restype = ctypes.c_int
        for name in ("lserve_build_page_stats", "lserve_select_pages", "lserve_sparse_prefill",
                     "lserve_sparse_decode"):
            getattr(lib, name).restype = ctypes.c_int
        _lib = lib
    return _lib


@dataclass
class AttnDesc:
    """Mirror of lserve_attn_desc."""
    num_q_heads: int
    num_kv_heads: int
    streaming_flags: Sequence[int]
    head_dim: int = 128
    page_size: int = 64
    logical_page_size: int = 16
    dtype: torch.dtype = torch.float16
    sink_tokens: int = 128
    local_tokens: int = 512
    sm_scale: float = 0.0

    def __post_init__(self):
        flags = [1 if f else 0 for f in self.streaming_flags]
        self._flags = (ctypes.c_uint8 * max(1, len(flags)))(*flags)
        self._c = _CAttnDesc(
            self.num_q_heads, self.num_kv_heads, self.head_dim, self.page_size, self.logical_page_size,
            {torch.float16: 0, torch.bfloat16: 1}.get(self.dtype, -1), self.sink_tokens, self.local_tokens,
            ctypes.cast(self._flags, ctypes.POINTER(ctypes.c_uint8)), float(self.sm_scale))

    def c(self):
        return ctypes.byref(self._c)


@dataclass
class PagedKV:
    """Mirror of lserve_paged_kv; keeps the tensors alive."""
    k_pool: Optional[torch.Tensor]
    v_pool: Optional[torch.Tensor]
    stats: Optional[torch.Tensor]
    page_table: torch.Tensor
    seq_lens: torch.Tensor
    # two-way cache: heads per page of the main pool (0 = all KV heads) and the streaming heads' bounded pool
    pool_heads: int = 0
    k_pool_stream: Optional[torch.Tensor] = None
    v_pool_stream: Optional[torch.Tensor] = None
    ring_table: Optional[torch.Tensor] = None
    # 16: pools of the layer's 16-bit dtype [pages, heads, N_P, D]; 8 or 4: quantised pages, uint8
    # [pages, heads, 64 * D * kv_bits / 8 + 256]
    kv_bits: int = 16

    def c(self):
        num_pages = 0
        for t in (self.k_pool, self.v_pool, self.stats):
            if t is not None:
                num_pages = t.shape[0]
        num_pages_stream = 0 if self.k_pool_stream is None else self.k_pool_stream.shape[0]
        self._c = _CPagedKV(_ptr(self.k_pool), _ptr(self.v_pool), _ptr(self.stats), _ptr(self.page_table),
                            _ptr(self.seq_lens), self.page_table.shape[0], self.page_table.shape[1], num_pages,
                            self.pool_heads, _ptr(self.k_pool_stream), _ptr(self.v_pool_stream),
                            _ptr(self.ring_table), num_pages_stream, self.kv_bits)
        return ctypes.byref(self._c)


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("lserve binding takes contiguous tensors")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _check(rc: int, where: str) -> None:
    if rc != 0:
        raise LserveError(rc, where)


def lserve_strerror(code: int) -> str:
    return load_library().lserve_strerror(int(code)).decode()


def lserve_last_hip_error() -> int:
    return int(load_library().lserve_last_hip_error())


def lserve_init() -> None:
    _check(load_library().lserve_init(), "lserve_init")


def lserve_workspace_bytes(which_call: int, desc: AttnDesc, batch: int = 0, max_pages_per_seq: int = 0,
                           sel_stride_or_budget_pages: int = 0, total_tokens: int = 0) -> int:
    return int(load_library().lserve_workspace_bytes(which_call, desc.c(), batch, max_pages_per_seq,
                                                     sel_stride_or_budget_pages, total_tokens))


def lserve_build_page_stats(desc: AttnDesc, kv: PagedKV, start_pos: Optional[torch.Tensor] = None,
                            max_tail_pages: int = 0, stream=None) -> None:
    _check(load_library().lserve_build_page_stats(desc.c(), kv.c(), _ptr(start_pos), max_tail_pages,
                                                  _stream(stream)), "lserve_build_page_stats")


def lserve_append_kv(desc: AttnDesc, kv: PagedKV, k_new: torch.Tensor, v_new: torch.Tensor, cu_new: torch.Tensor,
                     start_pos: torch.Tensor, max_new_per_seq: int, stream=None) -> None:
    _check(load_library().lserve_append_kv(desc.c(), kv.c(), _ptr(k_new), _ptr(v_new), _ptr(cu_new), _ptr(start_pos),
                                           max_new_per_seq, _stream(stream)), "lserve_append_kv")


def lserve_select_pages(desc: AttnDesc, kv: PagedKV, q: torch.Tensor, budget_tokens: int,
                        sel_pages: torch.Tensor, sel_count: torch.Tensor, sel_seq_len: torch.Tensor,
                        scores_out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                        stream=None, stats_valid_len: Optional[torch.Tensor] = None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load_library().lserve_select_pages(desc.c(), kv.c(), _ptr(q), budget_tokens, _ptr(stats_valid_len),
                                              _ptr(sel_pages),
                                              _ptr(sel_count), _ptr(sel_seq_len), _ptr(scores_out),
                                              _ptr(workspace), ws_bytes, _stream(stream)), "lserve_select_pages")


def lserve_sparse_prefill(desc: AttnDesc, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor,
                          cu_seqlens: torch.Tensor, max_seqlen: int, out: torch.Tensor,
                          lse_out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                          stream=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load_library().lserve_sparse_prefill(desc.c(), _ptr(q), _ptr(k), _ptr(v), _ptr(cu_seqlens),
                                                cu_seqlens.shape[0] - 1, q.shape[0], max_seqlen, _ptr(out),
                                                _ptr(lse_out), _ptr(workspace), ws_bytes, _stream(stream)),
           "lserve_sparse_prefill")


@dataclass
class BlockMask:
    """Mirror of lserve_block_mask (device int32 tensors); keeps the tensors alive."""
    head_mask: torch.Tensor
    q_tile_start: torch.Tensor
    row_ptr: torch.Tensor
    cols: Optional[torch.Tensor]
    num_masks: int
    rows_per_mask: int

    @property
    def nnz(self) -> int:
        return 0 if self.cols is None else int(self.cols.numel())

    def c(self):
        self._c = _CBlockMask(_ptr(self.head_mask), _ptr(self.q_tile_start), _ptr(self.row_ptr), _ptr(self.cols),
                              self.num_masks, self.rows_per_mask, self.nnz)
        return ctypes.byref(self._c)


def lserve_masked_prefill_workspace_bytes(desc: AttnDesc, batch: int, total_tokens: int, max_seqlen: int,
                                          num_masks: int, nnz: int) -> int:
    return int(load_library().lserve_masked_prefill_workspace_bytes(desc.c(), batch, total_tokens, max_seqlen,
                                                                    num_masks, nnz))


def lserve_sparse_prefill_masked(desc: AttnDesc, mask: BlockMask, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor,
                                 cu_seqlens: torch.Tensor, max_seqlen: int, out: torch.Tensor,
                                 lse_out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                                 stream=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load_library().lserve_sparse_prefill_masked(desc.c(), mask.c(), _ptr(q), _ptr(k), _ptr(v),
                                                       _ptr(cu_seqlens), cu_seqlens.shape[0] - 1, q.shape[0],
                                                       max_seqlen, _ptr(out), _ptr(lse_out), _ptr(workspace),
                                                       ws_bytes, _stream(stream)),
           "lserve_sparse_prefill_masked")


def lserve_paged_prefill_workspace_bytes(desc: AttnDesc, batch: int, max_pages_per_seq: int) -> int:
    return int(load_library().lserve_paged_prefill_workspace_bytes(desc.c(), batch, max_pages_per_seq))


def lserve_sparse_prefill_paged(desc: AttnDesc, kv: PagedKV, q: torch.Tensor, cu_q: torch.Tensor,
                                max_new_per_seq: int, max_seqlen: int, out: torch.Tensor,
                                lse_out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                                stream=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load_library().lserve_sparse_prefill_paged(desc.c(), kv.c(), _ptr(q), _ptr(cu_q), q.shape[0],
                                                      max_new_per_seq, max_seqlen, _ptr(out), _ptr(lse_out),
                                                      _ptr(workspace), ws_bytes, _stream(stream)),
           "lserve_sparse_prefill_paged")


def lserve_sparse_prefill_chunk(desc: AttnDesc, kv: PagedKV, q: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor,
                                cu_new: torch.Tensor, max_new_per_seq: int, out: torch.Tensor,
                                lse_out: Optional[torch.Tensor] = None, stream=None) -> None:
    _check(load_library().lserve_sparse_prefill_chunk(desc.c(), kv.c(), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(cu_new),
                                                      q.shape[0], max_new_per_seq, _ptr(out), _ptr(lse_out),
                                                      _stream(stream)), "lserve_sparse_prefill_chunk")


def lserve_sparse_decode(desc: AttnDesc, kv: PagedKV, q: torch.Tensor, sel_pages: Optional[torch.Tensor],
                         sel_count: Optional[torch.Tensor], sel_seq_len: Optional[torch.Tensor],
                         out: torch.Tensor, lse_out: Optional[torch.Tensor] = None,
                         workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    sel_stride = 0 if sel_pages is None else sel_pages.shape[-1]
    _check(load_library().lserve_sparse_decode(desc.c(), kv.c(), _ptr(q), _ptr(sel_pages), _ptr(sel_count),
                                               _ptr(sel_seq_len), sel_stride, _ptr(out), _ptr(lse_out),
                                               _ptr(workspace), ws_bytes, _stream(stream)), "lserve_sparse_decode")


def lserve_sparse_decode_noalloc(desc: AttnDesc, kv: PagedKV, q: torch.Tensor, sel_pages: Optional[torch.Tensor],
                                 sel_count: Optional[torch.Tensor], sel_seq_len: Optional[torch.Tensor],
                                 out: torch.Tensor, lse_out: Optional[torch.Tensor] = None, stream=None) -> None:
    sel_stride = 0 if sel_pages is None else sel_pages.shape[-1]
    _check(load_library().lserve_sparse_decode_noalloc(desc.c(), kv.c(), _ptr(q), _ptr(sel_pages), _ptr(sel_count),
                                                       _ptr(sel_seq_len), sel_stride, _ptr(out), _ptr(lse_out),
                                                       _stream(stream)), "lserve_sparse_decode_noalloc")


def lserve_probe_decode_read(desc: AttnDesc, kv: PagedKV, sel_pages: Optional[torch.Tensor],
                             sel_count: Optional[torch.Tensor], sel_seq_len: Optional[torch.Tensor], stream=None) -> None:
    sel_stride = 0 if sel_pages is None else sel_pages.shape[-1]
    _check(load_library().lserve_probe_decode_read(desc.c(), kv.c(), _ptr(sel_pages), _ptr(sel_count), _ptr(sel_seq_len),
                                                   sel_stride, _stream(stream)), "lserve_probe_decode_read")

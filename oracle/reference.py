"""ctypes binding of the C oracle (oracle/lserve_oracle.c).

TEST INFRASTRUCTURE ONLY: argument marshalling for the plain double-precision CPU
definitions of key statistics, page scores (Eq. 2), top-K page selection, paged
sparse decode and block-sparse prefill (Eq. 1 under the block mask of Sec. 3.1).
Inputs are CPU torch tensors in fp16 / bf16 storage and int32 tables; outputs are
float64 / int32 numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lserve_oracle.c")
_LIB = os.path.join(_HERE, "liblserve_oracle.so")
_lib = None


def build_oracle(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP over independent rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build_oracle()
        lib = ctypes.CDLL(_LIB)
        lib.oracle_widen.restype = ctypes.c_double
        lib.oracle_widen.argtypes = [ctypes.c_uint16, ctypes.c_int]
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_count_nonempty_tiles.restype = ctypes.c_longlong
        lib.oracle_count_nonempty_tiles.argtypes = [ctypes.c_int] * 5
        lib.oracle_block_sparse_speedup.restype = ctypes.c_double
        lib.oracle_block_sparse_speedup.argtypes = [ctypes.c_longlong, ctypes.c_longlong]
        _lib = lib
    return _lib


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float16:
        return 0
    if t.dtype == torch.bfloat16:
        return 1
    raise TypeError(f"oracle takes fp16 or bf16 storage, got {t.dtype}")


def _bits(t: torch.Tensor) -> np.ndarray:
    """Raw 16-bit patterns of a CPU fp16/bf16 tensor, without copying."""
    assert t.device.type == "cpu"
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


def _i32(t) -> np.ndarray:
    if isinstance(t, torch.Tensor):
        t = t.cpu().numpy()
    return np.ascontiguousarray(t, dtype=np.int32)


def _u8(x) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(x, dtype=np.uint8))


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def widen(bits: int, dtype: int) -> float:
    return float(_load().oracle_widen(int(bits), int(dtype)))


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def page_stats(k_pool: torch.Tensor, page_table, seq_lens, logical_page_size: int,
               stats: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Channel-wise max/min of the keys of every non-empty logical page.

    Returns [num_pages, Hkv, g, 2, D] in the pool's dtype (index 0 = max, 1 = min).
    """
    num_pages, Hkv, NP, D = k_pool.shape
    g = NP // logical_page_size
    if stats is None:
        stats = torch.zeros((num_pages, Hkv, g, 2, D), dtype=k_pool.dtype)
    pt, sl = _i32(page_table), _i32(seq_lens)
    kb, sb = _bits(k_pool), _bits(stats)
    assert sb.ctypes.data == stats.data_ptr()
    _load().oracle_page_stats(_p(kb), _p(pt), _p(sl), ctypes.c_int(pt.shape[0]),
                              ctypes.c_int(pt.shape[1]), ctypes.c_int(Hkv), ctypes.c_int(D),
                              ctypes.c_int(NP), ctypes.c_int(logical_page_size),
                              ctypes.c_int(_dtype_code(k_pool)), _p(sb))
    return stats


def append_kv(k_new: torch.Tensor, v_new: torch.Tensor, cu_new, start_pos, page_table,
              k_pool: torch.Tensor, v_pool: torch.Tensor) -> None:
    """Write new tokens ([total_new, Hkv, D]) into the paged pools in place at positions start_pos[b] + j."""
    num_pages, Hkv, NP, D = k_pool.shape
    assert k_pool.is_contiguous() and v_pool.is_contiguous()
    pt, cu, sp = _i32(page_table), _i32(cu_new), _i32(start_pos)
    kn, vn, kb, vb = _bits(k_new), _bits(v_new), _bits(k_pool), _bits(v_pool)
    assert kb.ctypes.data == k_pool.data_ptr() and vb.ctypes.data == v_pool.data_ptr()
    _load().oracle_append_kv(_p(kn), _p(vn), _p(cu), _p(sp), _p(pt), ctypes.c_int(pt.shape[0]),
                             ctypes.c_int(pt.shape[1]), ctypes.c_int(Hkv), ctypes.c_int(D),
                             ctypes.c_int(NP), _p(kb), _p(vb))


def page_scores(q: torch.Tensor, stats: torch.Tensor, page_table, seq_lens, page_size: int,
                want_logical: bool = False) -> Tuple[np.ndarray, Optional[np.ndarray]]:
    """Physical-page scores [B, Hkv, max_pages] (and per-head logical scores [B, H, max_pages, g])."""
    B, H, D = q.shape
    _, Hkv, g, _, _ = stats.shape
    pt, sl = _i32(page_table), _i32(seq_lens)
    max_pages = pt.shape[1]
    ps = np.zeros((B, Hkv, max_pages), dtype=np.float64)
    ls = np.zeros((B, H, max_pages, g), dtype=np.float64) if want_logical else None
    qb, sb = _bits(q), _bits(stats)
    _load().oracle_page_scores(_p(qb), _p(sb), _p(pt), _p(sl), ctypes.c_int(B),
                               ctypes.c_int(max_pages), ctypes.c_int(H), ctypes.c_int(Hkv),
                               ctypes.c_int(D), ctypes.c_int(page_size),
                               ctypes.c_int(page_size // g), ctypes.c_int(_dtype_code(q)),
                               _p(ps), _p(ls))
    return ps, ls


def select_pages(scores: np.ndarray, seq_lens, page_size: int, budget_tokens: int,
                 k_stride: Optional[int] = None):
    """Top-K pages per (sequence, KV head): (sel_pages [B,Hkv,k_stride], sel_count, sel_seq_len)."""
    B, Hkv, max_pages = scores.shape
    K = budget_tokens // page_size
    if k_stride is None:
        k_stride = K
    sl = _i32(seq_lens)
    scores = np.ascontiguousarray(scores, dtype=np.float64)
    sel = np.full((B, Hkv, k_stride), -1, dtype=np.int32)
    cnt = np.zeros((B, Hkv), dtype=np.int32)
    ssl = np.zeros((B,), dtype=np.int32)
    _load().oracle_select_pages(_p(scores), _p(sl), ctypes.c_int(B), ctypes.c_int(Hkv),
                                ctypes.c_int(max_pages), ctypes.c_int(page_size),
                                ctypes.c_int(budget_tokens), ctypes.c_int(k_stride),
                                _p(sel), _p(cnt), _p(ssl))
    return sel, cnt, ssl


def sparse_decode(q: torch.Tensor, k_pool: torch.Tensor, v_pool: torch.Tensor, page_table,
                  seq_lens, sel_pages, sel_count, sel_seq_len, streaming_flags: Sequence[int],
                  sink_tokens: int, local_tokens: int, sm_scale: Optional[float] = None):
    """Decode attention over the listed pages; returns (out [B,H,D] f64, lse [B,H] f64)."""
    B, H, D = q.shape
    _, Hkv, NP, _ = k_pool.shape
    pt, sl = _i32(page_table), _i32(seq_lens)
    sel, cnt, ssl = _i32(sel_pages), _i32(sel_count), _i32(sel_seq_len)
    flags = _u8(streaming_flags)
    out = np.zeros((B, H, D), dtype=np.float64)
    lse = np.zeros((B, H), dtype=np.float64)
    scale = float(sm_scale) if sm_scale else 1.0 / float(np.sqrt(D))
    qb, kb, vb = _bits(q), _bits(k_pool), _bits(v_pool)
    _load().oracle_sparse_decode(_p(qb), _p(kb), _p(vb), _p(pt), _p(sl), _p(sel), _p(cnt), _p(ssl),
                                 ctypes.c_int(sel.shape[-1]), _p(flags), ctypes.c_int(B),
                                 ctypes.c_int(pt.shape[1]), ctypes.c_int(H), ctypes.c_int(Hkv),
                                 ctypes.c_int(D), ctypes.c_int(NP), ctypes.c_int(_dtype_code(q)),
                                 ctypes.c_int(sink_tokens), ctypes.c_int(local_tokens),
                                 ctypes.c_double(scale), _p(out), _p(lse))
    return out, lse


def quantize_kv(x: torch.Tensor, bits: int = 8):
    """Asymmetric quantisation of KV features to `bits` bits (8 or 4), one (scale, zero point) per token
    and KV head (Sec. 3.2: scale factors and zero points are stored next to the token features).

    x [..., D] in fp16 / bf16 storage.  With lo / hi the smallest / largest feature of a token and
    top = 2^bits - 1:
        zero  = fp16(lo)                     (saturating at the largest finite fp16)
        scale = fp16((hi - zero) / top)      (same saturation)
        code  = clamp(rint((x - zero) / scale), 0, top),   all codes 0 when scale == 0
    and the stored code stands for the value code * scale + zero.  The arithmetic that decides a
    code runs in IEEE fp32 with round-to-nearest-even, the precision of the GPU kernel, so codes
    can be compared bit for bit.  Returns (codes uint8 [..., D], scale fp16 [...], zero fp16 [...]).
    """
    if bits not in (4, 8):
        raise ValueError("bits must be 4 or 8")
    top = np.float32(2 ** bits - 1)
    xf = x.detach().cpu().float().numpy().astype(np.float32)
    big = np.float32(65504.0)
    lo = xf.min(axis=-1)
    hi = xf.max(axis=-1)
    zero = np.clip(lo, -big, big).astype(np.float16)
    zf = zero.astype(np.float32)
    with np.errstate(over="ignore", invalid="ignore", divide="ignore"):
        scale = np.minimum((hi - zf) / top, big).astype(np.float16)
        sf = scale.astype(np.float32)
        t = (xf - zf[..., None]) / sf[..., None]
        codes = np.clip(np.rint(t), 0.0, top)
    codes = np.where(sf[..., None] > 0, codes, 0.0).astype(np.uint8)
    return codes, scale, zero


def quantize_q8(x: torch.Tensor):
    """quantize_kv with 8 bits."""
    return quantize_kv(x, 8)


def dequantize_q8(codes: np.ndarray, scale: np.ndarray, zero: np.ndarray) -> np.ndarray:
    """Values the stored codes stand for (any bit width): code * scale + zero, exact in float64."""
    return codes.astype(np.float64) * scale.astype(np.float64)[..., None] + zero.astype(np.float64)[..., None]


def sparse_decode_values(q: torch.Tensor, k_values: np.ndarray, v_values: np.ndarray, page_table,
                         seq_lens, sel_pages, sel_count, sel_seq_len, streaming_flags: Sequence[int],
                         sink_tokens: int, local_tokens: int, sm_scale: Optional[float] = None):
    """sparse_decode over pools given as float64 values [pages, Hkv, NP, D] (a dequantised cache)."""
    B, H, D = q.shape
    _, Hkv, NP, _ = k_values.shape
    pt, sl = _i32(page_table), _i32(seq_lens)
    sel, cnt, ssl = _i32(sel_pages), _i32(sel_count), _i32(sel_seq_len)
    flags = _u8(streaming_flags)
    out = np.zeros((B, H, D), dtype=np.float64)
    lse = np.zeros((B, H), dtype=np.float64)
    scale = float(sm_scale) if sm_scale else 1.0 / float(np.sqrt(D))
    kv = np.ascontiguousarray(k_values, dtype=np.float64)
    vv = np.ascontiguousarray(v_values, dtype=np.float64)
    _load().oracle_sparse_decode_values(_p(_bits(q)), _p(kv), _p(vv), _p(pt), _p(sl), _p(sel), _p(cnt), _p(ssl),
                                        ctypes.c_int(sel.shape[-1]), _p(flags), ctypes.c_int(B),
                                        ctypes.c_int(pt.shape[1]), ctypes.c_int(H), ctypes.c_int(Hkv),
                                        ctypes.c_int(D), ctypes.c_int(NP), ctypes.c_int(_dtype_code(q)),
                                        ctypes.c_int(sink_tokens), ctypes.c_int(local_tokens),
                                        ctypes.c_double(scale), _p(out), _p(lse))
    return out, lse


def sparse_prefill_rows(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, cu_seqlens,
                        streaming_flags: Sequence[int], tile: int, sink_tokens: int,
                        local_tokens: int, rows_token, rows_head,
                        sm_scale: Optional[float] = None):
    """Block-sparse causal prefill for the listed (token, head) rows: (out [R,D] f64, lse [R])."""
    total, H, D = q.shape
    Hkv = k.shape[1]
    cu = _i32(cu_seqlens)
    rt, rh = _i32(rows_token), _i32(rows_head)
    flags = _u8(streaming_flags)
    out = np.zeros((rt.shape[0], D), dtype=np.float64)
    lse = np.zeros((rt.shape[0],), dtype=np.float64)
    scale = float(sm_scale) if sm_scale else 1.0 / float(np.sqrt(D))
    qb, kb, vb = _bits(q), _bits(k), _bits(v)
    _load().oracle_sparse_prefill_rows(_p(qb), _p(kb), _p(vb), _p(cu), ctypes.c_int(cu.shape[0] - 1),
                                       ctypes.c_int(H), ctypes.c_int(Hkv), ctypes.c_int(D),
                                       ctypes.c_int(_dtype_code(q)), ctypes.c_int(tile),
                                       ctypes.c_int(sink_tokens), ctypes.c_int(local_tokens),
                                       _p(flags), ctypes.c_double(scale), _p(rt), _p(rh),
                                       ctypes.c_int(rt.shape[0]), _p(out), _p(lse))
    return out, lse


def paged_prefill_rows(q: torch.Tensor, k_pool: torch.Tensor, v_pool: torch.Tensor, page_table, seq_lens, cu_q,
                       streaming_flags: Sequence[int], sink_tokens: int, local_tokens: int, rows_token, rows_head,
                       sm_scale: Optional[float] = None):
    """Chunked prefill rows over a paged cache that already holds the chunk: (out [R,D] f64, lse [R])."""
    total, H, D = q.shape
    num_pages, Hkv, NP, _ = k_pool.shape
    pt, sl, cu = _i32(page_table), _i32(seq_lens), _i32(cu_q)
    rt, rh = _i32(rows_token), _i32(rows_head)
    flags = _u8(streaming_flags)
    out = np.zeros((rt.shape[0], D), dtype=np.float64)
    lse = np.zeros((rt.shape[0],), dtype=np.float64)
    scale = float(sm_scale) if sm_scale else 1.0 / float(np.sqrt(D))
    qb, kb, vb = _bits(q), _bits(k_pool), _bits(v_pool)
    _load().oracle_paged_prefill_rows(_p(qb), _p(kb), _p(vb), _p(pt), _p(sl), _p(cu), ctypes.c_int(pt.shape[0]),
                                      ctypes.c_int(pt.shape[1]), ctypes.c_int(H), ctypes.c_int(Hkv), ctypes.c_int(D),
                                      ctypes.c_int(NP), ctypes.c_int(_dtype_code(q)), ctypes.c_int(sink_tokens),
                                      ctypes.c_int(local_tokens), _p(flags), ctypes.c_double(scale), _p(rt), _p(rh),
                                      ctypes.c_int(rt.shape[0]), _p(out), _p(lse))
    return out, lse


def chunk_prefill_rows(q: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor, k_hist: np.ndarray,
                       v_hist: np.ndarray, hist_lens, cu_new, streaming_flags: Sequence[int], tile: int,
                       sink_tokens: int, local_tokens: int, rows_token, rows_head, sm_scale: Optional[float] = None):
    """Chunked prefill rows with the history given as values: k_hist / v_hist are float64 [batch, hist_stride, Hkv, D]
    (what the cache stands for at positions below hist_lens; NaN where it holds nothing), the chunk's own K / V are
    the 16-bit tensors.  Returns (out [R, D] f64, lse [R])."""
    total, H, D = q.shape
    Hkv = k_new.shape[1]
    hl, cu = _i32(hist_lens), _i32(cu_new)
    rt, rh = _i32(rows_token), _i32(rows_head)
    flags = _u8(streaming_flags)
    kh = np.ascontiguousarray(k_hist, dtype=np.float64)
    vh = np.ascontiguousarray(v_hist, dtype=np.float64)
    assert kh.shape == vh.shape and kh.shape[0] == hl.shape[0] and kh.shape[2:] == (Hkv, D)
    out = np.zeros((rt.shape[0], D), dtype=np.float64)
    lse = np.zeros((rt.shape[0],), dtype=np.float64)
    scale = float(sm_scale) if sm_scale else 1.0 / float(np.sqrt(D))
    qb, kb, vb = _bits(q), _bits(k_new), _bits(v_new)
    _load().oracle_chunk_prefill_rows(_p(qb), _p(kb), _p(vb), _p(kh), _p(vh), _p(hl), _p(cu), ctypes.c_int(hl.shape[0]),
                                      ctypes.c_int(kh.shape[1]), ctypes.c_int(H), ctypes.c_int(Hkv), ctypes.c_int(D),
                                      ctypes.c_int(tile), ctypes.c_int(_dtype_code(q)), ctypes.c_int(sink_tokens),
                                      ctypes.c_int(local_tokens), _p(flags), ctypes.c_double(scale), _p(rt), _p(rh),
                                      ctypes.c_int(rt.shape[0]), _p(out), _p(lse))
    return out, lse


def block_mask_prefill_rows(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, cu_seqlens,
                            streaming_flags: Sequence[int], tile: int, sink_tokens: int, local_tokens: int,
                            head_mask, q_tile_start, row_ptr, cols, rows_per_mask: int, rows_token, rows_head,
                            sm_scale: Optional[float] = None):
    """Prefill rows under a general block mask (CSR of kept key tiles per query tile, per mask; head_mask[h]
    picks the mask of query head h, -1 = the analytic dense / streaming mask): (out [R,D] f64, lse [R])."""
    total, H, D = q.shape
    Hkv = k.shape[1]
    cu = _i32(cu_seqlens)
    rt, rh = _i32(rows_token), _i32(rows_head)
    hm, qs, rp, cl = _i32(head_mask), _i32(q_tile_start), _i32(row_ptr), _i32(cols)
    if cl.size == 0:
        cl = np.zeros((1,), dtype=np.int32)
    flags = _u8(streaming_flags)
    out = np.zeros((rt.shape[0], D), dtype=np.float64)
    lse = np.zeros((rt.shape[0],), dtype=np.float64)
    scale = float(sm_scale) if sm_scale else 1.0 / float(np.sqrt(D))
    qb, kb, vb = _bits(q), _bits(k), _bits(v)
    _load().oracle_block_mask_prefill_rows(_p(qb), _p(kb), _p(vb), _p(cu), ctypes.c_int(cu.shape[0] - 1),
                                           ctypes.c_int(H), ctypes.c_int(Hkv), ctypes.c_int(D),
                                           ctypes.c_int(_dtype_code(q)), ctypes.c_int(tile),
                                           ctypes.c_int(sink_tokens), ctypes.c_int(local_tokens), _p(flags),
                                           ctypes.c_double(scale), _p(hm), _p(qs), _p(rp), _p(cl),
                                           ctypes.c_int(rows_per_mask), _p(rt), _p(rh),
                                           ctypes.c_int(rt.shape[0]), _p(out), _p(lse))
    return out, lse


def count_nonempty_tiles(n_tokens: int, tile: int, sink_tokens: int, local_tokens: int,
                         streaming: bool) -> int:
    return int(_load().oracle_count_nonempty_tiles(n_tokens, tile, sink_tokens, local_tokens,
                                                   1 if streaming else 0))


def block_sparse_speedup(nonempty_tiles: int, total_tiles: int) -> float:
    return float(_load().oracle_block_sparse_speedup(nonempty_tiles, total_tiles))

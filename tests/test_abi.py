"""The C-ABI library loads, exports every symbol the header declares, and rejects bad arguments
on the host before touching the GPU (so these run without one)."""
import ctypes
import os
import re

import pytest
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    import paper_2502_14866_amd as L

    if not os.path.exists(L.library_path()):
        from paper_2502_14866_amd.build import build_library

        build_library()
    L.load_library()
    return L


def test_every_declared_symbol_is_exported(L):
    header = open(os.path.join(ROOT, "include", "lserve.h")).read()
    declared = set(re.findall(r"^(?:int|size_t|const char \*)\s*(lserve_[a-z_]+)\s*\(", header, flags=re.M))
    assert {"lserve_build_page_stats", "lserve_select_pages", "lserve_sparse_prefill", "lserve_sparse_decode",
            "lserve_workspace_bytes", "lserve_strerror", "lserve_last_hip_error"} <= declared
    lib = ctypes.CDLL(L.library_path())
    for name in declared:
        assert hasattr(lib, name), name


def test_workspace_sizes_and_error_strings(L):
    d = L.AttnDesc(32, 8, [1, 1, 1, 1, 0, 0, 0, 0])
    assert L.lserve_workspace_bytes(L.LSERVE_CALL_SELECT_PAGES, d, 16, 513, 64, 0) == 16 * 8 * 513 * 4
    assert L.lserve_workspace_bytes(L.LSERVE_CALL_SPARSE_DECODE, d, 16, 513, 64, 0) > 0
    assert L.lserve_workspace_bytes(L.LSERVE_CALL_SPARSE_PREFILL, d, 1, 0, 0, 65536) == 0  # Q, K, V read in place
    assert L.lserve_workspace_bytes(L.LSERVE_CALL_BUILD_PAGE_STATS, d, 16, 513, 64, 0) == 0
    bad = L.AttnDesc(32, 8, [0] * 8, head_dim=64)
    assert L.lserve_workspace_bytes(L.LSERVE_CALL_SPARSE_DECODE, bad, 16, 513, 64, 0) == 0
    assert "success" in L.lserve_strerror(0)
    for code in (-1, -2, -3, -4, -99):
        assert L.lserve_strerror(code)


def _dummy_kv(L, batch=2, max_pages=4, hkv=2):
    # host tensors are enough: every call below must fail validation before any launch
    k = torch.zeros((8, hkv, 64, 128), dtype=torch.float16)
    st = torch.zeros((8, hkv, 4, 2, 128), dtype=torch.float16)
    pt = torch.zeros((batch, max_pages), dtype=torch.int32)
    sl = torch.ones((batch + 2,), dtype=torch.int32)[:batch]
    return L.PagedKV(k, k.clone(), st, pt, sl)


def _rc(fn):
    from paper_2502_14866_amd.binding import LserveError

    try:
        fn()
    except LserveError as e:
        return e.code
    return 0


def test_invalid_arguments_are_rejected_on_the_host(L):
    kv = _dummy_kv(L)
    q = torch.zeros((2, 4, 128), dtype=torch.float16)
    out = torch.zeros_like(q)
    sel = torch.zeros((2, 2, 4), dtype=torch.int32)
    cnt = torch.zeros((2, 2), dtype=torch.int32)
    ssl = torch.zeros((4,), dtype=torch.int32)
    ws = torch.zeros((1 << 20,), dtype=torch.uint8)
    good = dict(num_q_heads=4, num_kv_heads=2, streaming_flags=[1, 0])
    stream = 0

    def desc(**kw):
        a = dict(good)
        a.update(kw)
        return L.AttnDesc(**a)

    assert _rc(lambda: L.lserve_build_page_stats(desc(head_dim=64), kv, None, 0, stream)) == -2
    assert _rc(lambda: L.lserve_build_page_stats(desc(dtype=torch.float32), kv, None, 0, stream)) == -2
    assert _rc(lambda: L.lserve_build_page_stats(desc(num_q_heads=5), kv, None, 0, stream)) == -2
    assert _rc(lambda: L.lserve_build_page_stats(desc(num_q_heads=32), kv, None, 0, stream)) == -2  # n = 16
    assert _rc(lambda: L.lserve_build_page_stats(desc(page_size=64, logical_page_size=24), kv, None, 0, stream)) == -1
    assert _rc(lambda: L.lserve_build_page_stats(desc(page_size=48, logical_page_size=16), kv, None, 0, stream)) == -2
    assert _rc(lambda: L.lserve_build_page_stats(desc(local_tokens=0), kv, None, 0, stream)) == -1
    assert _rc(lambda: L.lserve_build_page_stats(desc(), kv, None, -1, stream)) == -1
    nostats = L.PagedKV(kv.k_pool, kv.v_pool, None, kv.page_table, kv.seq_lens)
    assert _rc(lambda: L.lserve_build_page_stats(desc(), nostats, None, 0, stream)) == -1
    # append: non-positive launch bound, missing statistics with a selecting head, missing source
    kn = torch.zeros((4, 2, 128), dtype=torch.float16)
    cu4 = torch.zeros((4,), dtype=torch.int32)
    assert _rc(lambda: L.lserve_append_kv(desc(), kv, kn, kn, cu4, cu4, 0, stream)) == -1
    assert _rc(lambda: L.lserve_append_kv(desc(), nostats, kn, kn, cu4, cu4, 1, stream)) == -1
    assert _rc(lambda: L.lserve_append_kv(desc(), kv, None, kn, cu4, cu4, 1, stream)) == -1
    assert _rc(lambda: L.lserve_append_kv(desc(head_dim=64), kv, kn, kn, cu4, cu4, 1, stream)) == -2
    # selection: budget below one page, missing outputs, workspace too small
    assert _rc(lambda: L.lserve_select_pages(desc(), kv, q, 32, sel, cnt, ssl, None, ws, stream)) == -1
    assert _rc(lambda: L.lserve_select_pages(desc(), kv, q, 256, sel, cnt, ssl, None, None, stream)) == -3
    assert _rc(lambda: L.lserve_select_pages(desc(), kv, q, 256, sel, cnt, ssl, None, ws[:16], stream)) == -3
    # misaligned pointer
    assert _rc(lambda: L.lserve_select_pages(desc(), kv, q.view(-1)[1:], 256, sel, cnt, ssl, None, ws, stream)) == -1
    # two-way cache: a main pool without the streaming heads needs the bounded pool wherever streaming heads
    # are touched; pool_heads must be Hkv or the number of non-streaming heads; the ring needs its table
    dense_only = L.PagedKV(kv.k_pool[:, :1].contiguous(), kv.v_pool[:, :1].contiguous(), kv.stats[:, :1].contiguous(),
                           kv.page_table, kv.seq_lens, pool_heads=1)
    assert _rc(lambda: L.lserve_sparse_decode(desc(), dense_only, q, sel, cnt, ssl, out, None, ws, stream)) == -1
    bad_heads = L.PagedKV(kv.k_pool, kv.v_pool, kv.stats, kv.page_table, kv.seq_lens, pool_heads=3)
    assert _rc(lambda: L.lserve_build_page_stats(desc(), bad_heads, None, 0, stream)) == -1
    no_table = L.PagedKV(kv.k_pool, kv.v_pool, kv.stats, kv.page_table, kv.seq_lens, k_pool_stream=kv.k_pool,
                         v_pool_stream=kv.v_pool)
    assert _rc(lambda: L.lserve_sparse_decode(desc(), no_table, q, sel, cnt, ssl, out, None, ws, stream)) == -1
    # the fused statistics refresh reads keys: the key pool must be given
    nok = L.PagedKV(None, None, kv.stats, kv.page_table, kv.seq_lens)
    assert _rc(lambda: L.lserve_select_pages(desc(), nok, q, 256, sel, cnt, ssl, None, ws, stream, stats_valid_len=ssl)) == -1
    # decode: selecting head present but no selection given; workspace missing
    assert _rc(lambda: L.lserve_sparse_decode(desc(), kv, q, None, None, None, out, None, ws, stream)) == -1
    assert _rc(lambda: L.lserve_sparse_decode(desc(), kv, q, sel, cnt, ssl, out, None, None, stream)) == -3
    # prefill: page size other than 64, max_seqlen beyond the token count
    cu = torch.tensor([0, 2, 0, 0], dtype=torch.int32)[:2]
    assert _rc(lambda: L.lserve_sparse_prefill(desc(page_size=32), q, q[:, :2].contiguous(), q[:, :2].contiguous(), cu, 2, out, None, ws,
                                               stream)) == -2
    assert _rc(lambda: L.lserve_sparse_prefill(desc(), q, q[:, :2].contiguous(), q[:, :2].contiguous(), cu, 3, out,
                                               None, ws, stream)) == -1
    # masked prefill: missing arrays, non-positive counts, workspace smaller than the masked call needs
    i4 = torch.zeros((8,), dtype=torch.int32)
    kk = q[:, :2].contiguous()
    good_mask = L.BlockMask(i4[:4], i4[:2], i4[:3], i4[:1], 1, 1)
    assert _rc(lambda: L.lserve_sparse_prefill_masked(desc(), L.BlockMask(i4[:4], i4[:2], i4[:3], i4[:1], 0, 1), q, kk, kk,
                                                      cu, 2, out, None, ws, stream)) == -1
    assert _rc(lambda: L.lserve_sparse_prefill_masked(desc(), L.BlockMask(i4[1:5], i4[:2], i4[:3], i4[:1], 1, 1), q, kk,
                                                      kk, cu, 2, out, None, ws, stream)) == -1  # misaligned
    need = L.lserve_masked_prefill_workspace_bytes(desc(), 1, 2, 2, 1, 1)
    assert need > 0
    assert _rc(lambda: L.lserve_sparse_prefill_masked(desc(), good_mask, q, kk, kk, cu, 2, out, None, ws[:need - 16],
                                                      stream)) == -3
    assert L.lserve_masked_prefill_workspace_bytes(desc(), 1, 2, 2, 0, 1) == 0
    # paged prefill: chunk bounds, two-way caches are not supported
    assert _rc(lambda: L.lserve_sparse_prefill_paged(desc(), kv, q, cu4, 0, 64, out, None, ws, stream)) == -1
    assert _rc(lambda: L.lserve_sparse_prefill_paged(desc(), kv, q, cu4, 2, 1, out, None, ws, stream)) == -1
    assert _rc(lambda: L.lserve_sparse_prefill_paged(desc(), dense_only, q, cu4, 2, 64, out, None, ws, stream)) == -1
    assert _rc(lambda: L.lserve_sparse_prefill_paged(desc(page_size=32), kv, q, cu4, 2, 64, out, None, ws, stream)) == -2
    assert L.lserve_paged_prefill_workspace_bytes(desc(), 2, 4) == 0  # keys and values read from the pages
    # chunk prefill (history in the cache, the chunk's K / V alongside): missing chunk tensors, bounds, page size;
    # a two-way cache is fine here, but its ring needs its table
    assert _rc(lambda: L.lserve_sparse_prefill_chunk(desc(), kv, q, None, kn, cu4, 2, out, None, stream)) == -1
    assert _rc(lambda: L.lserve_sparse_prefill_chunk(desc(), kv, q, kn, kn, cu4, 0, out, None, stream)) == -1
    assert _rc(lambda: L.lserve_sparse_prefill_chunk(desc(), kv, q, kn, kn, cu4, 3, out, None, stream)) == -1
    assert _rc(lambda: L.lserve_sparse_prefill_chunk(desc(page_size=32), kv, q, kn, kn, cu4, 2, out, None, stream)) == -2
    assert _rc(lambda: L.lserve_sparse_prefill_chunk(desc(), no_table, q, kn, kn, cu4, 2, out, None, stream)) == -1
    assert _rc(lambda: L.lserve_sparse_prefill_chunk(desc(), dense_only, q, kn, kn, cu4, 2, out, None, stream)) == -1
    # quantised pages: only 8 or 4 bits and 64-token pages; no statistics from the pages, no paged prefill
    def q8(bits=8):
        return L.PagedKV(kv.k_pool, kv.v_pool, kv.stats, kv.page_table, kv.seq_lens, kv_bits=bits)
    d32 = desc(page_size=32)
    assert _rc(lambda: L.lserve_sparse_decode(desc(), q8(5), q, sel, cnt, ssl, out, None, ws, stream)) == -1
    assert _rc(lambda: L.lserve_sparse_decode(d32, q8(4), q, sel, cnt, ssl, out, None, ws, stream)) == -2
    assert _rc(lambda: L.lserve_sparse_decode(d32, q8(), q, sel, cnt, ssl, out, None, ws, stream)) == -2
    assert _rc(lambda: L.lserve_append_kv(d32, q8(), kn, kn, cu4, cu4, 1, stream)) == -2
    assert _rc(lambda: L.lserve_build_page_stats(desc(), q8(), None, 0, stream)) == -2
    assert _rc(lambda: L.lserve_select_pages(desc(), q8(), q, 256, sel, cnt, ssl, None, ws, stream, stats_valid_len=ssl)) == -2
    assert _rc(lambda: L.lserve_sparse_prefill_paged(desc(), q8(), q, cu4, 2, 64, out, None, ws, stream)) == -2


def test_decode_rejects_an_index_space_beyond_32_bits_and_accepts_wide_tables(L):
    """The launch plan numbers batch * (entries per sequence) with 32-bit integers: beyond that the call is
    refused on the host (pointers are never dereferenced before validation, so one small buffer stands in
    for all of them).  Entries per sequence above 65535 are fine."""
    lib = L.load_library()
    hkv = 64
    d = L.AttnDesc(64, hkv, [0] * hkv)
    batch = 65535
    pt = torch.zeros((batch, 1), dtype=torch.int32)
    sl = torch.ones((batch,), dtype=torch.int32)
    k = torch.zeros((1, hkv, 64, 128), dtype=torch.float16)
    kv = L.PagedKV(k, k, None, pt, sl)
    p = ctypes.c_void_p(k.data_ptr())
    ws_bytes = ctypes.c_size_t(1 << 40)

    def call(sel_stride):
        return lib.lserve_sparse_decode(d.c(), kv.c(), p, p, p, p, sel_stride, p, None, p, ws_bytes, None)

    assert 65535 * 64 * 601 > 2 ** 31
    assert call(600) == -2
    assert L.lserve_workspace_bytes(L.LSERVE_CALL_SPARSE_DECODE, d, batch, 1, 600, 0) > 0
    # 64 selecting heads x 2049 entries = 131136 entries per sequence: above 16 bits, accepted by the host checks
    # (a workspace of 16 bytes is what stops this call before any launch)
    kv1 = L.PagedKV(k, k, None, pt[:1], sl[:4][:1])
    assert lib.lserve_sparse_decode(d.c(), kv1.c(), p, p, p, p, 2048, p, None, p, ctypes.c_size_t(16), None) == -3


def test_selector_needs_no_statistics_when_every_head_is_streaming(L):
    lib = L.load_library()
    d = L.AttnDesc(4, 2, [1, 1])
    k = torch.zeros((8, 2, 64, 128), dtype=torch.float16)
    pt = torch.zeros((2, 4), dtype=torch.int32)
    sl = torch.ones((4,), dtype=torch.int32)[:2]
    kv = L.PagedKV(k, k, None, pt, sl)
    p = ctypes.c_void_p(k.data_ptr())
    # passes the statistics check and is stopped by the last host check (workspace too small) ...
    assert lib.lserve_select_pages(d.c(), kv.c(), p, 256, None, p, p, p, None, p, ctypes.c_size_t(16), None) == -3
    # ... whereas a selecting head without statistics is an invalid argument
    d2 = L.AttnDesc(4, 2, [1, 0])
    assert lib.lserve_select_pages(d2.c(), kv.c(), p, 256, None, p, p, p, None, p, ctypes.c_size_t(16), None) == -1


def test_library_reads_no_environment_variable():
    csrc = os.path.join(ROOT, "paper_2502_14866_amd", "csrc")
    for f in os.listdir(csrc):
        assert "getenv" not in open(os.path.join(csrc, f)).read(), f


def test_product_path_does_not_reach_for_the_oracle():
    pkg = os.path.join(ROOT, "paper_2502_14866_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "lserve_oracle" not in text

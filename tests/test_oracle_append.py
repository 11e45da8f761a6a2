"""Pins for the oracle's KV write-back (Sec. 3.2): a pure index map, checked against an
independent gather / scatter written with torch indexing and against brute-force reads."""
import numpy as np
import torch

import oracle
from workloads import scatter_prefill_kv_to_pages

from helpers import gather_tokens


def _pool(num_pages, Hkv, NP, D, seed):
    g = torch.Generator().manual_seed(seed)
    return torch.randn((num_pages, Hkv, NP, D), generator=g).to(torch.float16)


def test_append_from_empty_equals_the_indexing_scatter():
    Hkv, NP, D = 3, 16, 8
    lengths = [1, 16, 37]
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    g = torch.Generator().manual_seed(3)
    perm = torch.randperm(12, generator=g).to(torch.int32)
    page_table = perm.reshape(3, 4)
    k_new = torch.randn((int(cu[-1]), Hkv, D), generator=g).to(torch.float16)
    v_new = torch.randn((int(cu[-1]), Hkv, D), generator=g).to(torch.float16)
    k_a, v_a = _pool(12, Hkv, NP, D, 1), _pool(12, Hkv, NP, D, 2)
    k_b, v_b = k_a.clone(), v_a.clone()
    oracle.append_kv(k_new, v_new, cu, np.zeros(3, np.int32), page_table, k_a, v_a)
    scatter_prefill_kv_to_pages(k_new, v_new, cu, k_b, v_b, page_table)
    assert torch.equal(k_a.view(torch.int16), k_b.view(torch.int16))
    assert torch.equal(v_a.view(torch.int16), v_b.view(torch.int16))


def test_append_at_an_offset_lands_where_a_gather_reads_it_and_touches_nothing_else():
    Hkv, NP, D = 2, 8, 4
    start = np.array([5, 8, 0], np.int32)
    n_new = [7, 1, 0]
    cu = np.concatenate([[0], np.cumsum(n_new)]).astype(np.int32)
    page_table = torch.tensor([[4, 0, 7], [2, 6, 1], [3, 5, 8]], dtype=torch.int32)
    g = torch.Generator().manual_seed(11)
    k_new = torch.randn((8, Hkv, D), generator=g).to(torch.bfloat16)
    v_new = torch.randn((8, Hkv, D), generator=g).to(torch.bfloat16)
    k0 = torch.randn((9, Hkv, NP, D), generator=g).to(torch.bfloat16)
    v0 = torch.randn((9, Hkv, NP, D), generator=g).to(torch.bfloat16)
    k1, v1 = k0.clone(), v0.clone()
    oracle.append_kv(k_new, v_new, cu, start, page_table, k1, v1)
    touched = torch.zeros((9, NP), dtype=torch.bool)
    for b in range(3):
        L = int(start[b]) + n_new[b]
        kk = gather_tokens(k1, page_table, b, L)  # [L, Hkv, D] float64 (exact for 16-bit storage)
        vv = gather_tokens(v1, page_table, b, L)
        old = gather_tokens(k0, page_table, b, L)
        s = int(start[b])
        assert np.array_equal(kk[s:], k_new[cu[b]:cu[b + 1]].double().numpy())
        assert np.array_equal(vv[s:], v_new[cu[b]:cu[b + 1]].double().numpy())
        assert np.array_equal(kk[:s], old[:s])  # earlier tokens of the sequence stay
        for pos in range(int(start[b]), L):
            touched[int(page_table[b, pos // NP]), pos % NP] = True
    assert int(touched.sum()) == 8
    keep = ~touched[:, None, :, None].expand_as(k0)
    assert torch.equal(k1[keep], k0[keep]) and torch.equal(v1[keep], v0[keep])

"""Pins for the oracle's sparse decode and block-sparse prefill.

References used here are not the oracle's own code: torch's CPU scaled-dot-product
attention in float64 on explicitly gathered keys/values, hand-written masks of tiny
worked examples, closed forms, the figures the paper prints, and invariants.
"""
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from workloads import Workload, make_decode_inputs, make_prefill_inputs

from helpers import gather_tokens, small_decode_workload

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "block_sparsity_example.txt")


def _sdpa(q, k, v, mask=None, scale=None):
    """q [D], k/v [n, D] float64 numpy -> textbook softmax attention via torch's CPU routine."""
    qt = torch.from_numpy(np.asarray(q))[None, None, None, :]
    kt = torch.from_numpy(np.asarray(k))[None, None]
    vt = torch.from_numpy(np.asarray(v))[None, None]
    m = None if mask is None else torch.from_numpy(np.asarray(mask))[None, None, None, :]
    return F.scaled_dot_product_attention(qt, kt, vt, attn_mask=m, scale=scale)[0, 0, 0].numpy()


def _all_pages_selection(w, seq):
    P = [(int(l) + w.page_size - 1) // w.page_size for l in seq]
    K = max(P)
    sel = np.full((w.batch, w.num_kv_heads, K), -1, dtype=np.int32)
    cnt = np.zeros((w.batch, w.num_kv_heads), dtype=np.int32)
    for b in range(w.batch):
        sel[b, :, :P[b]] = np.arange(P[b])
        cnt[b] = P[b]
    return sel, cnt, np.asarray(seq, dtype=np.int32)


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
def test_decode_with_every_page_listed_is_textbook_attention(dtype):
    w = small_decode_workload(dtype=dtype, streaming_kv_heads=())
    inp = make_decode_inputs(w)
    seq = inp.seq_lens_at(0)
    sel, cnt, ssl = _all_pages_selection(w, seq)
    out, lse = oracle.sparse_decode(inp.q[0], inp.k_pool, inp.v_pool, inp.page_table, seq, sel, cnt, ssl,
                                    w.streaming_flags(), w.sink_tokens, w.local_tokens)
    pt = inp.page_table.numpy()
    for b in range(w.batch):
        L = int(seq[b])
        K, V = gather_tokens(inp.k_pool, pt, b, L), gather_tokens(inp.v_pool, pt, b, L)
        q = inp.q[0, b].to(torch.float64).numpy()
        for h in range(w.num_q_heads):
            ref = _sdpa(q[h], K[:, h // w.group], V[:, h // w.group])
            np.testing.assert_allclose(out[b, h], ref, rtol=1e-10, atol=1e-12)
            logits = K[:, h // w.group] @ q[h] / np.sqrt(w.head_dim)
            # softmax weights rebuilt from lse sum to one
            assert abs(np.exp(logits - lse[b, h]).sum() - 1.0) < 1e-10
            vv = V[:, h // w.group]
            assert (out[b, h] <= vv.max(axis=0) + 1e-12).all() and (out[b, h] >= vv.min(axis=0) - 1e-12).all()


def test_decode_attends_exactly_the_listed_pages_plus_pages_newer_than_the_selection():
    w = small_decode_workload(streaming_kv_heads=(), lengths=(1000, 1500), decode_steps=70)
    inp = make_decode_inputs(w)
    step = 69
    seq = inp.seq_lens_at(step)  # 1070, 1570
    sel_len = inp.seq_lens_at(0)  # selection made 69 tokens earlier: one or two pages are newer
    rng = np.random.default_rng(0)
    K = 5
    sel = np.full((w.batch, w.num_kv_heads, K), -1, dtype=np.int32)
    cnt = np.zeros((w.batch, w.num_kv_heads), dtype=np.int32)
    for b in range(w.batch):
        P0 = (int(sel_len[b]) + 63) // 64
        for hk in range(w.num_kv_heads):
            c = 3 + (hk % 3)
            sel[b, hk, :c] = np.sort(rng.choice(P0, size=c, replace=False))
            cnt[b, hk] = c
    out, _ = oracle.sparse_decode(inp.q[step], inp.k_pool, inp.v_pool, inp.page_table, seq, sel, cnt,
                                  sel_len, w.streaming_flags(), w.sink_tokens, w.local_tokens)
    pt = inp.page_table.numpy()
    for b in range(w.batch):
        L, L0 = int(seq[b]), int(sel_len[b])
        Kc, Vc = gather_tokens(inp.k_pool, pt, b, L), gather_tokens(inp.v_pool, pt, b, L)
        q = inp.q[step, b].to(torch.float64).numpy()
        for h in range(w.num_q_heads):
            hk = h // w.group
            pages = set(sel[b, hk, :cnt[b, hk]].tolist()) | set(range((L0 + 63) // 64, (L + 63) // 64))
            tok = np.array([u for u in range(L) if u // 64 in pages])
            ref = _sdpa(q[h], Kc[tok, hk], Vc[tok, hk])
            np.testing.assert_allclose(out[b, h], ref, rtol=1e-10, atol=1e-12)


def test_streaming_decode_sees_only_sink_and_local_pages():
    w = small_decode_workload(lengths=(1000, 70), sink_tokens=100, local_tokens=130)  # s = 2, w = 3
    inp = make_decode_inputs(w)
    seq = inp.seq_lens_at(0)
    sel, cnt, ssl = _all_pages_selection(w, seq)
    args = (inp.page_table, seq, sel, cnt, ssl, w.streaming_flags(), w.sink_tokens, w.local_tokens)
    out, _ = oracle.sparse_decode(inp.q[0], inp.k_pool, inp.v_pool, *args)
    pt = inp.page_table.numpy()
    # sequence 0: 1001 tokens = 16 pages; streaming head 0 sees pages {0, 1} and {13, 14, 15}
    K, V = gather_tokens(inp.k_pool, pt, 0, 1001), gather_tokens(inp.v_pool, pt, 0, 1001)
    tok = np.array(list(range(0, 128)) + list(range(13 * 64, 1001)))
    q = inp.q[0, 0].to(torch.float64).numpy()
    for h in range(w.group):  # query heads of streaming KV head 0
        np.testing.assert_allclose(out[0, h], _sdpa(q[h], K[tok, 0], V[tok, 0]), rtol=1e-10, atol=1e-12)
    # sequence 1: 71 tokens = 2 pages, sink and local overlap: plain attention over everything
    K1, V1 = gather_tokens(inp.k_pool, pt, 1, 71), gather_tokens(inp.v_pool, pt, 1, 71)
    q1 = inp.q[0, 1].to(torch.float64).numpy()
    np.testing.assert_allclose(out[1, 0], _sdpa(q1[0], K1[:, 0], V1[:, 0]), rtol=1e-10, atol=1e-12)
    # garbage in every page outside sink + local leaves the streaming head bit-unchanged
    k2, v2 = inp.k_pool.clone(), inp.v_pool.clone()
    for p in range(2, 13):
        k2[int(inp.page_table[0, p]), 0] = 77.0
        v2[int(inp.page_table[0, p]), 0] = -55.0
    out2, _ = oracle.sparse_decode(inp.q[0], k2, v2, *args)
    assert np.array_equal(out[:, :w.group], out2[:, :w.group])
    assert np.array_equal(out[:, w.group:], out2[:, w.group:])  # other KV head untouched as well


def test_decode_of_a_single_token_context_returns_its_value():
    w = small_decode_workload(lengths=(0, 0), decode_steps=1)
    inp = make_decode_inputs(w)
    seq = inp.seq_lens_at(0)  # 1, 1
    sel, cnt, ssl = _all_pages_selection(w, seq)
    out, lse = oracle.sparse_decode(inp.q[0], inp.k_pool, inp.v_pool, inp.page_table, seq, sel, cnt, ssl,
                                    w.streaming_flags(), w.sink_tokens, w.local_tokens)
    for b in range(w.batch):
        v0 = inp.v_pool[int(inp.page_table[b, 0]), :, 0].to(torch.float64).numpy()
        for h in range(w.num_q_heads):
            np.testing.assert_allclose(out[b, h], v0[h // w.group], rtol=0, atol=1e-15)


def _prefill_workload(**kw):
    base = dict(name="tinyp", batch=1, num_q_heads=4, num_kv_heads=2, dtype="fp16",
                streaming_kv_heads=(0,), sink_tokens=64, local_tokens=128, prefill_tokens=400, seed=11)
    base.update(kw)
    return Workload(**base)


def _all_rows(total, H):
    tok = np.repeat(np.arange(total, dtype=np.int32), H)
    head = np.tile(np.arange(H, dtype=np.int32), total)
    return tok, head


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
def test_dense_prefill_is_causal_textbook_attention_per_sequence(dtype):
    w = _prefill_workload(dtype=dtype, streaming_kv_heads=(), batch=2)
    pin = make_prefill_inputs(w, lengths=(150, 203))
    total = 353
    tok, head = _all_rows(total, w.num_q_heads)
    out, lse = oracle.sparse_prefill_rows(pin.q, pin.k, pin.v, pin.cu_seqlens, w.streaming_flags(), 64,
                                          w.sink_tokens, w.local_tokens, tok, head)
    out = out.reshape(total, w.num_q_heads, w.head_dim)
    q, k, v = (x.to(torch.float64) for x in (pin.q, pin.k, pin.v))
    for (a, e) in ((0, 150), (150, 353)):
        qs = q[a:e].permute(1, 0, 2)[None]  # [1, H, n, D]
        ks = k[a:e].permute(1, 0, 2).repeat_interleave(w.group, dim=0)[None]
        vs = v[a:e].permute(1, 0, 2).repeat_interleave(w.group, dim=0)[None]
        ref = F.scaled_dot_product_attention(qs, ks, vs, is_causal=True)[0].permute(1, 0, 2).numpy()
        np.testing.assert_allclose(out[a:e], ref, rtol=1e-9, atol=1e-12)
    # first token of each sequence attends itself only
    v64 = v.numpy()
    for t0 in (0, 150):
        for h in range(w.num_q_heads):
            np.testing.assert_allclose(out[t0, h], v64[t0, h // w.group], rtol=0, atol=1e-15)


def test_streaming_prefill_matches_a_hand_written_mask():
    # 8 tokens, tile 2, sink 2 tokens (1 tile), local 4 tokens (2 tiles incl. the diagonal one).
    # Row t (tile t//2) sees tile 0, its own tile and the tile before it, causally.
    hand_mask = np.array([
        [1, 0, 0, 0, 0, 0, 0, 0],
        [1, 1, 0, 0, 0, 0, 0, 0],
        [1, 1, 1, 0, 0, 0, 0, 0],
        [1, 1, 1, 1, 0, 0, 0, 0],
        [1, 1, 1, 1, 1, 0, 0, 0],
        [1, 1, 1, 1, 1, 1, 0, 0],
        [1, 1, 0, 0, 1, 1, 1, 0],
        [1, 1, 0, 0, 1, 1, 1, 1],
    ], dtype=bool)
    w = _prefill_workload(prefill_tokens=8, num_q_heads=2, num_kv_heads=1, streaming_kv_heads=(0,))
    pin = make_prefill_inputs(w)
    tok, head = _all_rows(8, 2)
    out, _ = oracle.sparse_prefill_rows(pin.q, pin.k, pin.v, pin.cu_seqlens, [1], 2, 2, 4, tok, head)
    out = out.reshape(8, 2, w.head_dim)
    q, k, v = (x.to(torch.float64).numpy() for x in (pin.q, pin.k, pin.v))
    for t in range(8):
        for h in range(2):
            ref = _sdpa(q[t, h], k[:, 0], v[:, 0], mask=hand_mask[t])
            np.testing.assert_allclose(out[t, h], ref, rtol=1e-10, atol=1e-12)


def test_streaming_prefill_with_window_covering_everything_is_dense():
    w = _prefill_workload(sink_tokens=64, local_tokens=512)  # 400 tokens < 512
    pin = make_prefill_inputs(w)
    tok, head = _all_rows(400, w.num_q_heads)
    a, la = oracle.sparse_prefill_rows(pin.q, pin.k, pin.v, pin.cu_seqlens, [1, 0], 64, 64, 512, tok, head)
    b, lb = oracle.sparse_prefill_rows(pin.q, pin.k, pin.v, pin.cu_seqlens, [0, 0], 64, 64, 512, tok, head)
    assert np.array_equal(a, b) and np.array_equal(la, lb)


def test_prefill_row_t_equals_decode_at_length_t_plus_one():
    """Ties the two definitions together: same token set, so same output (streaming and dense)."""
    from workloads import scatter_prefill_kv_to_pages

    w = _prefill_workload(prefill_tokens=700, sink_tokens=64, local_tokens=192)
    pin = make_prefill_inputs(w)
    dw = small_decode_workload(batch=1, lengths=(700,), decode_steps=1, streaming_kv_heads=(0,),
                               sink_tokens=64, local_tokens=192)
    dinp = make_decode_inputs(dw)
    scatter_prefill_kv_to_pages(pin.k, pin.v, pin.cu_seqlens.tolist(), dinp.k_pool, dinp.v_pool, dinp.page_table)
    rows = np.array([0, 63, 64, 65, 255, 256, 300, 511, 512, 699], dtype=np.int32)
    tok = np.repeat(rows, w.num_q_heads)
    head = np.tile(np.arange(w.num_q_heads, dtype=np.int32), len(rows))
    pre, pre_lse = oracle.sparse_prefill_rows(pin.q, pin.k, pin.v, pin.cu_seqlens, w.streaming_flags(), 64,
                                              64, 192, tok, head)
    pre = pre.reshape(len(rows), w.num_q_heads, -1)
    for i, t in enumerate(rows):
        seq = np.array([t + 1], dtype=np.int32)
        sel, cnt, ssl = _all_pages_selection(dw, seq)
        dec, dec_lse = oracle.sparse_decode(pin.q[t:t + 1], dinp.k_pool, dinp.v_pool, dinp.page_table, seq,
                                            sel, cnt, ssl, dw.streaming_flags(), 64, 192)
        np.testing.assert_allclose(pre[i], dec[0], rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(pre_lse.reshape(len(rows), -1)[i], dec_lse[0], rtol=1e-12)


def test_streaming_prefill_ignores_everything_outside_sink_and_band():
    w = _prefill_workload(prefill_tokens=640, sink_tokens=64, local_tokens=128)  # s = 1, w = 2
    pin = make_prefill_inputs(w)
    rows = np.arange(576, 640, dtype=np.int32)  # query tile 9 sees tiles {0, 8, 9}
    tok, head = np.repeat(rows, 2), np.tile(np.array([0, 1], dtype=np.int32), len(rows))  # streaming heads
    a, _ = oracle.sparse_prefill_rows(pin.q, pin.k, pin.v, pin.cu_seqlens, [1, 0], 64, 64, 128, tok, head)
    k2, v2 = pin.k.clone(), pin.v.clone()
    k2[64:512, 0] = 31.0
    v2[64:512, 0] = -9.0
    b, _ = oracle.sparse_prefill_rows(pin.q, k2, v2, pin.cu_seqlens, [1, 0], 64, 64, 128, tok, head)
    assert np.array_equal(a, b)


def _golden():
    vals = {}
    with open(GOLDEN) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                key, val = line.split()
                vals[key] = float(val)
    return vals


def test_block_counts_match_the_papers_printed_example_and_closed_forms():
    g = _golden()
    # Sec. 3.1: 10 non-empty tiles of 21 -> 2.1x
    assert abs(oracle.block_sparse_speedup(int(g["nonempty_tiles"]), int(g["total_tiles"])) - g["speedup"]) < 1e-12
    # a causal grid with 21 tiles is 6 x 6 tiles: 6 * 7 / 2
    assert oracle.count_nonempty_tiles(6 * 64, 64, 0, 0, False) == int(g["total_tiles"])
    # streaming pattern of the figure: one sink + two local blocks -> three blocks per query block
    s, wl = int(g["streaming_sink_blocks"]), int(g["streaming_local_blocks"])
    n_tiles = 12
    total = oracle.count_nonempty_tiles(n_tiles * 64, 64, s * 64, wl * 64, True)
    head = oracle.count_nonempty_tiles(3 * 64, 64, s * 64, wl * 64, True)  # rows 0..2: 1 + 2 + 3
    assert head == 6
    assert total - head == (n_tiles - 3) * int(g["streaming_blocks_per_row"])
    # closed form cnt(i) = min(i+1, w) + max(0, min(s, i-w+1)) summed over rows, ragged tail included
    for (n, T, sink, local) in ((2048, 64, 64, 256), (1000, 64, 128, 512), (333, 16, 20, 50)):
        s_, w_ = -(-sink // T), -(-local // T)
        nt = -(-n // T)
        closed = sum(min(i + 1, w_) + max(0, min(s_, i - w_ + 1)) for i in range(nt))
        assert oracle.count_nonempty_tiles(n, T, sink, local, True) == closed
        assert oracle.count_nonempty_tiles(n, T, sink, local, False) == nt * (nt + 1) // 2
    assert oracle.count_nonempty_tiles(2048, 64, 64, 256, True) == 150


# ---- prefill under a general block mask (Sec. 3.1, Sec. 3.4) --------------------------------------

def _mask_rows(pin, w, lengths, masks, head_mask, tile=64):
    from helpers import block_mask_csr
    qts, rp, cl, R = block_mask_csr(masks, lengths, tile)
    total = sum(lengths)
    tok, head = _all_rows(total, w.num_q_heads)
    out, lse = oracle.block_mask_prefill_rows(pin.q, pin.k, pin.v, pin.cu_seqlens, w.streaming_flags(), tile,
                                              w.sink_tokens, w.local_tokens, head_mask, qts, rp, cl, R, tok, head)
    return out.reshape(total, w.num_q_heads, w.head_dim), lse.reshape(total, w.num_q_heads)


def test_block_mask_with_every_lower_tile_is_dense_and_with_the_analytic_tiles_is_streaming():
    w = _prefill_workload(batch=2, sink_tokens=64, local_tokens=128)
    lengths = (150, 203)
    pin = make_prefill_inputs(w, lengths=lengths)
    total = sum(lengths)
    tok, head = _all_rows(total, w.num_q_heads)
    lower = lambda b, i: range(i + 1)
    s, wl = 1, 2
    lam = lambda b, i: [j for j in range(i + 1) if j < s or j > i - wl]
    # mask 0 = all lower tiles for heads 0, 1 (KV head 0 is flagged streaming but the mask overrides it);
    # mask 1 = the streaming tiles for heads 2, 3 (KV head 1 is flagged dense)
    out, lse = _mask_rows(pin, w, lengths, [lower, lam], [0, 0, 1, 1])
    dense, dl = oracle.sparse_prefill_rows(pin.q, pin.k, pin.v, pin.cu_seqlens, [0, 0], 64, w.sink_tokens,
                                           w.local_tokens, tok, head)
    strm, sl = oracle.sparse_prefill_rows(pin.q, pin.k, pin.v, pin.cu_seqlens, [1, 1], 64, w.sink_tokens,
                                          w.local_tokens, tok, head)
    dense, strm = dense.reshape(total, 4, -1), strm.reshape(total, 4, -1)
    np.testing.assert_allclose(out[:, :2], dense[:, :2], rtol=0, atol=0)
    np.testing.assert_allclose(out[:, 2:], strm[:, 2:], rtol=0, atol=0)
    np.testing.assert_allclose(lse[:, :2], dl.reshape(total, 4)[:, :2], rtol=0, atol=0)
    # head_mask = -1 falls back to the analytic mask of the flags
    out2, _ = _mask_rows(pin, w, lengths, [lower], [-1, -1, -1, -1])
    mixed, _ = oracle.sparse_prefill_rows(pin.q, pin.k, pin.v, pin.cu_seqlens, w.streaming_flags(), 64,
                                          w.sink_tokens, w.local_tokens, tok, head)
    np.testing.assert_allclose(out2, mixed.reshape(total, 4, -1), rtol=0, atol=0)


def test_block_mask_rows_equal_textbook_attention_under_the_expanded_boolean_mask():
    rng = np.random.default_rng(5)
    w = _prefill_workload(batch=2, num_q_heads=2, num_kv_heads=1, streaming_kv_heads=())
    lengths = (23, 17)
    pin = make_prefill_inputs(w, lengths=lengths)
    T = 4
    kept = {}

    def rnd(b, i):  # random subset of the lower tiles, always with the diagonal, different per sequence
        if (b, i) not in kept:
            kept[(b, i)] = [j for j in range(i) if rng.random() < 0.4] + [i]
        return kept[(b, i)]

    empty_diag = lambda b, i: [j for j in range(i) if j % 2 == 0]  # the first tile row keeps nothing at all
    out, lse = _mask_rows(pin, w, lengths, [rnd, empty_diag], [0, 1], tile=T)
    q, k, v = (x.to(torch.float64).numpy() for x in (pin.q, pin.k, pin.v))
    start = 0
    for b, n in enumerate(lengths):
        for t in range(n):
            for h, fn in ((0, rnd), (1, empty_diag)):
                tiles = set(fn(b, t // T))
                mask = np.array([(u <= t) and (u // T in tiles) for u in range(n)])
                if not mask.any():
                    assert np.all(out[start + t, h] == 0) and lse[start + t, h] == -np.inf
                    continue
                ref = _sdpa(q[start + t, h], k[start:start + n, 0], v[start:start + n, 0], mask=mask)
                np.testing.assert_allclose(out[start + t, h], ref, rtol=1e-10, atol=1e-12)
        start += n


# ---- chunked prefill over a paged cache ---------------------------------------------------------------

def test_paged_chunk_rows_equal_the_contiguous_prefill_rows_and_the_decode_of_the_same_position():
    """Scatter a contiguous prefill into pages: the chunk holding the last n tokens must reproduce the rows of
    the contiguous prefill (independent function, independent addressing), whatever the chunk boundary; and a
    one-token chunk is a decode step with the analytic page lists."""
    from workloads import scatter_prefill_kv_to_pages
    w = _prefill_workload(batch=2, sink_tokens=64, local_tokens=128)
    lengths = (300, 131)
    pin = make_prefill_inputs(w, lengths=lengths)
    NP = 64
    g = torch.Generator().manual_seed(3)
    page_table = torch.randperm(16, generator=g).to(torch.int32).reshape(2, 8)
    k_pool = torch.randn((16, w.num_kv_heads, NP, w.head_dim), generator=g).to(pin.k.dtype)
    v_pool = torch.randn((16, w.num_kv_heads, NP, w.head_dim), generator=g).to(pin.k.dtype)
    scatter_prefill_kv_to_pages(pin.k, pin.v, pin.cu_seqlens, k_pool, v_pool, page_table)
    total = sum(lengths)
    tok, head = _all_rows(total, w.num_q_heads)
    full, full_lse = oracle.sparse_prefill_rows(pin.q, pin.k, pin.v, pin.cu_seqlens, w.streaming_flags(), NP,
                                                w.sink_tokens, w.local_tokens, tok, head)
    full = full.reshape(total, w.num_q_heads, -1)
    for chunk in ((300, 131), (100, 67), (1, 1), (64, 3)):
        qs, idx = [], []
        for b, (L, n) in enumerate(zip(lengths, chunk)):
            a = int(pin.cu_seqlens[b]) + L - n
            qs.append(pin.q[a:a + n])
            idx.extend(range(a, a + n))
        qc = torch.cat(qs)
        cu_q = np.concatenate([[0], np.cumsum(chunk)]).astype(np.int32)
        t2, h2 = _all_rows(sum(chunk), w.num_q_heads)
        out, lse = oracle.paged_prefill_rows(qc, k_pool, v_pool, page_table, np.asarray(lengths, np.int32), cu_q,
                                             w.streaming_flags(), w.sink_tokens, w.local_tokens, t2, h2)
        out = out.reshape(sum(chunk), w.num_q_heads, -1)
        np.testing.assert_allclose(out, full[idx], rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(lse.reshape(sum(chunk), -1), full_lse.reshape(total, -1)[idx], rtol=1e-12, atol=1e-12)


# ---- chunked prefill in the order of the prefill flow: history from the cache, the chunk's K / V alongside ----------

def test_chunk_rows_with_history_values_equal_the_contiguous_prefill_rows():
    """Cut a contiguous prefill into history + chunk at several places (none, off a tile boundary, on one, one
    token): with the history handed over as exactly the 16-bit values, the rows of the chunk must reproduce the
    rows of the contiguous prefill (another function with other addressing)."""
    w = _prefill_workload(batch=2, sink_tokens=64, local_tokens=128)
    lengths = (300, 131)
    pin = make_prefill_inputs(w, lengths=lengths)
    total = sum(lengths)
    tok, head = _all_rows(total, w.num_q_heads)
    full, full_lse = oracle.sparse_prefill_rows(pin.q, pin.k, pin.v, pin.cu_seqlens, w.streaming_flags(), 64,
                                                w.sink_tokens, w.local_tokens, tok, head)
    full = full.reshape(total, w.num_q_heads, -1)
    full_lse = full_lse.reshape(total, w.num_q_heads)
    for chunk in ((300, 131), (100, 67), (1, 1), (64, 3), (236, 0)):
        hist = [L - n for L, n in zip(lengths, chunk)]
        stride = max(max(hist), 1)
        k_hist = np.full((2, stride, w.num_kv_heads, w.head_dim), np.nan)
        v_hist = np.full_like(k_hist, np.nan)
        qs, ks, vs, idx = [], [], [], []
        for b, (L, n) in enumerate(zip(lengths, chunk)):
            a = int(pin.cu_seqlens[b])
            k_hist[b, :hist[b]] = pin.k[a:a + hist[b]].to(torch.float64).numpy()
            v_hist[b, :hist[b]] = pin.v[a:a + hist[b]].to(torch.float64).numpy()
            qs.append(pin.q[a + hist[b]:a + L]); ks.append(pin.k[a + hist[b]:a + L]); vs.append(pin.v[a + hist[b]:a + L])
            idx.extend(range(a + hist[b], a + L))
        qc, kc, vc = torch.cat(qs), torch.cat(ks), torch.cat(vs)
        cu_new = np.concatenate([[0], np.cumsum(chunk)]).astype(np.int32)
        t2, h2 = _all_rows(sum(chunk), w.num_q_heads)
        out, lse = oracle.chunk_prefill_rows(qc, kc, vc, k_hist, v_hist, np.asarray(hist, np.int32), cu_new,
                                             w.streaming_flags(), 64, w.sink_tokens, w.local_tokens, t2, h2)
        np.testing.assert_allclose(out.reshape(sum(chunk), w.num_q_heads, -1), full[idx], rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(lse.reshape(sum(chunk), -1), full_lse[idx], rtol=1e-12, atol=1e-12)


def test_chunk_rows_against_sdpa_under_the_expanded_mask_and_never_touch_dropped_history():
    """Direct pin: torch attention under the boolean mask written out token by token, over keys = history values
    followed by the chunk.  History positions no streaming query of the chunk may see hold NaN for the streaming
    head (a bounded cache has dropped them); history values that are no 16-bit numbers (a dequantised cache) are
    taken as they are."""
    w = _prefill_workload(batch=1, sink_tokens=64, local_tokens=128)   # heads: KV head 0 streaming, 1 dense
    T, S, n = 64, 333, 150
    pin = make_prefill_inputs(w, lengths=(n,))
    g = np.random.default_rng(5)
    k_hist = g.standard_normal((1, S, w.num_kv_heads, w.head_dim)) * 1.37   # arbitrary doubles
    v_hist = g.standard_normal((1, S, w.num_kv_heads, w.head_dim))
    s_t, w_t = 1, 2
    first_tile = S // T
    for u in range(S):   # what the first chunk row cannot see, no later row can: sink tiles and the local band only
        if not (u // T < s_t or u // T > first_tile - w_t):
            k_hist[0, u, 0] = np.nan
            v_hist[0, u, 0] = np.nan
    tok, head = _all_rows(n, w.num_q_heads)
    out, lse = oracle.chunk_prefill_rows(pin.q, pin.k, pin.v, k_hist, v_hist, [S], [0, n], w.streaming_flags(), T,
                                         w.sink_tokens, w.local_tokens, tok, head)
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    out = out.reshape(n, w.num_q_heads, -1)
    q = pin.q.to(torch.float64).numpy()
    group = w.num_q_heads // w.num_kv_heads
    for j in (0, 1, 30, 31, 95, n - 1):
        t = S + j
        for h in range(w.num_q_heads):
            hk = h // group
            keys = np.concatenate([k_hist[0, :, hk], pin.k[:, hk].to(torch.float64).numpy()])
            vals = np.concatenate([v_hist[0, :, hk], pin.v[:, hk].to(torch.float64).numpy()])
            allowed = np.array([(u <= t) and (hk != 0 or u // T < s_t or u // T > t // T - w_t) for u in range(S + n)])
            ref = _sdpa(q[j, h], np.nan_to_num(keys), np.nan_to_num(vals), mask=allowed)
            np.testing.assert_allclose(out[j, h], ref, rtol=1e-10, atol=1e-12)

"""Pins for the oracle's key statistics, page scores (Eq. 2) and top-K selection.

Each check compares the oracle with something it does not compute itself: numpy
routines on the gathered keys, brute force over tokens, closed forms, bounds and
invariances.  A dropped term, wrong sign, wrong index or transposed operand in the
oracle fails at least one of them.
"""
import numpy as np
import pytest
import torch

import oracle
from workloads import make_decode_inputs

from helpers import gather_tokens, small_decode_workload


def _setup(**kw):
    w = small_decode_workload(**kw)
    inp = make_decode_inputs(w)
    seq = inp.seq_lens_at(0)
    stats = oracle.page_stats(inp.k_pool, inp.page_table, seq, w.logical_page_size)
    return w, inp, seq, stats


def test_widen_matches_numpy_and_torch_for_every_bit_pattern():
    bits = np.arange(65536, dtype=np.uint16)
    ref16 = bits.view(np.float16).astype(np.float64)
    refbf = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    for i in range(0, 65536, 7):
        a, b = oracle.widen(int(bits[i]), 0), oracle.widen(int(bits[i]), 1)
        assert (np.isnan(a) and np.isnan(ref16[i])) or a == ref16[i]
        assert (np.isnan(b) and np.isnan(refbf[i])) or b == refbf[i]


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
def test_stats_equal_numpy_min_max_over_gathered_keys(dtype):
    w, inp, seq, stats = _setup(dtype=dtype)
    NL, NP = w.logical_page_size, w.page_size
    g = NP // NL
    pt = inp.page_table.numpy()
    for b in range(w.batch):
        L = int(seq[b])
        K = gather_tokens(inp.k_pool, pt, b, L)  # [L, Hkv, D]
        for l in range((L + NL - 1) // NL):
            blk = K[l * NL:min(L, (l + 1) * NL)]
            page, j = pt[b, (l * NL) // NP], ((l * NL) % NP) // NL
            got = stats[page, :, j].to(torch.float64).numpy()  # [Hkv, 2, D]
            np.testing.assert_array_equal(got[:, 0], blk.max(axis=0))
            np.testing.assert_array_equal(got[:, 1], blk.min(axis=0))
            # bounds every token of the logical page, channel by channel
            assert (blk <= got[:, 0][None]).all() and (blk >= got[:, 1][None]).all()
    assert g == stats.shape[2]


def test_stats_do_not_depend_on_where_pages_sit_in_the_pool():
    w, inp, seq, stats = _setup()
    perm = torch.randperm(inp.num_pages, generator=torch.Generator().manual_seed(3))
    inv = torch.empty_like(perm)
    inv[perm] = torch.arange(inp.num_pages)
    k2 = inp.k_pool[perm]  # new page id i holds old page perm[i]
    pt2 = inv[inp.page_table.long()].to(torch.int32)
    stats2 = oracle.page_stats(k2, pt2, seq, w.logical_page_size)
    for b in range(w.batch):
        P = (int(seq[b]) + w.page_size - 1) // w.page_size
        for p in range(P - 1):  # full pages: every logical page is written
            a = stats[int(inp.page_table[b, p])]
            c = stats2[int(pt2[b, p])]
            assert torch.equal(a, c)


def _brute_logical_scores(w, inp, seq):
    """S_h^l = sum_c max_t (q_h[c] * K[t][c]) straight from the keys, no statistics involved."""
    NL = w.logical_page_size
    pt = inp.page_table.numpy()
    out = []
    for b in range(w.batch):
        L = int(seq[b])
        K = gather_tokens(inp.k_pool, pt, b, L)
        q = inp.q[0, b].to(torch.float64).numpy()  # [H, D]
        nl = (L + NL - 1) // NL
        s = np.zeros((w.num_q_heads, nl))
        for l in range(nl):
            blk = K[l * NL:min(L, (l + 1) * NL)]  # [t, Hkv, D]
            for h in range(w.num_q_heads):
                prod = blk[:, h // w.group, :] * q[h][None, :]  # [t, D]
                s[h, l] = prod.max(axis=0).sum()
        out.append(s)
    return out


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
def test_logical_scores_equal_sum_of_channelwise_max_over_tokens(dtype):
    w, inp, seq, stats = _setup(dtype=dtype)
    _, ls = oracle.page_scores(inp.q[0], stats, inp.page_table, seq, w.page_size, want_logical=True)
    g = w.page_size // w.logical_page_size
    brute = _brute_logical_scores(w, inp, seq)
    for b in range(w.batch):
        nl = brute[b].shape[1]
        got = ls[b].reshape(w.num_q_heads, -1)[:, :nl]  # [H, max_pages*g] -> logical order
        np.testing.assert_allclose(got, brute[b], rtol=1e-12, atol=1e-12)
        assert ls[b].shape[-1] == g


def test_score_upper_bounds_every_token_logit_and_is_tight_for_one_token_pages():
    w, inp, seq, stats = _setup()
    NL = w.logical_page_size
    _, ls = oracle.page_scores(inp.q[0], stats, inp.page_table, seq, w.page_size, want_logical=True)
    pt = inp.page_table.numpy()
    for b in range(w.batch):
        L = int(seq[b])
        K = gather_tokens(inp.k_pool, pt, b, L)
        q = inp.q[0, b].to(torch.float64).numpy()
        flat = ls[b].reshape(w.num_q_heads, -1)
        for h in range(w.num_q_heads):
            logits = K[:, h // w.group, :] @ q[h]  # [L]
            bound = np.repeat(flat[h], NL)[:L]
            assert (bound >= logits - 1e-9).all()
        if L % NL == 1:  # last logical page holds exactly one token: equality
            for h in range(w.num_q_heads):
                assert abs(flat[h, (L - 1) // NL] - K[L - 1, h // w.group] @ q[h]) < 1e-9
    # lengths (300+1, 777+1): 301 % 16 == 13, 778 % 16 == 10 -> force a one-token tail explicitly
    w2, inp2, _, _ = _setup(lengths=(320, 640))
    seq2 = inp2.seq_lens_at(0)  # 321, 641: both leave a single token in the last logical page
    st2 = oracle.page_stats(inp2.k_pool, inp2.page_table, seq2, w2.logical_page_size)
    _, ls2 = oracle.page_scores(inp2.q[0], st2, inp2.page_table, seq2, w2.page_size, want_logical=True)
    for b in range(w2.batch):
        L = int(seq2[b])
        K = gather_tokens(inp2.k_pool, inp2.page_table.numpy(), b, L)
        q = inp2.q[0, b].to(torch.float64).numpy()
        for h in range(w2.num_q_heads):
            tight = ls2[b].reshape(w2.num_q_heads, -1)[h, (L - 1) // NL]
            assert abs(tight - K[L - 1, h // w2.group] @ q[h]) < 1e-9


def test_constant_page_scores_q_dot_k():
    w, inp, seq, _ = _setup()
    # overwrite every key of sequence 0's page 1 with one vector: the score must be q . k
    page = int(inp.page_table[0, 1])
    vec = inp.k_pool[page, :, 0].clone()  # [Hkv, D]
    inp.k_pool[page] = vec[:, None, :]
    stats = oracle.page_stats(inp.k_pool, inp.page_table, seq, w.logical_page_size)
    _, ls = oracle.page_scores(inp.q[0], stats, inp.page_table, seq, w.page_size, want_logical=True)
    q = inp.q[0, 0].to(torch.float64).numpy()
    for h in range(w.num_q_heads):
        want = q[h] @ vec[h // w.group].to(torch.float64).numpy()
        np.testing.assert_allclose(ls[0, h, 1], want, rtol=0, atol=1e-9)


def test_page_score_is_group_max_then_logical_max_and_tighter_than_flat_paging():
    w, inp, seq, stats = _setup()
    ps, ls = oracle.page_scores(inp.q[0], stats, inp.page_table, seq, w.page_size, want_logical=True)
    brute = _brute_logical_scores(w, inp, seq)
    g = w.page_size // w.logical_page_size
    # flat paging: one logical page per physical page (g = 1)
    stats_flat = oracle.page_stats(inp.k_pool, inp.page_table, seq, w.page_size)
    ps_flat, _ = oracle.page_scores(inp.q[0], stats_flat, inp.page_table, seq, w.page_size)
    for b in range(w.batch):
        L = int(seq[b])
        P = (L + w.page_size - 1) // w.page_size
        nl = brute[b].shape[1]
        padded = np.full((w.num_q_heads, P * g), -np.inf)
        padded[:, :nl] = brute[b]
        per_head_page = padded.reshape(w.num_q_heads, P, g).max(axis=2)  # max over logical pages
        want = per_head_page.reshape(w.num_kv_heads, w.group, P).max(axis=1)  # max over the group
        np.testing.assert_allclose(ps[b, :, :P], want, rtol=1e-12)
        assert (ps[b, :, P:] == 0).all()
        # hierarchical bound is never looser than the flat one at physical page size
        assert (ps[b, :, :P] <= ps_flat[b, :, :P] + 1e-9).all()
    # with MHA (group of one) the page score is Eq. 2 followed by the max over logical pages
    w1, inp1, seq1, st1 = _setup(num_q_heads=2, num_kv_heads=2)
    ps1, ls1 = oracle.page_scores(inp1.q[0], st1, inp1.page_table, seq1, w1.page_size, want_logical=True)
    for b in range(w1.batch):
        P = (int(seq1[b]) + 63) // 64
        np.testing.assert_allclose(ps1[b, :, :P - 1], ls1[b, :, :P - 1].max(axis=-1), rtol=1e-12)


def _exhaustive_topk(scores_row, P, K):
    """All pages ranked by score (stable: lower index first among equals); newest page forced."""
    if P <= K:
        return list(range(P))
    order = sorted(range(P - 1), key=lambda p: (-scores_row[p], p))
    return sorted(order[:K - 1] + [P - 1])


def test_selection_equals_exhaustive_ranking():
    w, inp, seq, stats = _setup(budget_tokens=256, lengths=(300, 2000))
    ps, _ = oracle.page_scores(inp.q[0], stats, inp.page_table, seq, w.page_size)
    sel, cnt, ssl = oracle.select_pages(ps, seq, w.page_size, w.budget_tokens)
    K = w.budget_tokens // w.page_size
    brute = _brute_logical_scores(w, inp, seq)
    g = w.page_size // w.logical_page_size
    for b in range(w.batch):
        L = int(seq[b])
        P = (L + w.page_size - 1) // w.page_size
        padded = np.full((w.num_q_heads, P * g), -np.inf)
        padded[:, :brute[b].shape[1]] = brute[b]
        page_sc = padded.reshape(w.num_kv_heads, w.group, P, g).max(axis=(1, 3))
        for hk in range(w.num_kv_heads):
            want = _exhaustive_topk(page_sc[hk], P, K)
            got = list(sel[b, hk, :cnt[b, hk]])
            assert got == want
            assert got == sorted(set(got)) and got[-1] == P - 1 and max(got) < P
            assert (sel[b, hk, cnt[b, hk]:] == -1).all()
        assert ssl[b] == L


def test_selection_takes_all_pages_when_budget_covers_context_and_breaks_ties_low():
    seq = np.array([64 * 5 + 3, 64 * 9], dtype=np.int32)
    scores = np.zeros((2, 1, 12))
    scores[1, 0, :9] = [1.0, 5.0, 5.0, 2.0, 5.0, 0.5, 5.0, 9.0, -3.0]
    sel, cnt, _ = oracle.select_pages(scores, seq, 64, 64 * 6)
    assert cnt[0, 0] == 6 and list(sel[0, 0, :6]) == [0, 1, 2, 3, 4, 5]
    # K = 6 of P = 9: forced page 8, then 9.0 (page 7) and the four 5.0s -> pages 1, 2, 4, 6
    assert list(sel[1, 0, :cnt[1, 0]]) == [1, 2, 4, 6, 7, 8]
    sel, cnt, _ = oracle.select_pages(scores, seq, 64, 64 * 4)
    # K = 4: forced 8, page 7, then two of the tied 5.0s: the lower indices 1 and 2
    assert list(sel[1, 0, :cnt[1, 0]]) == [1, 2, 7, 8]


def test_planted_needles_are_selected_and_selection_ignores_pool_placement():
    w, inp, seq, stats = _setup(needles_per_seq=3, lengths=(3000, 5000), budget_tokens=512,
                                sink_tokens=128, local_tokens=256)
    ps, _ = oracle.page_scores(inp.q[0], stats, inp.page_table, seq, w.page_size)
    sel, cnt, _ = oracle.select_pages(ps, seq, w.page_size, w.budget_tokens)
    for b in range(w.batch):
        for hk in range(w.num_kv_heads):
            if hk in w.streaming_kv_heads:
                continue
            chosen = set(sel[b, hk, :cnt[b, hk]].tolist())
            for pos in inp.needle_pos[b].tolist():
                assert pos // w.page_size in chosen
    perm = torch.randperm(inp.num_pages, generator=torch.Generator().manual_seed(5))
    inv = torch.empty_like(perm)
    inv[perm] = torch.arange(inp.num_pages)
    pt2 = inv[inp.page_table.long()].to(torch.int32)
    st2 = oracle.page_stats(inp.k_pool[perm], pt2, seq, w.logical_page_size)
    ps2, _ = oracle.page_scores(inp.q[0], st2, pt2, seq, w.page_size)
    sel2, cnt2, _ = oracle.select_pages(ps2, seq, w.page_size, w.budget_tokens)
    assert np.array_equal(sel, sel2) and np.array_equal(cnt, cnt2)

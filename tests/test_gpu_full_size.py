"""Full-size configurations in the launch shape the benchmark times, checked on sampled outputs.

The oracle cannot run the whole workload in seconds, so a few sequences (decode) or rows (prefill)
are checked element by element: their pages are gathered into a small pool for the oracle while the
GPU runs the complete problem.
"""
import numpy as np
import pytest
import torch

import oracle
from workloads import get_config, make_decode_inputs, make_prefill_inputs

from helpers import sub_problem
from parity import LSE_TOL_PREFILL, SCORE_REL_TOL, assert_attention_close, assert_lse_close, compare_selection

pytestmark = pytest.mark.gpu


def _run_decode_config(name, seqs, steps, **over):
    import paper_2502_14866_amd as L
    from paper_2502_14866_amd.session import DecodeSession

    L.load_library()
    dev = torch.device("cuda:0")
    w = get_config(name, **over)
    inp = make_decode_inputs(w, device=dev)
    B, C = w.batch, w.reuse_interval
    sess = DecodeSession(inp.k_pool, inp.v_pool, inp.page_table, w.num_q_heads, w.streaming_flags(), w.sink_tokens,
                         w.local_tokens, w.budget_tokens, logical_page_size=w.logical_page_size, reuse_interval=C,
                         want_scores=True)
    pad = (B + 3) // 4 * 4
    lens = torch.zeros((steps + 1, pad), dtype=torch.int32, device=dev)
    for t in range(steps + 1):
        lens[t, :B] = inp.prompt_lens + t
    sess.set_seq_lens(lens[0, :B])
    sess.build_stats_full()
    sub = sub_problem(inp, seqs)
    sw = sub.workload
    flags = w.streaming_flags()
    near_ties = 0
    for t in range(steps):
        out = sess.step(inp.q[t], lens[t + 1, :B], lens[t, :B])
        seq_cpu = sub.seq_lens_at(t)
        sel_gpu = sess.sel_pages.cpu().numpy()[list(seqs)]
        cnt_gpu = sess.sel_count.cpu().numpy()[list(seqs)]
        ssl_gpu = sess.sel_seq_len.cpu().numpy()[list(seqs)]
        if t % C == 0:
            stats = oracle.page_stats(sub.k_pool, sub.page_table, seq_cpu, sw.logical_page_size)
            scores, _ = oracle.page_scores(sub.q[t], stats, sub.page_table, seq_cpu, sw.page_size)
            sel_ref, cnt_ref, ssl_ref = oracle.select_pages(scores, seq_cpu, sw.page_size, sw.budget_tokens)
            got_scores = sess.scores.cpu().numpy()[list(seqs)].astype(np.float64)
            for hk in range(w.num_kv_heads):
                if not flags[hk]:
                    np.testing.assert_allclose(got_scores[:, hk], scores[:, hk], rtol=SCORE_REL_TOL, atol=1e-4)
            near_ties += compare_selection(sel_gpu, cnt_gpu, sel_ref, cnt_ref, scores, flags)
            assert np.array_equal(ssl_gpu, ssl_ref)
            if sub.needle_pos is not None and t == 0:
                for i in range(len(seqs)):
                    for hk in range(w.num_kv_heads):
                        if flags[hk]:
                            continue
                        chosen = set(sel_gpu[i, hk, :cnt_gpu[i, hk]].tolist())
                        assert all(int(p) // w.page_size in chosen for p in sub.needle_pos[i])
        ref, _ = oracle.sparse_decode(sub.q[t], sub.k_pool, sub.v_pool, sub.page_table, seq_cpu, sel_gpu, cnt_gpu,
                                      ssl_gpu, flags, w.sink_tokens, w.local_tokens)
        assert_attention_close(out[list(seqs)], ref, f"{name} step {t}")
    print(f"[{name}] sampled sequences {list(seqs)}: near-tie selections {near_ties}")
    return near_ties


def test_cfg2_full_size_decode_sampled_sequences():
    assert _run_decode_config("cfg2", seqs=(0, 7, 15), steps=6) <= 1


def test_cfg4_long_context_decode_retrieves_needles():
    assert _run_decode_config("cfg4", seqs=(1, 3), steps=5) <= 1


def test_more_than_8192_candidate_pages_take_the_top_k_path_that_ranks_from_memory():
    """16-token pages at 140000 tokens: 8750 pages per sequence, more than the selector keeps in LDS."""
    assert _run_decode_config("cfg4", seqs=(0, 1), steps=5, batch=2, context=140000, page_size=16,
                              logical_page_size=16) <= 1


def test_cfg5_ragged_mha_decode_sampled_sequences():
    assert _run_decode_config("cfg5", seqs=(0, 13, 31), steps=5) <= 1


def test_cfg3_full_size_prefill_sampled_rows():
    import paper_2502_14866_amd as L

    L.load_library()
    dev = torch.device("cuda:0")
    w = get_config("cfg3")
    pin = make_prefill_inputs(w, device=dev)
    desc = L.AttnDesc(w.num_q_heads, w.num_kv_heads, w.streaming_flags(), dtype=w.torch_dtype,
                      sink_tokens=w.sink_tokens, local_tokens=w.local_tokens)
    n = w.prefill_tokens
    ws = torch.empty((L.lserve_workspace_bytes(L.LSERVE_CALL_SPARSE_PREFILL, desc, 1, 0, 0, n),), dtype=torch.uint8,
                     device=dev)
    out = torch.empty_like(pin.q)
    lse = torch.empty((w.num_q_heads, n), dtype=torch.float32, device=dev)
    L.lserve_sparse_prefill(desc, pin.q, pin.k, pin.v, pin.cu_seqlens, n, out, lse, ws)
    torch.cuda.synchronize()
    rng = np.random.default_rng(3)
    rows = np.unique(np.concatenate([[0, 1, 63, 64, 65, 127, 128, 255, 256, 639, 640, 641, n - 65, n - 64, n - 1],
                                     rng.integers(0, n, size=9)])).astype(np.int32)
    heads = np.arange(w.num_q_heads, dtype=np.int32)  # every head: streaming 0-15, dense 16-31
    tok = np.repeat(rows, len(heads))
    hd = np.tile(heads, len(rows))
    q, k, v = pin.q.cpu(), pin.k.cpu(), pin.v.cpu()
    ref, lse_ref = oracle.sparse_prefill_rows(q, k, v, pin.cu_seqlens.cpu(), w.streaming_flags(), 64, w.sink_tokens,
                                              w.local_tokens, tok, hd)
    got = out[torch.from_numpy(tok).long().to(dev), torch.from_numpy(hd).long().to(dev)]
    assert_attention_close(got, ref, "cfg3 sampled rows")
    got_lse = lse[torch.from_numpy(hd).long().to(dev), torch.from_numpy(tok).long().to(dev)].cpu().numpy()
    assert_lse_close(torch.from_numpy(got_lse), lse_ref, "cfg3 sampled rows lse", LSE_TOL_PREFILL["bf16"])

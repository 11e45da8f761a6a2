"""Parity of the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

import oracle
from workloads import Workload, get_config, make_decode_inputs, make_prefill_inputs, scatter_prefill_kv_to_pages

from helpers import small_decode_workload
from parity import LSE_TOL_PREFILL, SCORE_REL_TOL, assert_attention_close, assert_lse_close, compare_selection

pytestmark = pytest.mark.gpu


def _lib():
    import paper_2502_14866_amd as L

    L.load_library()
    return L


def _session(L, w, inp, dev, want_scores=True, want_lse=True):
    from paper_2502_14866_amd.session import DecodeSession

    return DecodeSession(inp.k_pool.to(dev), inp.v_pool.to(dev), inp.page_table.to(dev), w.num_q_heads,
                         w.streaming_flags(), w.sink_tokens, w.local_tokens, w.budget_tokens,
                         logical_page_size=w.logical_page_size, reuse_interval=w.reuse_interval,
                         want_scores=want_scores, want_lse=want_lse)


def _check_stats(w, inp, sess, seq_cpu):
    """Statistics of every non-empty logical page of the non-streaming heads, value for value."""
    ref = oracle.page_stats(inp.k_pool, inp.page_table, seq_cpu, w.logical_page_size)
    got = sess.stats.cpu()
    pt = inp.page_table.numpy()
    g = w.page_size // w.logical_page_size
    heads = [h for h in range(w.num_kv_heads) if h not in w.streaming_kv_heads]
    for b in range(w.batch):
        L_b = int(seq_cpu[b])
        P = (L_b + w.page_size - 1) // w.page_size
        pages = torch.from_numpy(pt[b, :P]).long()
        full = pages[:P - 1]
        for hk in heads:
            assert torch.equal(got[full, hk].float(), ref[full, hk].float()), (b, hk)
            tail_valid = -(-(L_b - (P - 1) * w.page_size) // w.logical_page_size)
            assert torch.equal(got[pages[-1], hk, :tail_valid].float(), ref[pages[-1], hk, :tail_valid].float())
    return ref


WORKLOADS = {
    "tiny_gqa": dict(),
    "ragged_tail": dict(lengths=(1, 63), decode_steps=3),
    "mha": dict(num_q_heads=4, num_kv_heads=4, streaming_kv_heads=(1, 3), lengths=(900, 130, 2049), batch=3),
    "gqa8_bf16": dict(num_q_heads=16, num_kv_heads=2, dtype="bf16", streaming_kv_heads=(1,), lengths=(4100, 700),
                      budget_tokens=1024),
    "all_streaming": dict(streaming_kv_heads=(0, 1), lengths=(5000, 200)),
    "all_dense_page32": dict(streaming_kv_heads=(), page_size=32, logical_page_size=8, lengths=(3000, 1500),
                             budget_tokens=512),
    "page128_g8": dict(page_size=128, logical_page_size=16, lengths=(6000, 3000), budget_tokens=1024,
                       sink_tokens=128, local_tokens=256),
    "page16_flat": dict(page_size=16, logical_page_size=16, lengths=(700, 333), budget_tokens=128, sink_tokens=16,
                        local_tokens=64),
    "group3": dict(num_q_heads=6, num_kv_heads=2, lengths=(1500, 2600), budget_tokens=512),
    "hkv64": dict(num_q_heads=64, num_kv_heads=64, streaming_kv_heads=tuple(range(1, 64, 2)), lengths=(300, 70),
                  budget_tokens=128, decode_steps=3),
    "hkv64_n8": dict(num_q_heads=512, num_kv_heads=64, streaming_kv_heads=tuple(range(0, 64, 3)), lengths=(200, 129),
                     budget_tokens=128, decode_steps=2),
    # 32 selecting heads x (2048 + 1) index-table entries per sequence = 65568: more than 16 bits of entries, the
    # budget covers the context (so the decode is dense attention over every page)
    "wide_tables_mha32": dict(num_q_heads=32, num_kv_heads=32, streaming_kv_heads=(), lengths=(300, 777),
                              budget_tokens=2048 * 64, decode_steps=2),
}


@pytest.mark.parametrize("name", list(WORKLOADS))
def test_decode_loop_matches_oracle(name):
    """Statistics, scores, selection (bit-exact sets) and decode output over a short decode loop."""
    L = _lib()
    dev = torch.device("cuda:0")
    kw = dict(WORKLOADS[name])
    kw.setdefault("decode_steps", 5)
    kw.setdefault("reuse_interval", 2)
    w = small_decode_workload(**kw)
    inp = make_decode_inputs(w)
    sess = _session(L, w, inp, dev)
    flags = w.streaming_flags()
    near_ties = 0
    sel_ref = cnt_ref = ssl_ref = None
    prev = inp.prompt_lens.to(dev)
    for step in range(w.decode_steps):
        seq_cpu = inp.seq_lens_at(step)
        seq = seq_cpu.to(dev)
        q = inp.q[step].to(dev)
        sess.set_seq_lens(seq)
        if step == 0:
            sess.build_stats_full()
        else:
            sess.update_stats_tail(prev, 1)
        stats_ref = _check_stats(w, inp, sess, seq_cpu)
        if step % w.reuse_interval == 0:
            sess.select(q)
            scores_ref, _ = oracle.page_scores(inp.q[step], stats_ref, inp.page_table, seq_cpu, w.page_size)
            sel_ref, cnt_ref, ssl_ref = oracle.select_pages(scores_ref, seq_cpu, w.page_size, w.budget_tokens)
            got_scores = sess.scores.cpu().numpy().astype(np.float64)
            for hk in range(w.num_kv_heads):
                if flags[hk]:
                    assert (got_scores[:, hk] == 0).all()
                else:
                    np.testing.assert_allclose(got_scores[:, hk], scores_ref[:, hk], rtol=SCORE_REL_TOL, atol=1e-4)
            near_ties += compare_selection(sess.sel_pages.cpu().numpy(), sess.sel_count.cpu().numpy(), sel_ref,
                                           cnt_ref, scores_ref, flags)
            assert np.array_equal(sess.sel_seq_len.cpu().numpy(), ssl_ref)
        out = sess.decode(q)
        # the oracle attends the GPU's own selection, so a near-tie cannot leak into this comparison
        ref, lse_ref = oracle.sparse_decode(inp.q[step], inp.k_pool, inp.v_pool, inp.page_table, seq_cpu,
                                            sess.sel_pages.cpu().numpy(), sess.sel_count.cpu().numpy(),
                                            sess.sel_seq_len.cpu().numpy(), flags, w.sink_tokens, w.local_tokens)
        assert_attention_close(out, ref, f"{name} step {step}")
        assert_lse_close(sess.lse, lse_ref, f"{name} step {step}")
        prev = seq
    print(f"[{name}] near-tie selections: {near_ties}")
    assert near_ties <= 1


def test_decode_ignores_nan_in_slots_past_the_sequence_end():
    L = _lib()
    dev = torch.device("cuda:0")
    w = small_decode_workload(lengths=(70, 130), decode_steps=1, budget_tokens=1024)
    inp = make_decode_inputs(w)
    seq_cpu = inp.seq_lens_at(0)
    for b in range(w.batch):  # poison every slot past the end of the tail page
        Lb = int(seq_cpu[b])
        page = int(inp.page_table[b, (Lb - 1) // 64])
        inp.k_pool[page, :, Lb % 64:] = float("nan")
        inp.v_pool[page, :, Lb % 64:] = float("nan")
    sess = _session(L, w, inp, dev)
    sess.set_seq_lens(seq_cpu.to(dev))
    sess.build_stats_full()
    sess.select(inp.q[0].to(dev))
    out = sess.decode(inp.q[0].to(dev))
    ref, _ = oracle.sparse_decode(inp.q[0], inp.k_pool, inp.v_pool, inp.page_table, seq_cpu,
                                  sess.sel_pages.cpu().numpy(), sess.sel_count.cpu().numpy(),
                                  sess.sel_seq_len.cpu().numpy(), w.streaming_flags(), w.sink_tokens, w.local_tokens)
    assert_attention_close(out, ref, "nan tail")


def test_decode_is_deterministic_and_stale_selection_adds_new_pages():
    L = _lib()
    dev = torch.device("cuda:0")
    w = small_decode_workload(lengths=(1000, 1900), decode_steps=140, budget_tokens=512)
    inp = make_decode_inputs(w)
    sess = _session(L, w, inp, dev)
    sess.set_seq_lens(inp.seq_lens_at(0).to(dev))
    sess.build_stats_full()
    sess.select(inp.q[0].to(dev))
    step = 139  # 139 tokens later: two or three pages are newer than the selection
    seq_cpu = inp.seq_lens_at(step)
    sess.set_seq_lens(seq_cpu.to(dev))
    q = inp.q[step].to(dev)
    a = sess.decode(q).clone()
    b = sess.decode(q).clone()
    assert torch.equal(a, b)
    ref, _ = oracle.sparse_decode(inp.q[step], inp.k_pool, inp.v_pool, inp.page_table, seq_cpu,
                                  sess.sel_pages.cpu().numpy(), sess.sel_count.cpu().numpy(),
                                  sess.sel_seq_len.cpu().numpy(), w.streaming_flags(), w.sink_tokens, w.local_tokens)
    assert_attention_close(a, ref, "stale selection")


def test_planted_needles_are_retrieved_by_the_gpu_selector():
    L = _lib()
    dev = torch.device("cuda:0")
    w = get_config("cfg4", context=16384, batch=2, decode_steps=1)
    inp = make_decode_inputs(w)
    sess = _session(L, w, inp, dev)
    seq_cpu = inp.seq_lens_at(0)
    sess.set_seq_lens(seq_cpu.to(dev))
    sess.build_stats_full()
    sess.select(inp.q[0].to(dev))
    sel, cnt = sess.sel_pages.cpu().numpy(), sess.sel_count.cpu().numpy()
    for b in range(w.batch):
        for hk in range(4, 8):
            chosen = set(sel[b, hk, :cnt[b, hk]].tolist())
            for pos in inp.needle_pos[b].tolist():
                assert pos // 64 in chosen


def _prefill(L, w, pin, dev, max_seqlen=None):
    desc = L.AttnDesc(w.num_q_heads, w.num_kv_heads, w.streaming_flags(), dtype=w.torch_dtype,
                      sink_tokens=w.sink_tokens, local_tokens=w.local_tokens)
    q, k, v = pin.q.to(dev), pin.k.to(dev), pin.v.to(dev)
    cu = pin.cu_seqlens.to(dev)
    total = q.shape[0]
    lens = (pin.cu_seqlens[1:] - pin.cu_seqlens[:-1]).tolist()
    ws = torch.empty((L.lserve_workspace_bytes(L.LSERVE_CALL_SPARSE_PREFILL, desc, len(lens), 0, 0, total),),
                     dtype=torch.uint8, device=dev)
    out = torch.full_like(q, float("nan"))
    lse = torch.empty((w.num_q_heads, total), dtype=torch.float32, device=dev)
    L.lserve_sparse_prefill(desc, q, k, v, cu, max_seqlen or max(lens), out, lse, ws)
    torch.cuda.synchronize()
    return out, lse


def _oracle_rows(w, pin, tok, head):
    return oracle.sparse_prefill_rows(pin.q, pin.k, pin.v, pin.cu_seqlens, w.streaming_flags(), 64, w.sink_tokens,
                                      w.local_tokens, tok, head)


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
@pytest.mark.parametrize("lengths", [(1,), (64,), (65, 300), (777, 256, 1000)])
def test_prefill_matches_oracle_on_every_row(dtype, lengths):
    L = _lib()
    dev = torch.device("cuda:0")
    w = Workload(name="p", batch=len(lengths), num_q_heads=4, num_kv_heads=2, dtype=dtype, streaming_kv_heads=(0,),
                 sink_tokens=64, local_tokens=192, seed=21)
    pin = make_prefill_inputs(w, lengths=lengths)
    out, lse = _prefill(L, w, pin, dev)
    total = sum(lengths)
    tok = np.repeat(np.arange(total, dtype=np.int32), w.num_q_heads)
    head = np.tile(np.arange(w.num_q_heads, dtype=np.int32), total)
    ref, lse_ref = _oracle_rows(w, pin, tok, head)
    assert_attention_close(out, ref.reshape(total, w.num_q_heads, -1), f"prefill {dtype} {lengths}")
    assert_lse_close(lse.t().contiguous(), lse_ref.reshape(total, w.num_q_heads), "prefill lse", LSE_TOL_PREFILL[dtype])


def test_cfg1_prefill_then_decode_full_comparison():
    """Config 1: 2048-token prefill compared on every row, K/V scattered to pages, one decode step."""
    L = _lib()
    dev = torch.device("cuda:0")
    w = get_config("cfg1")
    pin = make_prefill_inputs(w)
    out, _ = _prefill(L, w, pin, dev)
    total = w.prefill_tokens
    tok = np.repeat(np.arange(total, dtype=np.int32), w.num_q_heads)
    head = np.tile(np.arange(w.num_q_heads, dtype=np.int32), total)
    ref, _ = _oracle_rows(w, pin, tok, head)
    assert_attention_close(out, ref.reshape(total, w.num_q_heads, -1), "cfg1 prefill")

    inp = make_decode_inputs(w)
    scatter_prefill_kv_to_pages(pin.k, pin.v, pin.cu_seqlens.tolist(), inp.k_pool, inp.v_pool, inp.page_table)
    sess = _session(L, w, inp, dev)
    seq_cpu = inp.seq_lens_at(0)  # 2049
    sess.set_seq_lens(seq_cpu.to(dev))
    sess.build_stats_full()
    stats_ref = _check_stats(w, inp, sess, seq_cpu)
    q = inp.q[0].to(dev)
    sess.select(q)
    scores_ref, _ = oracle.page_scores(inp.q[0], stats_ref, inp.page_table, seq_cpu, w.page_size)
    sel_ref, cnt_ref, _ = oracle.select_pages(scores_ref, seq_cpu, w.page_size, w.budget_tokens)
    ties = compare_selection(sess.sel_pages.cpu().numpy(), sess.sel_count.cpu().numpy(), sel_ref, cnt_ref,
                             scores_ref, w.streaming_flags())
    assert ties == 0
    dec = sess.decode(q)
    dref, _ = oracle.sparse_decode(inp.q[0], inp.k_pool, inp.v_pool, inp.page_table, seq_cpu,
                                   sess.sel_pages.cpu().numpy(), sess.sel_count.cpu().numpy(),
                                   sess.sel_seq_len.cpu().numpy(), w.streaming_flags(), w.sink_tokens, w.local_tokens)
    assert_attention_close(dec, dref, "cfg1 decode")


def test_hip_graph_replays_of_a_decode_episode_equal_the_eager_run():
    """An episode (statistics update, selection every C steps, decode) captured in a HIP graph must
    reproduce the eager results bit for bit on every replay, with eager work between replays."""
    L = _lib()
    from paper_2502_14866_amd.session import DecodeSession

    dev = torch.device("cuda:0")
    w = small_decode_workload(batch=4, lengths=(3000, 700, 5000, 64), decode_steps=8, reuse_interval=4,
                              budget_tokens=1024, num_q_heads=8, num_kv_heads=2)
    inp = make_decode_inputs(w, device=dev)
    E, B = w.decode_steps, w.batch
    sess = DecodeSession(inp.k_pool, inp.v_pool, inp.page_table, w.num_q_heads, w.streaming_flags(), w.sink_tokens,
                         w.local_tokens, w.budget_tokens, reuse_interval=w.reuse_interval)
    lens = torch.zeros((E + 1, 4), dtype=torch.int32, device=dev)
    for t in range(E + 1):
        lens[t, :B] = inp.prompt_lens + t
    sess.set_seq_lens(lens[0, :B])
    sess.build_stats_full()
    outs = torch.zeros((E,) + tuple(sess.out.shape), dtype=sess.out.dtype, device=dev)

    def episode():
        sess.restart()
        for t in range(E):
            sess.step(inp.q[t], lens[t + 1, :B], lens[t, :B])
            outs[t].copy_(sess.out)

    episode()
    torch.cuda.synchronize()
    eager = outs.clone()
    sel_eager = sess.sel_pages.clone()
    assert torch.isfinite(eager.float()).all()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        episode()
    torch.cuda.synchronize()
    for rep in range(4):
        outs.fill_(0)
        sess.sel_pages.fill_(-7)  # eager work between replays; the graph must rebuild all of it
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(outs, eager), f"replay {rep} differs from the eager episode"
        assert torch.equal(sess.sel_pages, sel_eager)


@pytest.mark.parametrize("fused_stats", [True, False])
def test_session_step_loop_with_lazy_statistics_matches_oracle(fused_stats):
    """DecodeSession.step refreshes the statistics only at a selector run (inside the scoring kernel, or by a
    separate launch right before it); the statistics left behind, the selection made then and every step's
    output must still match the oracle."""
    L = _lib()
    dev = torch.device("cuda:0")
    w = small_decode_workload(batch=3, lengths=(1000, 127, 2500), decode_steps=9, reuse_interval=4,
                              budget_tokens=512)
    inp = make_decode_inputs(w)
    sess = _session(L, w, inp, dev)
    sess.fused_stats = fused_stats
    flags = w.streaming_flags()
    lens = torch.zeros((w.decode_steps + 1, 4), dtype=torch.int32, device=dev)
    for t in range(w.decode_steps + 1):
        lens[t, :w.batch] = inp.prompt_lens.to(dev) + t
    sess.set_seq_lens(lens[0, :w.batch])
    sess.build_stats_full()
    near_ties = 0
    for t in range(w.decode_steps):
        seq_cpu = inp.seq_lens_at(t)
        out = sess.step(inp.q[t].to(dev), lens[t + 1, :w.batch], lens[t, :w.batch])
        if t % w.reuse_interval == 0:
            stats_ref = _check_stats(w, inp, sess, seq_cpu)
            scores_ref, _ = oracle.page_scores(inp.q[t], stats_ref, inp.page_table, seq_cpu, w.page_size)
            sel_ref, cnt_ref, _ = oracle.select_pages(scores_ref, seq_cpu, w.page_size, w.budget_tokens)
            near_ties += compare_selection(sess.sel_pages.cpu().numpy(), sess.sel_count.cpu().numpy(), sel_ref,
                                           cnt_ref, scores_ref, flags)
        ref, _ = oracle.sparse_decode(inp.q[t], inp.k_pool, inp.v_pool, inp.page_table, seq_cpu,
                                      sess.sel_pages.cpu().numpy(), sess.sel_count.cpu().numpy(),
                                      sess.sel_seq_len.cpu().numpy(), flags, w.sink_tokens, w.local_tokens)
        assert_attention_close(out, ref, f"session step {t}")
    print(f"[session loop, fused_stats={fused_stats}] near-tie selections {near_ties}")
    assert near_ties <= 1


def test_selector_rebuilds_every_stale_logical_page_itself():
    """stats_valid_len = 0, a page boundary and the current length: the selector's own statistics pass must
    leave the same statistics, scores and selection as a full rebuild followed by a plain selector run."""
    L = _lib()
    dev = torch.device("cuda:0")
    w = small_decode_workload(batch=3, lengths=(1500, 640, 2100), budget_tokens=512, dtype="bf16")
    inp = make_decode_inputs(w)
    seq_cpu = inp.seq_lens_at(0)
    q = inp.q[0].to(dev)
    ref = _session(L, w, inp, dev)
    ref.set_seq_lens(seq_cpu.to(dev))
    ref.build_stats_full()
    ref.select(q)
    got = _session(L, w, inp, dev)
    got.set_seq_lens(seq_cpu.to(dev))
    got.build_stats_full()
    valid = torch.tensor([0, 640, int(seq_cpu[2]), 0], dtype=torch.int32, device=dev)[:3]
    # spoil everything the selector is told to rebuild, so that reading a stored row there would show
    for b in range(3):
        if int(valid[b]) >= int(seq_cpu[b]):
            continue  # nothing is stale for this sequence
        lo_page = int(valid[b]) // w.page_size
        pages = inp.page_table[b, lo_page:(int(seq_cpu[b]) + w.page_size - 1) // w.page_size].long().to(dev)
        lo_logical = (int(valid[b]) % w.page_size) // w.logical_page_size
        got.stats[pages[1:]] = float("nan")
        if len(pages):
            got.stats[pages[0], :, lo_logical:] = float("nan")
    got.select(q, stats_valid_len=valid)
    torch.cuda.synchronize()
    _check_stats(w, inp, got, seq_cpu)
    assert torch.equal(got.sel_pages, ref.sel_pages) and torch.equal(got.sel_count, ref.sel_count)
    assert torch.equal(got.scores, ref.scores)


@pytest.mark.parametrize("length", [4800, 24000, 80000, 140000])
def test_exact_ties_go_to_the_lower_page_index_in_every_ranking_path(length):
    """All keys zero but for a handful of pages: almost every score is exactly 0, so the budget is filled from a
    huge tie.  16-token pages at these lengths give 300, 1500, 5000 and 8750 candidate pages: one wavefront, four
    and eight wavefronts ranking from registers, and the ranking from memory.  The selection must equal the
    oracle's, which takes ties in index order, entry for entry."""
    L = _lib()
    dev = torch.device("cuda:0")
    w = small_decode_workload(batch=2, lengths=(length, length // 2 + 5), budget_tokens=16 * 24, page_size=16,
                              logical_page_size=16, sink_tokens=16, local_tokens=32)
    inp = make_decode_inputs(w)
    seq_cpu = inp.seq_lens_at(0)
    inp.k_pool.zero_()
    rng = np.random.default_rng(length)
    for b in range(2):
        n_pages = (int(seq_cpu[b]) + 15) // 16
        for p in rng.choice(n_pages - 1, size=5, replace=False):  # a few pages that do stand out
            inp.k_pool[inp.page_table[b, p].long()] = torch.randn((w.num_kv_heads, 16, 128)).to(inp.k_pool.dtype)
    sess = _session(L, w, inp, dev)
    sess.set_seq_lens(seq_cpu.to(dev))
    sess.build_stats_full()
    sess.select(inp.q[0].to(dev))
    torch.cuda.synchronize()
    stats_ref = oracle.page_stats(inp.k_pool, inp.page_table, seq_cpu, w.logical_page_size)
    scores_ref, _ = oracle.page_scores(inp.q[0], stats_ref, inp.page_table, seq_cpu, w.page_size)
    sel_ref, cnt_ref, _ = oracle.select_pages(scores_ref, seq_cpu, w.page_size, w.budget_tokens)
    flags = w.streaming_flags()
    sel, cnt = sess.sel_pages.cpu().numpy(), sess.sel_count.cpu().numpy()
    for hk in range(w.num_kv_heads):
        if flags[hk]:
            continue
        assert (scores_ref[:, hk] == 0).mean() > 0.9  # the tie is there
        assert np.array_equal(cnt[:, hk], cnt_ref[:, hk])
        assert np.array_equal(sel[:, hk], sel_ref[:, hk]), f"KV head {hk}"


@pytest.mark.parametrize("case", [
    dict(lengths=(1500, 300, 2100), budget_tokens=512),                                    # one list fits the budget whole
    dict(lengths=(40000, 700), budget_tokens=512, page_size=16, logical_page_size=16),     # several wavefronts per list
    dict(lengths=(140000, 5000), budget_tokens=512, page_size=16, logical_page_size=16),   # ranking from memory
])
def test_a_callers_score_array_reads_zero_past_the_last_page_and_for_streaming_heads(case):
    """The scoring launch writes only the pages a sequence has; the zeros of the header's contract (entries at or
    past P_b, rows of streaming heads) come from the ranking launch.  The array is poisoned first."""
    L = _lib()
    dev = torch.device("cuda:0")
    w = small_decode_workload(batch=len(case["lengths"]), **case)
    inp = make_decode_inputs(w)
    seq_cpu = inp.seq_lens_at(0)
    sess = _session(L, w, inp, dev)
    sess.set_seq_lens(seq_cpu.to(dev))
    sess.build_stats_full()
    sess.scores.fill_(float("nan"))
    sess.select(inp.q[0].to(dev))
    torch.cuda.synchronize()
    stats_ref = oracle.page_stats(inp.k_pool, inp.page_table, seq_cpu, w.logical_page_size)
    scores_ref, _ = oracle.page_scores(inp.q[0], stats_ref, inp.page_table, seq_cpu, w.page_size)
    got = sess.scores.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    flags = w.streaming_flags()
    for b in range(w.batch):
        n_pages = (int(seq_cpu[b]) + w.page_size - 1) // w.page_size
        for hk in range(w.num_kv_heads):
            if flags[hk]:
                assert not got[b, hk].any()
            else:
                assert not got[b, hk, n_pages:].any()
                np.testing.assert_allclose(got[b, hk, :n_pages], scores_ref[b, hk, :n_pages], rtol=SCORE_REL_TOL, atol=1e-4)


def test_the_read_probe_runs_over_the_same_tables_as_the_decode_call_and_changes_nothing():
    """lserve_probe_decode_read is a measurement aid: it walks the index tables a decode call would walk and only
    reads.  A ragged batch and a selection that is three pages old."""
    L = _lib()
    dev = torch.device("cuda:0")
    w = small_decode_workload(batch=3, lengths=(1500, 300, 2100), budget_tokens=512, decode_steps=4)
    inp = make_decode_inputs(w)
    sess = _session(L, w, inp, dev)
    sess.set_seq_lens(inp.seq_lens_at(0).to(dev))
    sess.build_stats_full()
    sess.select(inp.q[0].to(dev))
    sess.set_seq_lens((inp.seq_lens_at(0) + 3 * w.page_size).clamp(max=inp.page_table.shape[1] * w.page_size).to(dev))
    before = [t.clone() for t in (sess.kv.k_pool, sess.kv.v_pool, sess.sel_pages, sess.sel_count, sess.sel_seq_len)]
    L.lserve_probe_decode_read(sess.desc, sess.kv, sess.sel_pages, sess.sel_count, sess.sel_seq_len)
    torch.cuda.synchronize()
    after = (sess.kv.k_pool, sess.kv.v_pool, sess.sel_pages, sess.sel_count, sess.sel_seq_len)
    assert all(torch.equal(a, b) for a, b in zip(before, after))
    with pytest.raises(L.LserveError):  # a selecting head needs the selection
        L.lserve_probe_decode_read(sess.desc, sess.kv, None, None, None)


# ---- KV write-back with fused statistics (Sec. 3.2, Sec. 3.5.2) ---------------------------------

def _append_case(L, w, dev, start, n_new, seed, k_pool, v_pool, stats, page_table):
    """One lserve_append_kv call next to the oracle's write-back; returns the oracle's pools."""
    g = torch.Generator().manual_seed(seed)
    total = int(sum(n_new))
    dt = k_pool.dtype
    k_new = torch.randn((max(total, 1), w.num_kv_heads, 128), generator=g).to(dt)[:total]
    v_new = torch.randn((max(total, 1), w.num_kv_heads, 128), generator=g).to(dt)[:total]
    cu = np.concatenate([[0], np.cumsum(n_new)]).astype(np.int32)
    desc = L.AttnDesc(num_q_heads=w.num_q_heads, num_kv_heads=w.num_kv_heads, streaming_flags=w.streaming_flags(),
                      head_dim=128, page_size=w.page_size, logical_page_size=w.logical_page_size, dtype=dt,
                      sink_tokens=w.sink_tokens, local_tokens=w.local_tokens)
    seq = torch.tensor([s + n for s, n in zip(start, n_new)], dtype=torch.int32, device=dev)
    kv = L.PagedKV(k_pool, v_pool, stats, page_table, seq)
    pad = torch.zeros((1, w.num_kv_heads, 128), dtype=dt)
    L.lserve_append_kv(desc, kv, torch.cat([k_new, pad]).to(dev), torch.cat([v_new, pad]).to(dev),
                       torch.from_numpy(cu).to(dev), torch.tensor(start, dtype=torch.int32, device=dev),
                       max(max(n_new), 1))
    torch.cuda.synchronize()
    return k_new, v_new, cu


@pytest.mark.parametrize("name,kw", [
    ("gqa_fp16", dict()),
    ("bf16_page32", dict(dtype="bf16", page_size=32, logical_page_size=8, sink_tokens=32, local_tokens=64,
                         budget_tokens=128)),
    ("page128_g8", dict(page_size=128, logical_page_size=16, sink_tokens=128, local_tokens=256, budget_tokens=512)),
    ("flat16", dict(page_size=16, logical_page_size=16, sink_tokens=16, local_tokens=64, budget_tokens=128)),
])
def test_append_writes_pools_bit_exact_and_keeps_statistics_equal_to_a_rebuild(name, kw):
    L = _lib()
    dev = torch.device("cuda:0")
    w = small_decode_workload(batch=3, lengths=(1, 1, 1), **kw)
    NP = w.page_size
    max_pages = 12
    g = torch.Generator().manual_seed(5)
    page_table = torch.randperm(3 * max_pages, generator=g).to(torch.int32).reshape(3, max_pages)
    dt = torch.float16 if w.dtype == "fp16" else torch.bfloat16
    num_pages = 3 * max_pages
    k_ref = torch.randn((num_pages, w.num_kv_heads, NP, 128), generator=g).to(dt)  # stale contents, as in a reused pool
    v_ref = torch.randn((num_pages, w.num_kv_heads, NP, 128), generator=g).to(dt)
    k_dev, v_dev = k_ref.to(dev), v_ref.to(dev)
    gl = NP // w.logical_page_size
    stats = torch.full((num_pages, w.num_kv_heads, gl, 2, 128), float("nan"), dtype=dt, device=dev)
    pt_dev = page_table.to(dev)
    # a chunked prefill, single-token decode appends, a ragged multi-token append and an empty one
    rounds = [(3 * NP + 5, NP - 1, 1), (1, 1, 1), (1, 1, 0), (2 * NP, 7, 3), (0, 1, NP + 1), (1, 0, 0)]
    start = [0, 0, 0]
    heads = [h for h in range(w.num_kv_heads) if h not in w.streaming_kv_heads]
    for it, n_new in enumerate(rounds):
        k_new, v_new, cu = _append_case(L, w, dev, start, list(n_new), 100 + it, k_dev, v_dev, stats, pt_dev)
        oracle.append_kv(k_new, v_new, cu, np.asarray(start, np.int32), page_table, k_ref, v_ref)
        start = [s + n for s, n in zip(start, n_new)]
        assert torch.equal(k_dev.cpu().view(torch.int16), k_ref.view(torch.int16)), (name, it)
        assert torch.equal(v_dev.cpu().view(torch.int16), v_ref.view(torch.int16)), (name, it)
        seq = np.asarray(start, np.int32)
        live = [b for b in range(3) if seq[b] > 0]
        ref = oracle.page_stats(k_ref, page_table[live], seq[live], w.logical_page_size)
        got = stats.cpu()
        for b in live:
            for lpage in range(-(-int(seq[b]) // w.logical_page_size)):
                t0 = lpage * w.logical_page_size
                phys, j = int(page_table[b, t0 // NP]), (t0 % NP) // w.logical_page_size
                for hk in heads:
                    assert torch.equal(got[phys, hk, j].float(), ref[phys, hk, j].float()), (name, it, b, lpage, hk)


def test_append_then_select_and_decode_match_the_oracle_without_a_statistics_pass():
    """Prefill write-back and per-step appends keep the statistics current, so the selector runs with no
    lserve_build_page_stats call at all."""
    L = _lib()
    dev = torch.device("cuda:0")
    w = small_decode_workload(lengths=(700, 1300), decode_steps=6, budget_tokens=512, reuse_interval=2)
    inp = make_decode_inputs(w)
    sess = _session(L, w, inp, dev)
    # the generator's pools hold every token already; fill the device pools through the entry point instead
    sess.kv.k_pool.zero_()
    sess.kv.v_pool.zero_()
    sess.stats.fill_(float("nan"))
    NP = w.page_size
    flags = w.streaming_flags()

    def append(start, n_new):
        ks, vs = [], []
        for b in range(w.batch):
            pos = torch.arange(start[b], start[b] + n_new[b])
            phys = inp.page_table[b].long()[pos // NP]
            ks.append(inp.k_pool[phys, :, pos % NP])
            vs.append(inp.v_pool[phys, :, pos % NP])
        cu = np.concatenate([[0], np.cumsum(n_new)]).astype(np.int32)
        L.lserve_append_kv(sess.desc, sess.kv, torch.cat(ks).contiguous().to(dev), torch.cat(vs).contiguous().to(dev),
                           torch.from_numpy(cu).to(dev), torch.tensor(start, dtype=torch.int32, device=dev),
                           max(n_new))

    have = [0] * w.batch
    for step in range(w.decode_steps):
        seq_cpu = inp.seq_lens_at(step)
        want = [int(x) for x in seq_cpu]
        append(have, [a - h for a, h in zip(want, have)])  # the prompt in one call, then one token per step
        have = want
        sess.set_seq_lens(seq_cpu.to(dev))
        q = inp.q[step].to(dev)
        stats_ref = _check_stats(w, inp, sess, seq_cpu)
        if step % w.reuse_interval == 0:
            sess.select(q)
            scores_ref, _ = oracle.page_scores(inp.q[step], stats_ref, inp.page_table, seq_cpu, w.page_size)
            sel_ref, cnt_ref, ssl_ref = oracle.select_pages(scores_ref, seq_cpu, w.page_size, w.budget_tokens)
            assert compare_selection(sess.sel_pages.cpu().numpy(), sess.sel_count.cpu().numpy(), sel_ref, cnt_ref,
                                     scores_ref, flags) <= 1
        out = sess.decode(q)
        ref, lse_ref = oracle.sparse_decode(inp.q[step], inp.k_pool, inp.v_pool, inp.page_table, seq_cpu,
                                            sess.sel_pages.cpu().numpy(), sess.sel_count.cpu().numpy(),
                                            sess.sel_seq_len.cpu().numpy(), flags, w.sink_tokens, w.local_tokens)
        assert_attention_close(out, ref, f"append step {step}")
        assert_lse_close(sess.lse, lse_ref, f"append step {step}")


# ---- two-way paged cache: dense heads in the main pool, streaming heads in a bounded ring (Sec. 3.2) ------

def _ring_slot(p, s, w_):
    return p if p < s else s + (p - s) % w_


def _two_way_layout(w, inp, dev, seed=9):
    """Main pool with the non-streaming heads only, an empty (NaN) bounded pool for the streaming heads and a
    scattered ring table.  Pure re-indexing of the generator's one-pool inputs."""
    dense = [h for h in range(w.num_kv_heads) if h not in w.streaming_kv_heads]
    stream = list(w.streaming_kv_heads)
    s = -(-w.sink_tokens // w.page_size)
    w_ = -(-w.local_tokens // w.page_size)
    ring = s + w_
    g = torch.Generator().manual_seed(seed)
    n_ring_pages = w.batch * ring + 3
    ring_table = torch.randperm(n_ring_pages, generator=g)[: w.batch * ring].to(torch.int32).reshape(w.batch, ring)
    k_main = inp.k_pool[:, dense].contiguous()
    v_main = inp.v_pool[:, dense].contiguous()
    shape = (n_ring_pages, len(stream), w.page_size, 128)
    k_ring = torch.full(shape, float("nan"), dtype=inp.k_pool.dtype)
    v_ring = torch.full(shape, float("nan"), dtype=inp.k_pool.dtype)
    return dense, stream, s, w_, ring_table, k_main, v_main, k_ring, v_ring


def test_two_way_cache_decode_and_append_equal_the_one_pool_path_and_the_oracle():
    """Streaming heads read from / written to a ring of s + w pages per sequence, dense heads compacted in the
    main pool: outputs must be bit-identical to the one-pool GPU path (same arithmetic, other addresses) and
    within tolerance of the oracle; the ring is filled only through lserve_append_kv."""
    L = _lib()
    dev = torch.device("cuda:0")
    w = small_decode_workload(batch=3, num_q_heads=8, num_kv_heads=4, streaming_kv_heads=(0, 2),
                              lengths=(700, 64, 1500), decode_steps=8, reuse_interval=2, budget_tokens=256,
                              sink_tokens=64, local_tokens=192)
    inp = make_decode_inputs(w)
    dense, stream, s, w_, ring_table, k_main, v_main, k_ring, v_ring = _two_way_layout(w, inp, dev)
    flags = w.streaming_flags()
    NP = w.page_size
    one = _session(L, w, inp, dev)
    from paper_2502_14866_amd.session import DecodeSession
    two = DecodeSession(torch.zeros_like(k_main).to(dev), torch.zeros_like(v_main).to(dev), inp.page_table.to(dev),
                        w.num_q_heads, flags, w.sink_tokens, w.local_tokens, w.budget_tokens,
                        logical_page_size=w.logical_page_size, reuse_interval=w.reuse_interval, want_scores=True,
                        want_lse=True, k_pool_stream=k_ring.to(dev), v_pool_stream=v_ring.to(dev),
                        ring_table=ring_table.to(dev))
    two.stats.fill_(float("nan"))

    def append(start, n_new):
        ks, vs = [], []
        for b in range(w.batch):
            pos = torch.arange(start[b], start[b] + n_new[b])
            phys = inp.page_table[b].long()[pos // NP]
            ks.append(inp.k_pool[phys, :, pos % NP])
            vs.append(inp.v_pool[phys, :, pos % NP])
        cu = np.concatenate([[0], np.cumsum(n_new)]).astype(np.int32)
        L.lserve_append_kv(two.desc, two.kv, torch.cat(ks).contiguous().to(dev), torch.cat(vs).contiguous().to(dev),
                           torch.from_numpy(cu).to(dev), torch.tensor(start, dtype=torch.int32, device=dev),
                           max(max(n_new), 1))

    have = [0] * w.batch
    for step in range(w.decode_steps):
        seq_cpu = inp.seq_lens_at(step)
        want = [int(x) for x in seq_cpu]
        if step == 0:  # the prompt in two chunks, so that local pages of the first chunk get overwritten
            mid = [x // 2 for x in want]
            append(have, mid)
            append(mid, [a - m for a, m in zip(want, mid)])
        else:
            append(have, [a - h for a, h in zip(want, have)])
        have = want
        torch.cuda.synchronize()
        # main pool: every token of the dense heads, bit for bit; ring: the pages a streaming head attends
        km, kr = two.kv.k_pool.cpu(), two.kv.k_pool_stream.cpu()
        vm, vr = two.kv.v_pool.cpu(), two.kv.v_pool_stream.cpu()
        for b in range(w.batch):
            Lb = want[b]
            P = -(-Lb // NP)
            pos = torch.arange(Lb)
            phys = inp.page_table[b].long()[pos // NP]
            assert torch.equal(km[phys, :, pos % NP].view(torch.int16), inp.k_pool[phys][:, dense][torch.arange(Lb), :, pos % NP].view(torch.int16))
            assert torch.equal(vm[phys, :, pos % NP].view(torch.int16), inp.v_pool[phys][:, dense][torch.arange(Lb), :, pos % NP].view(torch.int16))
            for p in [q for q in range(P) if q < s or q >= P - w_]:
                n_tok = min(NP, Lb - p * NP)
                src = int(inp.page_table[b, p])
                dst = int(ring_table[b, _ring_slot(p, s, w_)])
                assert torch.equal(kr[dst, :, :n_tok].view(torch.int16), inp.k_pool[src][stream][:, :n_tok].view(torch.int16)), (step, b, p)
                assert torch.equal(vr[dst, :, :n_tok].view(torch.int16), inp.v_pool[src][stream][:, :n_tok].view(torch.int16)), (step, b, p)
        seq = seq_cpu.to(dev)
        q = inp.q[step].to(dev)
        one.set_seq_lens(seq)
        two.set_seq_lens(seq)
        one.build_stats_full()
        if step % w.reuse_interval == 0:
            one.select(q)
            two.select(q)  # statistics were kept current by the appends
            assert torch.equal(one.sel_pages, two.sel_pages) and torch.equal(one.sel_count, two.sel_count)
            assert torch.equal(one.scores, two.scores)
        o1 = one.decode(q).clone()
        o2 = two.decode(q)
        assert torch.equal(o1.view(torch.int16), o2.view(torch.int16)), step
        assert torch.equal(one.lse, two.lse)
        ref, lse_ref = oracle.sparse_decode(inp.q[step], inp.k_pool, inp.v_pool, inp.page_table, seq_cpu,
                                            two.sel_pages.cpu().numpy(), two.sel_count.cpu().numpy(),
                                            two.sel_seq_len.cpu().numpy(), flags, w.sink_tokens, w.local_tokens)
        assert_attention_close(o2, ref, f"two-way step {step}")
        assert_lse_close(two.lse, lse_ref, f"two-way step {step}")
    # statistics of the dense heads in the compacted layout equal the one-pool statistics
    assert torch.equal(one.stats[:, dense].cpu().view(torch.int16)[inp.page_table[0, :5].long()],
                       two.stats.cpu().view(torch.int16)[inp.page_table[0, :5].long()])


# ---- prefill under a general block mask (Sec. 3.1, Sec. 3.4) ------------------------------------------

def _masked_prefill(L, w, pin, dev, lengths, masks, head_mask):
    from helpers import block_mask_csr
    qts, rp, cl, R = block_mask_csr(masks, lengths)
    desc = L.AttnDesc(w.num_q_heads, w.num_kv_heads, w.streaming_flags(), dtype=w.torch_dtype,
                      sink_tokens=w.sink_tokens, local_tokens=w.local_tokens)
    q, k, v = pin.q.to(dev), pin.k.to(dev), pin.v.to(dev)
    total = q.shape[0]

    def dev_i32(a, pad=4):  # 16-byte aligned device copies with a little slack
        t = torch.zeros((len(a) + pad,), dtype=torch.int32, device=dev)
        t[:len(a)] = torch.as_tensor(np.asarray(a, dtype=np.int32))
        return t[:len(a)]

    mask = L.BlockMask(dev_i32(head_mask), dev_i32(qts), dev_i32(rp), dev_i32(cl) if len(cl) else None,
                       len(masks), R)
    nbytes = L.lserve_masked_prefill_workspace_bytes(desc, len(lengths), total, max(lengths), len(masks), len(cl))
    assert nbytes >= L.lserve_workspace_bytes(L.LSERVE_CALL_SPARSE_PREFILL, desc, len(lengths), 0, 0, total)
    ws = torch.empty((nbytes,), dtype=torch.uint8, device=dev)
    out = torch.full_like(q, float("nan"))
    lse = torch.full((w.num_q_heads, total), float("nan"), dtype=torch.float32, device=dev)
    L.lserve_sparse_prefill_masked(desc, mask, q, k, v, pin.cu_seqlens.to(dev), max(lengths), out, lse, ws)
    torch.cuda.synchronize()
    tok = np.repeat(np.arange(total, dtype=np.int32), w.num_q_heads)
    head = np.tile(np.arange(w.num_q_heads, dtype=np.int32), total)
    ref, lse_ref = oracle.block_mask_prefill_rows(pin.q, pin.k, pin.v, pin.cu_seqlens, w.streaming_flags(), 64,
                                                  w.sink_tokens, w.local_tokens, head_mask, qts, rp, cl, R, tok, head)
    return out, lse, ref.reshape(total, w.num_q_heads, -1), lse_ref.reshape(total, w.num_q_heads)


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
@pytest.mark.parametrize("lengths", [(130,), (700, 64, 1000), (2049,)])
def test_masked_prefill_matches_oracle_on_every_row(dtype, lengths):
    """Random block masks (diagonal always kept), a vertical-and-slash style mask, the analytic fallback and
    a mask whose first rows keep nothing, on different heads of one call; every row against the oracle."""
    L = _lib()
    dev = torch.device("cuda:0")
    w = Workload(name="pm", batch=len(lengths), num_q_heads=8, num_kv_heads=2, dtype=dtype, streaming_kv_heads=(0,),
                 sink_tokens=64, local_tokens=192, seed=23)
    pin = make_prefill_inputs(w, lengths=lengths)
    rng = np.random.default_rng(7)
    kept = {}

    def rnd(b, i):
        if (b, i) not in kept:
            kept[(b, i)] = [j for j in range(i) if rng.random() < 0.3] + [i]
        return kept[(b, i)]

    vslash = lambda b, i: [j for j in range(i + 1) if j % 5 == 0 or i - j < 2]   # vertical lines and a slash
    holes = lambda b, i: [] if i < 2 else [j for j in range(i + 1) if j % 2 == 1]  # tile rows 0, 1 keep nothing; no diagonal on even rows
    # heads 0-3 share KV head 0 (flagged streaming), heads 4-7 KV head 1 (dense)
    head_mask = [0, 1, -1, 2, 0, -1, 1, 2]
    out, lse, ref, lse_ref = _masked_prefill(L, w, pin, dev, lengths, [rnd, vslash, holes], head_mask)
    empty = ~np.isfinite(lse_ref)
    assert empty.any()
    got = out.float().cpu().numpy()
    assert not np.isnan(got).any()
    assert (got[empty] == 0).all() and np.isneginf(lse.t().cpu().numpy()[empty]).all()
    assert_attention_close(out, ref, f"masked prefill {dtype} {lengths}")
    lse_got = lse.t().contiguous().cpu().numpy()
    np.testing.assert_allclose(lse_got[~empty], lse_ref[~empty], atol=LSE_TOL_PREFILL[dtype], rtol=0)


def test_masked_prefill_with_analytic_tiles_is_bit_identical_to_the_unmasked_call():
    L = _lib()
    dev = torch.device("cuda:0")
    lengths = (900, 333)
    w = Workload(name="pm2", batch=2, num_q_heads=4, num_kv_heads=2, dtype="fp16", streaming_kv_heads=(0,),
                 sink_tokens=64, local_tokens=192, seed=29)
    pin = make_prefill_inputs(w, lengths=lengths)
    s, wl = 1, 3
    lam = lambda b, i: [j for j in range(i + 1) if j < s or j > i - wl]
    lower = lambda b, i: range(i + 1)
    out_m, lse_m, _, _ = _masked_prefill(L, w, pin, dev, lengths, [lam, lower], [0, 0, 1, 1])
    out_u, lse_u = _prefill(L, w, pin, dev)
    assert torch.equal(out_m.view(torch.int16), out_u.view(torch.int16))
    assert torch.equal(lse_m, lse_u)


# ---- chunked prefill over the paged cache -----------------------------------------------------------------

@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
@pytest.mark.parametrize("case", [
    dict(lengths=(700, 64, 1000), chunks=(700, 64, 1000)),   # the whole prompt: must equal the contiguous call
    dict(lengths=(700, 64, 1000), chunks=(257, 1, 0)),       # chunk starts off every boundary; a one-token chunk; an idle sequence
    dict(lengths=(2049,), chunks=(513,)),
    dict(lengths=(300, 1300), chunks=(64, 256)),             # chunks aligned to tiles / blocks
])
def test_paged_chunk_prefill_matches_oracle_on_every_row(dtype, case):
    L = _lib()
    dev = torch.device("cuda:0")
    lengths, chunks = case["lengths"], case["chunks"]
    B_ = len(lengths)
    w = Workload(name="pp", batch=B_, num_q_heads=4, num_kv_heads=2, dtype=dtype, streaming_kv_heads=(0,),
                 sink_tokens=64, local_tokens=192, seed=31)
    pin = make_prefill_inputs(w, lengths=lengths)
    NP = 64
    max_pages = max(-(-l // NP) for l in lengths) + 1
    g = torch.Generator().manual_seed(17)
    page_table = torch.randperm(B_ * max_pages + 2, generator=g)[:B_ * max_pages].to(torch.int32).reshape(B_, max_pages)
    k_pool = torch.full((B_ * max_pages + 2, 2, NP, 128), float("nan"), dtype=pin.k.dtype)  # unused slots poison the result
    v_pool = torch.full_like(k_pool, float("nan"))
    scatter_prefill_kv_to_pages(pin.k, pin.v, pin.cu_seqlens, k_pool, v_pool, page_table)
    qs = []
    for b in range(B_):
        a = int(pin.cu_seqlens[b]) + lengths[b] - chunks[b]
        qs.append(pin.q[a:a + chunks[b]])
    qc = torch.cat(qs).contiguous()
    total_new = qc.shape[0]
    cu_q = np.concatenate([[0], np.cumsum(chunks)]).astype(np.int32)
    desc = L.AttnDesc(w.num_q_heads, w.num_kv_heads, w.streaming_flags(), dtype=w.torch_dtype,
                      sink_tokens=w.sink_tokens, local_tokens=w.local_tokens)
    pad4 = lambda a: torch.cat([torch.as_tensor(a, dtype=torch.int32), torch.zeros(4, dtype=torch.int32)]).to(dev)[:len(a)]
    kv = L.PagedKV(k_pool.to(dev), v_pool.to(dev), None, page_table.to(dev), pad4(list(lengths)))
    ws = torch.empty((L.lserve_paged_prefill_workspace_bytes(desc, B_, max_pages),), dtype=torch.uint8, device=dev)
    qd = torch.cat([qc, torch.zeros((1, 4, 128), dtype=qc.dtype)]).to(dev)[:total_new]
    out = torch.full((total_new, 4, 128), float("nan"), dtype=qc.dtype, device=dev)
    lse = torch.full((4, total_new), float("nan"), dtype=torch.float32, device=dev)
    L.lserve_sparse_prefill_paged(desc, kv, qd, pad4(cu_q), max(chunks), max(lengths), out, lse, ws)
    torch.cuda.synchronize()
    tok = np.repeat(np.arange(total_new, dtype=np.int32), 4)
    head = np.tile(np.arange(4, dtype=np.int32), total_new)
    # the oracle reads the same pools; NaN in unused slots must not reach it either
    ref, lse_ref = oracle.paged_prefill_rows(qc, k_pool, v_pool, page_table, np.asarray(lengths, np.int32), cu_q,
                                             w.streaming_flags(), w.sink_tokens, w.local_tokens, tok, head)
    assert_attention_close(out, ref.reshape(total_new, 4, -1), f"paged prefill {dtype} {case}")
    assert_lse_close(lse.t().contiguous(), lse_ref.reshape(total_new, 4), "paged prefill lse", LSE_TOL_PREFILL[dtype])
    if chunks == lengths:
        out_c, lse_c = _prefill(L, w, pin, dev)
        assert torch.equal(out.view(torch.int16), out_c.view(torch.int16))
        assert torch.equal(lse, lse_c)


@pytest.mark.parametrize("heads", [(6, 3, (1,)), (16, 16, (0, 5, 6, 7, 8, 15)), (24, 3, ()), (5, 5, (0, 1, 2, 3, 4))])
def test_prefill_head_layouts_that_do_not_divide_the_xcd_count(heads):
    """Head counts for which the XCD-aware work order falls back to plain round-robin, all-dense and all-streaming."""
    L = _lib()
    dev = torch.device("cuda:0")
    H, Hkv, streaming = heads
    lengths = (321, 640)
    w = Workload(name="ph", batch=2, num_q_heads=H, num_kv_heads=Hkv, dtype="fp16", streaming_kv_heads=streaming,
                 sink_tokens=64, local_tokens=128, seed=37)
    pin = make_prefill_inputs(w, lengths=lengths)
    out, lse = _prefill(L, w, pin, dev)
    total = sum(lengths)
    tok = np.repeat(np.arange(total, dtype=np.int32), H)
    head = np.tile(np.arange(H, dtype=np.int32), total)
    ref, lse_ref = _oracle_rows(w, pin, tok, head)
    assert_attention_close(out, ref.reshape(total, H, -1), f"prefill heads {heads}")
    assert_lse_close(lse.t().contiguous(), lse_ref.reshape(total, H), "prefill lse", LSE_TOL_PREFILL["fp16"])

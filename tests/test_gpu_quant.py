"""Quantised KV pages (Sec. 3.2, Sec. 3.5): the write-back's bytes against the oracle's quantiser, bit for
bit, and decode over those pages against the oracle's decode over the values the bytes stand for."""
import numpy as np
import pytest
import torch

import oracle
from workloads import make_decode_inputs

from helpers import small_decode_workload
from parity import assert_attention_close, assert_lse_close, compare_selection

pytestmark = pytest.mark.gpu

def slab_bytes(bits):
    """Bytes of one (page, head): 64 rows of 128 codes, then 64 (scale, zero) pairs of fp16."""
    return 64 * 128 * bits // 8 + 256


def _pack_rows(codes: np.ndarray, bits: int) -> np.ndarray:
    """[n, 128] codes -> [n, 128 * bits / 8] bytes in the page's row format (layout only)."""
    if bits == 8:
        return codes
    c = codes.reshape(-1, 16, 2, 4)  # word g, half (channels 8 g + 0..3 / 8 g + 4..7), byte j
    return (c[:, :, 0, :] | (c[:, :, 1, :] << 4)).reshape(-1, 64).astype(np.uint8)


def _unpack_rows(raw: np.ndarray, bits: int) -> np.ndarray:
    """[..., 128 * bits / 8] bytes -> [..., 128] codes."""
    if bits == 8:
        return raw
    w = raw.reshape(raw.shape[:-1] + (16, 4))
    return np.stack([w & 0xf, w >> 4], axis=-2).reshape(raw.shape[:-1] + (128,))


def _lib():
    import paper_2502_14866_amd as L

    L.load_library()
    return L


def _write_rows(pool_q: torch.Tensor, phys, hk, slot, x_rows: torch.Tensor, bits: int):
    """Oracle-quantised rows x_rows [n, 128] into slots (phys[i], hk, slot[i]) of a CPU byte pool."""
    codes, scale, zero = oracle.quantize_kv(x_rows, bits)
    rows = _pack_rows(codes, bits)
    rb, tail = 128 * bits // 8, 64 * 128 * bits // 8
    sz = np.stack([scale, zero], axis=-1).view(np.uint8).reshape(-1, 4)
    for i in range(x_rows.shape[0]):
        slab = pool_q[int(phys[i]), hk]
        slab[int(slot[i]) * rb:(int(slot[i]) + 1) * rb] = torch.from_numpy(rows[i])
        slab[tail + 4 * int(slot[i]):tail + 4 * int(slot[i]) + 4] = torch.from_numpy(sz[i])


def _values(pool_q: torch.Tensor, bits: int) -> np.ndarray:
    """[pages, heads, 64, 128] float64 values a CPU byte pool stands for (unwritten slots: whatever they hold)."""
    raw = pool_q.numpy()
    tail = 64 * 128 * bits // 8
    codes = _unpack_rows(raw[..., :tail].reshape(raw.shape[0], raw.shape[1], 64, 128 * bits // 8), bits)
    sz = np.ascontiguousarray(raw[..., tail:]).view(np.float16).reshape(raw.shape[0], raw.shape[1], 64, 2)
    with np.errstate(invalid="ignore", over="ignore"):
        return oracle.dequantize_q8(codes, sz[..., 0], sz[..., 1])


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
def test_quantising_append_writes_the_oracles_bytes_and_nothing_else(dtype, bits):
    L = _lib()
    SLAB = slab_bytes(bits)
    dev = torch.device("cuda:0")
    w = small_decode_workload(batch=3, lengths=(1, 1, 1), dtype=dtype)
    dt = torch.float16 if dtype == "fp16" else torch.bfloat16
    max_pages, num_pages = 8, 24
    g = torch.Generator().manual_seed(5)
    page_table = torch.randperm(num_pages, generator=g).to(torch.int32).reshape(3, max_pages)
    k_ref = torch.randint(0, 256, (num_pages, w.num_kv_heads, SLAB), generator=g, dtype=torch.uint8)  # a reused pool
    v_ref = torch.randint(0, 256, (num_pages, w.num_kv_heads, SLAB), generator=g, dtype=torch.uint8)
    k16 = torch.zeros((num_pages, w.num_kv_heads, 64, 128), dtype=dt)  # the keys themselves, for the statistics
    k_dev, v_dev = k_ref.to(dev), v_ref.to(dev)
    stats = torch.full((num_pages, w.num_kv_heads, 4, 2, 128), float("nan"), dtype=dt, device=dev)
    desc = L.AttnDesc(num_q_heads=w.num_q_heads, num_kv_heads=w.num_kv_heads, streaming_flags=w.streaming_flags(),
                      dtype=dt, sink_tokens=w.sink_tokens, local_tokens=w.local_tokens)
    pt_dev = page_table.to(dev)
    rounds = [(3 * 64 + 5, 63, 1), (1, 1, 1), (1, 1, 0), (128, 7, 3), (0, 1, 65), (1, 0, 0)]
    start = [0, 0, 0]
    heads = [h for h in range(w.num_kv_heads) if h not in w.streaming_kv_heads]
    for it, n_new in enumerate(rounds):
        gg = torch.Generator().manual_seed(100 + it)
        total = sum(n_new)
        # rows of different spread and offset, one constant row and one with a single outlier
        k_new = (torch.randn((total, w.num_kv_heads, 128), generator=gg) * (4 * torch.rand((total, w.num_kv_heads, 1), generator=gg))
                 + torch.randn((total, w.num_kv_heads, 1), generator=gg)).to(dt)
        v_new = torch.randn((total, w.num_kv_heads, 128), generator=gg).to(dt)
        k_new[0, 0] = 0.375
        v_new[0, 1, 5] = 300.0
        cu = np.concatenate([[0], np.cumsum(n_new)]).astype(np.int32)
        seq = torch.tensor([s + n for s, n in zip(start, n_new)], dtype=torch.int32, device=dev)
        kv = L.PagedKV(k_dev, v_dev, stats, pt_dev, seq, kv_bits=bits)
        pad = torch.zeros((1, w.num_kv_heads, 128), dtype=dt)
        L.lserve_append_kv(desc, kv, torch.cat([k_new, pad]).to(dev), torch.cat([v_new, pad]).to(dev),
                           torch.from_numpy(cu).to(dev), torch.tensor(start, dtype=torch.int32, device=dev),
                           max(max(n_new), 1))
        torch.cuda.synchronize()
        for b in range(3):
            pos = np.arange(start[b], start[b] + n_new[b])
            phys = page_table[b].numpy()[pos // 64]
            for hk in range(w.num_kv_heads):
                _write_rows(k_ref, phys, hk, pos % 64, k_new[cu[b]:cu[b + 1], hk], bits)
                _write_rows(v_ref, phys, hk, pos % 64, v_new[cu[b]:cu[b + 1], hk], bits)
                k16[torch.from_numpy(phys).long(), hk, torch.from_numpy(pos % 64).long()] = k_new[cu[b]:cu[b + 1], hk]
        start = [s + n for s, n in zip(start, n_new)]
        assert torch.equal(k_dev.cpu(), k_ref), (dtype, bits, it)
        assert torch.equal(v_dev.cpu(), v_ref), (dtype, bits, it)
        seq_np = np.asarray(start, np.int32)
        live = [b for b in range(3) if seq_np[b] > 0]
        ref = oracle.page_stats(k16, page_table[live], seq_np[live], w.logical_page_size)
        got = stats.cpu()
        for b in live:
            for lpage in range(-(-int(seq_np[b]) // w.logical_page_size)):
                t0 = lpage * w.logical_page_size
                phys, j = int(page_table[b, t0 // 64]), (t0 % 64) // w.logical_page_size
                for hk in heads:
                    assert torch.equal(got[phys, hk, j].float(), ref[phys, hk, j].float()), (dtype, it, b, lpage, hk)


QUANT_WORKLOADS = {
    "tiny_gqa": dict(),
    "ragged_tail": dict(lengths=(1, 63), decode_steps=3),
    "mha": dict(num_q_heads=4, num_kv_heads=4, streaming_kv_heads=(1, 3), lengths=(900, 130, 2049), batch=3),
    "gqa8_bf16": dict(num_q_heads=16, num_kv_heads=2, dtype="bf16", streaming_kv_heads=(1,), lengths=(4100, 700),
                      budget_tokens=1024),
    "group3_all_dense": dict(num_q_heads=6, num_kv_heads=2, streaming_kv_heads=(), lengths=(1500, 2600), budget_tokens=512),
    "group5_bf16": dict(num_q_heads=10, num_kv_heads=2, dtype="bf16", lengths=(333, 1000)),
}


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("name", list(QUANT_WORKLOADS))
def test_decode_loop_over_quantised_pages_matches_the_oracle(name, bits):
    """Pages are filled through the quantising write-back (the prompt in one call, then a token per step) into
    pools that start as 0xff bytes (NaN scales in every unused slot); statistics, selection and the decode
    output are compared at every step, the output against the oracle's decode over code * scale + zero."""
    from paper_2502_14866_amd.session import DecodeSession

    L = _lib()
    dev = torch.device("cuda:0")
    w = small_decode_workload(**dict(dict(decode_steps=4, reuse_interval=2), **QUANT_WORKLOADS[name]))
    inp = make_decode_inputs(w)
    dt = inp.k_pool.dtype
    num_pages = inp.k_pool.shape[0]
    k_q = torch.full((num_pages, w.num_kv_heads, slab_bytes(bits)), 0xff, dtype=torch.uint8)
    v_q = k_q.clone()
    sess = DecodeSession(k_q.to(dev), v_q.to(dev), inp.page_table.to(dev), w.num_q_heads, w.streaming_flags(),
                         w.sink_tokens, w.local_tokens, w.budget_tokens, logical_page_size=w.logical_page_size,
                         reuse_interval=w.reuse_interval, want_scores=True, want_lse=True, kv_bits=bits, dtype=dt)
    sess.stats.fill_(float("nan"))
    flags = w.streaming_flags()
    have = [0] * w.batch
    near_ties = 0
    for step in range(w.decode_steps):
        seq_cpu = inp.seq_lens_at(step)
        want = [int(x) for x in seq_cpu]
        ks, vs = [], []
        for b in range(w.batch):
            pos = torch.arange(have[b], want[b])
            phys = inp.page_table[b].long()[pos // 64]
            kb, vb = inp.k_pool[phys, :, pos % 64], inp.v_pool[phys, :, pos % 64]  # [n, Hkv, 128]
            ks.append(kb)
            vs.append(vb)
            for hk in range(w.num_kv_heads):
                _write_rows(k_q, phys, hk, pos % 64, kb[:, hk], bits)
                _write_rows(v_q, phys, hk, pos % 64, vb[:, hk], bits)
        n_new = [a - h for a, h in zip(want, have)]
        cu = np.concatenate([[0], np.cumsum(n_new)]).astype(np.int32)
        sess.append(torch.cat(ks).contiguous().to(dev), torch.cat(vs).contiguous().to(dev), torch.from_numpy(cu).to(dev),
                    torch.tensor(have, dtype=torch.int32, device=dev), max(n_new))
        have = want
        assert torch.equal(sess.kv.k_pool.cpu(), k_q), (name, bits, step)
        assert torch.equal(sess.kv.v_pool.cpu(), v_q), (name, bits, step)
        sess.set_seq_lens(seq_cpu.to(dev))
        q = inp.q[step].to(dev)
        stats_ref = oracle.page_stats(inp.k_pool, inp.page_table, seq_cpu, w.logical_page_size)
        if step % w.reuse_interval == 0:
            sess.select(q)
            scores_ref, _ = oracle.page_scores(inp.q[step], stats_ref, inp.page_table, seq_cpu, w.page_size)
            sel_ref, cnt_ref, ssl_ref = oracle.select_pages(scores_ref, seq_cpu, w.page_size, w.budget_tokens)
            near_ties += compare_selection(sess.sel_pages.cpu().numpy(), sess.sel_count.cpu().numpy(), sel_ref, cnt_ref,
                                           scores_ref, flags)
        out = sess.decode(q)
        ref, lse_ref = oracle.sparse_decode_values(inp.q[step], _values(k_q, bits), _values(v_q, bits), inp.page_table, seq_cpu,
                                                   sess.sel_pages.cpu().numpy(), sess.sel_count.cpu().numpy(),
                                                   sess.sel_seq_len.cpu().numpy(), flags, w.sink_tokens, w.local_tokens)
        assert_attention_close(out, ref, f"{name} {bits}-bit step {step}")
        assert_lse_close(sess.lse, lse_ref, f"{name} {bits}-bit step {step}")
    assert near_ties <= 1


@pytest.mark.parametrize("bits", [8, 4])
def test_two_way_cache_of_quantised_pages_equals_the_one_pool_path_bit_for_bit(bits):
    """Streaming heads in a bounded ring of quantised pages, dense heads compacted in the main pool (Sec. 3.2):
    the same bytes land at the other addresses and selection, outputs and log-sum-exp are identical to the
    one-pool quantised path, which the test above holds against the oracle."""
    from paper_2502_14866_amd.session import DecodeSession

    L = _lib()
    SLAB, rb, tail = slab_bytes(bits), 128 * bits // 8, 64 * 128 * bits // 8
    dev = torch.device("cuda:0")
    w = small_decode_workload(batch=3, num_q_heads=8, num_kv_heads=4, streaming_kv_heads=(0, 2),
                              lengths=(700, 64, 1500), decode_steps=6, reuse_interval=2, budget_tokens=256,
                              sink_tokens=64, local_tokens=192)
    inp = make_decode_inputs(w)
    dt = inp.k_pool.dtype
    flags = w.streaming_flags()
    dense = [h for h in range(w.num_kv_heads) if h not in w.streaming_kv_heads]
    stream = list(w.streaming_kv_heads)
    s, w_ = -(-w.sink_tokens // 64), -(-w.local_tokens // 64)
    ring = s + w_
    g = torch.Generator().manual_seed(9)
    n_ring_pages = w.batch * ring + 3
    ring_table = torch.randperm(n_ring_pages, generator=g)[: w.batch * ring].to(torch.int32).reshape(w.batch, ring)
    num_pages = inp.k_pool.shape[0]

    def session(heads, **kw):
        return DecodeSession(torch.zeros((num_pages, heads, SLAB), dtype=torch.uint8, device=dev),
                             torch.zeros((num_pages, heads, SLAB), dtype=torch.uint8, device=dev), inp.page_table.to(dev),
                             w.num_q_heads, flags, w.sink_tokens, w.local_tokens, w.budget_tokens,
                             logical_page_size=w.logical_page_size, reuse_interval=w.reuse_interval, want_scores=True,
                             want_lse=True, kv_bits=bits, dtype=dt, **kw)

    one = session(w.num_kv_heads)
    two = session(len(dense), k_pool_stream=torch.full((n_ring_pages, len(stream), SLAB), 0xff, dtype=torch.uint8, device=dev),
                  v_pool_stream=torch.full((n_ring_pages, len(stream), SLAB), 0xff, dtype=torch.uint8, device=dev),
                  ring_table=ring_table.to(dev))

    def append(start, n_new):
        ks, vs = [], []
        for b in range(w.batch):
            pos = torch.arange(start[b], start[b] + n_new[b])
            phys = inp.page_table[b].long()[pos // 64]
            ks.append(inp.k_pool[phys, :, pos % 64])
            vs.append(inp.v_pool[phys, :, pos % 64])
        cu = torch.from_numpy(np.concatenate([[0], np.cumsum(n_new)]).astype(np.int32)).to(dev)
        k_new, v_new = torch.cat(ks).contiguous().to(dev), torch.cat(vs).contiguous().to(dev)
        st = torch.tensor(start, dtype=torch.int32, device=dev)
        for sess in (one, two):
            sess.append(k_new, v_new, cu, st, max(max(n_new), 1))

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
        k1, v1 = one.kv.k_pool.cpu(), one.kv.v_pool.cpu()
        assert torch.equal(two.kv.k_pool.cpu(), k1[:, dense]) and torch.equal(two.kv.v_pool.cpu(), v1[:, dense])
        kr, vr = two.kv.k_pool_stream.cpu(), two.kv.v_pool_stream.cpu()
        for b in range(w.batch):
            P = -(-want[b] // 64)
            for p in [x for x in range(P) if x < s or x >= P - w_]:
                n_tok = min(64, want[b] - p * 64)
                src = int(inp.page_table[b, p])
                dst = int(ring_table[b, p if p < s else s + (p - s) % w_])
                for pool_r, pool_1 in ((kr, k1), (vr, v1)):
                    assert torch.equal(pool_r[dst, :, :rb * n_tok], pool_1[src][stream][:, :rb * n_tok]), (step, b, p)
                    assert torch.equal(pool_r[dst, :, tail:tail + 4 * n_tok], pool_1[src][stream][:, tail:tail + 4 * n_tok])
        seq = seq_cpu.to(dev)
        q = inp.q[step].to(dev)
        one.set_seq_lens(seq)
        two.set_seq_lens(seq)
        if step % w.reuse_interval == 0:
            one.select(q)
            two.select(q)
            assert torch.equal(one.sel_pages, two.sel_pages) and torch.equal(one.sel_count, two.sel_count)
            assert torch.equal(one.scores, two.scores)
        o1 = one.decode(q).clone()
        o2 = two.decode(q)
        assert torch.equal(o1.view(torch.int16), o2.view(torch.int16)), step
        assert torch.equal(one.lse, two.lse)


@pytest.mark.parametrize("bits", [8, 4])
def test_cfg2_full_size_quantised_cache_sampled_sequences(bits):
    """The benchmark's decode shape (16 x 32768 tokens, 32 / 8 heads): every prompt is written through the
    quantising write-back in one call, the selector runs on the statistics that call left, and decode runs over
    the quantised pages; three sequences are checked against the oracle (their pages gathered into a small pool:
    bytes bit for bit against the oracle's quantiser, selection, outputs)."""
    from paper_2502_14866_amd.session import DecodeSession
    from workloads import get_config

    from helpers import sub_problem

    L = _lib()
    dev = torch.device("cuda:0")
    w = get_config("cfg2")
    inp = make_decode_inputs(w, device=dev)
    B, Hkv = w.batch, w.num_kv_heads
    num_pages = inp.k_pool.shape[0]
    SLAB = slab_bytes(bits)
    sess = DecodeSession(torch.zeros((num_pages, Hkv, SLAB), dtype=torch.uint8, device=dev),
                         torch.zeros((num_pages, Hkv, SLAB), dtype=torch.uint8, device=dev), inp.page_table, w.num_q_heads,
                         w.streaming_flags(), w.sink_tokens, w.local_tokens, w.budget_tokens,
                         logical_page_size=w.logical_page_size, reuse_interval=w.reuse_interval, want_scores=True,
                         kv_bits=bits, dtype=inp.k_pool.dtype)
    lens = inp.prompt_lens.to(dev).to(torch.int32)
    pad = (B + 4) // 4 * 4
    cu = torch.zeros((pad,), dtype=torch.int32, device=dev)
    cu[1:B + 1] = torch.cumsum(lens, 0)
    seq = torch.zeros((pad,), dtype=torch.int32, device=dev)
    seq[:B] = lens
    ks, vs = [], []
    for b in range(B):
        pos = torch.arange(int(inp.prompt_lens[b]), device=dev)
        phys = inp.page_table[b].long()[pos // 64]
        ks.append(inp.k_pool[phys, :, pos % 64])
        vs.append(inp.v_pool[phys, :, pos % 64])
    sess.set_seq_lens(seq[:B])
    sess.append(torch.cat(ks).contiguous(), torch.cat(vs).contiguous(), cu, torch.zeros((pad,), dtype=torch.int32, device=dev),
                int(inp.prompt_lens.max()))
    del ks, vs
    q = inp.q[0]
    sess.select(q)
    out = sess.decode(q)
    torch.cuda.synchronize()

    seqs = (0, 7, 15)
    sub = sub_problem(inp, seqs)  # 16-bit pages of the sampled sequences, renumbered
    sw = sub.workload
    seq_cpu = sub.prompt_lens.to(torch.int32)
    flags = w.streaming_flags()
    # the same pages of the quantised pools, in the sub-problem's numbering
    rows = []
    for b in seqs:
        n_pages = (int(inp.prompt_lens[b]) + max(1, w.decode_steps) + 63) // 64
        rows.append(inp.page_table[b, :n_pages].long())
    idx = torch.cat(rows)
    k_q, v_q = sess.kv.k_pool[idx].cpu(), sess.kv.v_pool[idx].cpu()
    # bytes: every token of the three prompts against the oracle's quantiser
    for i, b in enumerate(seqs):
        Lb = int(seq_cpu[i])
        P = -(-Lb // 64)
        pages = sub.page_table[i, :P].long()
        for pool16, pool_q in ((sub.k_pool, k_q), (sub.v_pool, v_q)):
            x = pool16[pages].permute(1, 0, 2, 3).reshape(Hkv, P * 64, 128)[:, :Lb]  # [Hkv, Lb, 128]
            codes, scale, zero = oracle.quantize_kv(x, bits)
            got = pool_q[pages].numpy()  # [P, Hkv, SLAB]
            tail = 64 * 128 * bits // 8
            got_codes = _unpack_rows(got[..., :tail].reshape(P, Hkv, 64, 128 * bits // 8), bits)
            got_codes = np.transpose(got_codes, (1, 0, 2, 3)).reshape(Hkv, P * 64, 128)[:, :Lb]
            assert np.array_equal(got_codes, codes), (bits, b)
            sz = np.ascontiguousarray(got[..., tail:]).view(np.float16).reshape(P, Hkv, 64, 2)
            sz = np.transpose(sz, (1, 0, 2, 3)).reshape(Hkv, P * 64, 2)[:, :Lb]
            assert np.array_equal(sz[..., 0].view(np.uint16), scale.view(np.uint16)), (bits, b)
            assert np.array_equal(sz[..., 1].view(np.uint16), zero.view(np.uint16)), (bits, b)
    # selection from the statistics the write-back left
    stats = oracle.page_stats(sub.k_pool, sub.page_table, seq_cpu, sw.logical_page_size)
    scores, _ = oracle.page_scores(sub.q[0], stats, sub.page_table, seq_cpu, sw.page_size)
    sel_ref, cnt_ref, ssl_ref = oracle.select_pages(scores, seq_cpu, sw.page_size, sw.budget_tokens)
    sel_gpu = sess.sel_pages.cpu().numpy()[list(seqs)]
    cnt_gpu = sess.sel_count.cpu().numpy()[list(seqs)]
    ssl_gpu = sess.sel_seq_len.cpu().numpy()[list(seqs)]
    assert compare_selection(sel_gpu, cnt_gpu, sel_ref, cnt_ref, scores, flags) <= 1
    assert np.array_equal(ssl_gpu, ssl_ref)
    # decode over the values the bytes stand for
    ref, _ = oracle.sparse_decode_values(sub.q[0], _values(k_q, bits), _values(v_q, bits), sub.page_table, seq_cpu,
                                         sel_gpu, cnt_gpu, ssl_gpu, flags, w.sink_tokens, w.local_tokens)
    assert_attention_close(out[list(seqs)], ref, f"cfg2 {bits}-bit pages")

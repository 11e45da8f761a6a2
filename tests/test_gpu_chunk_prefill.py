"""lserve_sparse_prefill_chunk: chunked prefill in the order of the prefill flow (attention over the chunk with the
history in the cache, then write-back), every row against the oracle, over one pool and over the two-way cache."""
import numpy as np
import pytest
import torch

import oracle
from workloads import Workload, make_prefill_inputs

from parity import LSE_TOL_PREFILL, assert_attention_close, assert_lse_close

pytestmark = pytest.mark.gpu

NP = 64


def _lib():
    import paper_2502_14866_amd as L

    L.load_library()
    return L


def _pad4(a, dev):
    return torch.cat([torch.as_tensor(a, dtype=torch.int32), torch.zeros(4, dtype=torch.int32)]).to(dev)[:len(a)]


def _split(pin, lengths, hist):
    """Chunk tensors (q, k, v of the tokens at or past hist[b]) and the rows of `pin` they are."""
    qs, ks, vs, idx = [], [], [], []
    for b, (L_b, S) in enumerate(zip(lengths, hist)):
        a = int(pin.cu_seqlens[b])
        qs.append(pin.q[a + S:a + L_b])
        ks.append(pin.k[a + S:a + L_b])
        vs.append(pin.v[a + S:a + L_b])
        idx.extend(range(a + S, a + L_b))
    return torch.cat(qs).contiguous(), torch.cat(ks).contiguous(), torch.cat(vs).contiguous(), idx


def _history_values(pin, lengths, hist, dropped=None):
    """float64 [B, max hist, Hkv, D] of the history keys / values; `dropped(b, hk, u)` positions become NaN."""
    B, Hkv, D = len(lengths), pin.k.shape[1], pin.k.shape[2]
    stride = max(max(hist), 1)
    kh = np.full((B, stride, Hkv, D), np.nan)
    vh = np.full_like(kh, np.nan)
    for b, S in enumerate(hist):
        a = int(pin.cu_seqlens[b])
        kh[b, :S] = pin.k[a:a + S].to(torch.float64).numpy()
        vh[b, :S] = pin.v[a:a + S].to(torch.float64).numpy()
        if dropped is not None:
            for hk in range(Hkv):
                for u in range(S):
                    if dropped(b, hk, u):
                        kh[b, u, hk] = np.nan
                        vh[b, u, hk] = np.nan
    return kh, vh


def _check_chunk(L, w, pin, lengths, hist, kv, dev, what, dropped=None):
    qc, kc, vc, idx = _split(pin, lengths, hist)
    chunks = [L_b - S for L_b, S in zip(lengths, hist)]
    total_new = qc.shape[0]
    cu_new = np.concatenate([[0], np.cumsum(chunks)]).astype(np.int32)
    desc = L.AttnDesc(w.num_q_heads, w.num_kv_heads, w.streaming_flags(), dtype=w.torch_dtype,
                      sink_tokens=w.sink_tokens, local_tokens=w.local_tokens)
    H = w.num_q_heads
    pad_rows = lambda t: torch.cat([t, torch.zeros((1,) + tuple(t.shape[1:]), dtype=t.dtype)]).to(dev)[:t.shape[0]]
    out = torch.full((total_new, H, 128), float("nan"), dtype=qc.dtype, device=dev)
    lse = torch.full((H, total_new), float("nan"), dtype=torch.float32, device=dev)
    kv.seq_lens = _pad4(list(hist), dev)
    L.lserve_sparse_prefill_chunk(desc, kv, pad_rows(qc), pad_rows(kc), pad_rows(vc), _pad4(cu_new, dev), max(chunks), out,
                                  lse)
    torch.cuda.synchronize()
    tok = np.repeat(np.arange(total_new, dtype=np.int32), H)
    head = np.tile(np.arange(H, dtype=np.int32), total_new)
    kh, vh = _history_values(pin, lengths, hist, dropped)
    ref, lse_ref = oracle.chunk_prefill_rows(qc, kc, vc, kh, vh, np.asarray(hist, np.int32), cu_new, w.streaming_flags(),
                                             NP, w.sink_tokens, w.local_tokens, tok, head)
    assert np.isfinite(ref).all()
    assert_attention_close(out, ref.reshape(total_new, H, -1), what)
    assert_lse_close(lse.t().contiguous(), lse_ref.reshape(total_new, H), what + " lse", LSE_TOL_PREFILL[w.dtype])
    return desc, out, lse, (qc, kc, vc, cu_new, chunks)


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
@pytest.mark.parametrize("case", [
    dict(lengths=(700, 64, 1000), hist=(0, 0, 0)),          # no history: the plain prefill
    dict(lengths=(700, 64, 1000), hist=(443, 63, 1000)),    # chunks start off every boundary; one token; an idle sequence
    dict(lengths=(2049,), hist=(1536,)),                    # history ends on a block boundary
    dict(lengths=(300, 1300), hist=(236, 1044)),            # one-tile chunk next to a four-tile one
    dict(lengths=(200, 130), hist=(199, 1)),                # a one-token chunk (a decode step); a one-token history
])
def test_chunk_prefill_over_one_pool_matches_oracle_on_every_row(dtype, case):
    L = _lib()
    dev = torch.device("cuda:0")
    lengths, hist = case["lengths"], case["hist"]
    B_ = len(lengths)
    w = Workload(name="cp", batch=B_, num_q_heads=4, num_kv_heads=2, dtype=dtype, streaming_kv_heads=(0,),
                 sink_tokens=64, local_tokens=192, seed=41)
    pin = make_prefill_inputs(w, lengths=lengths)
    max_pages = max(-(-l // NP) for l in lengths) + 1
    g = torch.Generator().manual_seed(23)
    page_table = torch.randperm(B_ * max_pages + 2, generator=g)[:B_ * max_pages].to(torch.int32).reshape(B_, max_pages)
    k_pool = torch.full((B_ * max_pages + 2, 2, NP, 128), float("nan"), dtype=pin.k.dtype)  # only the history is there
    v_pool = torch.full_like(k_pool, float("nan"))
    for b, S in enumerate(hist):
        a = int(pin.cu_seqlens[b])
        pos = torch.arange(S)
        phys = page_table[b].long()[pos // NP]
        k_pool[phys, :, pos % NP] = pin.k[a:a + S]
        v_pool[phys, :, pos % NP] = pin.v[a:a + S]
    stats = torch.zeros((k_pool.shape[0], 2, 4, 2, 128), dtype=pin.k.dtype, device=dev)  # for the write-back below
    kv = L.PagedKV(k_pool.to(dev), v_pool.to(dev), stats, page_table.to(dev), _pad4(list(hist), dev))
    desc, out, lse, (qc, kc, vc, cu_new, chunks) = _check_chunk(L, w, pin, lengths, hist, kv, dev,
                                                                 f"chunk prefill {dtype} {case}")
    # the same rows through the other two calls: identical tile walks, identical bits
    if all(S == 0 for S in hist):
        out_c = torch.empty_like(out)
        lse_c = torch.empty_like(lse)
        L.lserve_sparse_prefill(desc, pin.q.to(dev), pin.k.to(dev), pin.v.to(dev), pin.cu_seqlens.to(dev), max(lengths),
                                out_c, lse_c, None)
        assert torch.equal(out.view(torch.int16), out_c.view(torch.int16)) and torch.equal(lse, lse_c)
    L.lserve_append_kv(desc, kv, kc.to(dev), vc.to(dev), _pad4(cu_new, dev), _pad4(list(hist), dev), max(max(chunks), 1))
    kv.seq_lens = _pad4(list(lengths), dev)
    out_p = torch.empty_like(out)
    lse_p = torch.empty_like(lse)
    qd = torch.cat([qc, torch.zeros((1, 4, 128), dtype=qc.dtype)]).to(dev)[:qc.shape[0]]
    L.lserve_sparse_prefill_paged(desc, kv, qd, _pad4(cu_new, dev), max(chunks), max(lengths), out_p, lse_p, None)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), out_p.view(torch.int16)) and torch.equal(lse, lse_p)


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
def test_prefill_in_chunks_over_the_two_way_cache_attention_first_then_write_back(dtype):
    """A prompt goes through in four chunks, each: attention with the history in the two-way cache, then write-back.
    Streaming heads live in a ring of s + w pages that wraps several times; what the ring has dropped is NaN in
    the oracle's history and must not be needed."""
    L = _lib()
    dev = torch.device("cuda:0")
    lengths = (1100, 333, 64)
    steps = [(300, 100, 0), (557, 101, 30), (558, 300, 64), (1100, 333, 64)]  # lengths after each chunk
    B_ = len(lengths)
    w = Workload(name="cp2", batch=B_, num_q_heads=8, num_kv_heads=4, dtype=dtype, streaming_kv_heads=(0, 2),
                 sink_tokens=64, local_tokens=192, seed=43)
    s_pages, w_pages = 1, 3
    ring = s_pages + w_pages
    pin = make_prefill_inputs(w, lengths=lengths)
    max_pages = max(-(-l // NP) for l in lengths) + 1
    g = torch.Generator().manual_seed(29)
    page_table = torch.randperm(B_ * max_pages + 2, generator=g)[:B_ * max_pages].to(torch.int32).reshape(B_, max_pages)
    ring_table = torch.randperm(B_ * ring + 3, generator=g)[:B_ * ring].to(torch.int32).reshape(B_, ring)
    nan = float("nan")
    k_main = torch.full((B_ * max_pages + 2, 2, NP, 128), nan, dtype=pin.k.dtype, device=dev)
    k_ring = torch.full((B_ * ring + 3, 2, NP, 128), nan, dtype=pin.k.dtype, device=dev)
    stats = torch.zeros((B_ * max_pages + 2, 2, 4, 2, 128), dtype=pin.k.dtype, device=dev)
    kv = L.PagedKV(k_main, k_main.clone(), stats, page_table.to(dev), _pad4([0] * B_, dev), pool_heads=2,
                   k_pool_stream=k_ring, v_pool_stream=k_ring.clone(), ring_table=ring_table.to(dev))
    hist = [0] * B_
    for now in steps:
        if all(a == h for a, h in zip(now, hist)):
            continue

        def dropped(b, hk, u, hist=tuple(hist)):  # streaming heads: only sink pages and the last w pages remain
            P = -(-hist[b] // NP)
            return hk in (0, 2) and not (u // NP < s_pages or u // NP >= P - w_pages)

        desc, out, lse, (qc, kc, vc, cu_new, chunks) = _check_chunk(L, w, pin, now, hist, kv, dev,
                                                                     f"two-way chunk {dtype} {hist}->{now}", dropped)
        L.lserve_append_kv(desc, kv, kc.to(dev), vc.to(dev), _pad4(cu_new, dev), _pad4(list(hist), dev), max(max(chunks), 1))
        hist = list(now)


# ---- the paper's cache: quantised pages, two-way -------------------------------------------------------------

def _cache_values(kv, bits, page_table, ring_table, hist, n_kv_heads, streaming, s_pages, w_pages):
    """float64 [B, max hist, Hkv, D] x 2 of what the cache holds for every history position (NaN where it holds
    nothing): bytes of the pools read back, codes / scales / zero points taken apart, code * scale + zero."""
    from test_gpu_quant import _values

    def vals(pool):
        return None if pool is None else _values(pool.cpu(), bits)
    km, vm, kr, vr = vals(kv.k_pool), vals(kv.v_pool), vals(kv.k_pool_stream), vals(kv.v_pool_stream)
    dense = [h for h in range(n_kv_heads) if h not in streaming]
    B = len(hist)
    stride = max(max(hist), 1)
    kh = np.full((B, stride, n_kv_heads, 128), np.nan)
    vh = np.full_like(kh, np.nan)
    for b, S in enumerate(hist):
        P = -(-S // NP)
        for u in range(S):
            p, t = u // NP, u % NP
            for hk in range(n_kv_heads):
                if kr is not None and hk in streaming:
                    if not (p < s_pages or p >= P - w_pages):
                        continue  # dropped by the ring
                    slot = p if p < s_pages else s_pages + (p - s_pages) % w_pages
                    page, rank = int(ring_table[b, slot]), list(streaming).index(hk)
                    kh[b, u, hk], vh[b, u, hk] = kr[page, rank, t], vr[page, rank, t]
                else:
                    page = int(page_table[b, p])
                    rank = dense.index(hk) if km.shape[1] != n_kv_heads else hk
                    kh[b, u, hk], vh[b, u, hk] = km[page, rank, t], vm[page, rank, t]
    return kh, vh


# bf16: the dequantised key is rounded to bf16 (2^-9 relative) like the scaled query, which adds a second term of the
# same size to the logit error: sqrt(2) x the 9e-3 four-sigma bound of the 16-bit cache
LSE_TOL_QUANT_HISTORY = {"fp16": 2e-3, "bf16": 1.3e-2}


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
@pytest.mark.parametrize("two_way", [False, True])
def test_prefill_in_chunks_over_quantised_pages_attention_first_then_quantising_write_back(dtype, bits, two_way):
    """The cache the paper keeps: low-bit pages, streaming heads in their ring.  Each chunk attends the numbers the
    bytes of the cache stand for (read back and dequantised on the CPU for the oracle) plus its own 16-bit K / V,
    then the quantising write-back adds it to the cache."""
    L = _lib()
    dev = torch.device("cuda:0")
    lengths = (900, 333, 64)
    steps = [(300, 100, 0), (557, 101, 30), (558, 300, 64), (900, 333, 64)]
    B_ = len(lengths)
    streaming = (0, 2)
    w = Workload(name="cpq", batch=B_, num_q_heads=8, num_kv_heads=4, dtype=dtype, streaming_kv_heads=streaming,
                 sink_tokens=64, local_tokens=192, seed=47)
    s_pages, w_pages = 1, 3
    ring = s_pages + w_pages
    pin = make_prefill_inputs(w, lengths=lengths)
    max_pages = max(-(-l // NP) for l in lengths) + 1
    g = torch.Generator().manual_seed(31)
    page_table = torch.randperm(B_ * max_pages + 2, generator=g)[:B_ * max_pages].to(torch.int32).reshape(B_, max_pages)
    ring_table = torch.randperm(B_ * ring + 3, generator=g)[:B_ * ring].to(torch.int32).reshape(B_, ring)
    slab = 64 * 128 * bits // 8 + 256
    main_heads = 2 if two_way else 4
    mk = lambda pages, heads: torch.full((pages, heads, slab), 0xff, dtype=torch.uint8, device=dev)  # NaN scales / zeros
    stats = torch.zeros((B_ * max_pages + 2, main_heads, 4, 2, 128), dtype=pin.k.dtype, device=dev)
    kv = L.PagedKV(mk(B_ * max_pages + 2, main_heads), mk(B_ * max_pages + 2, main_heads), stats, page_table.to(dev),
                   _pad4([0] * B_, dev), kv_bits=bits)
    if two_way:
        kv.pool_heads = 2
        kv.k_pool_stream, kv.v_pool_stream = mk(B_ * ring + 3, 2), mk(B_ * ring + 3, 2)
        kv.ring_table = ring_table.to(dev)
    desc = L.AttnDesc(w.num_q_heads, w.num_kv_heads, w.streaming_flags(), dtype=w.torch_dtype,
                      sink_tokens=w.sink_tokens, local_tokens=w.local_tokens)
    H = w.num_q_heads
    hist = [0] * B_
    for now in steps:
        qc, kc, vc, _ = _split(pin, now, hist)
        chunks = [a - h for a, h in zip(now, hist)]
        total_new = qc.shape[0]
        cu_new = np.concatenate([[0], np.cumsum(chunks)]).astype(np.int32)
        kh, vh = _cache_values(kv, bits, page_table, ring_table, hist, w.num_kv_heads, streaming if two_way else (),
                               s_pages, w_pages)
        out = torch.full((total_new, H, 128), float("nan"), dtype=qc.dtype, device=dev)
        lse = torch.full((H, total_new), float("nan"), dtype=torch.float32, device=dev)
        kv.seq_lens = _pad4(list(hist), dev)
        qd, kd, vd = qc.to(dev), kc.to(dev), vc.to(dev)
        L.lserve_sparse_prefill_chunk(desc, kv, qd, kd, vd, _pad4(cu_new, dev), max(chunks), out, lse)
        torch.cuda.synchronize()
        tok = np.repeat(np.arange(total_new, dtype=np.int32), H)
        head = np.tile(np.arange(H, dtype=np.int32), total_new)
        ref, lse_ref = oracle.chunk_prefill_rows(qc, kc, vc, kh, vh, np.asarray(hist, np.int32), cu_new,
                                                 w.streaming_flags(), NP, w.sink_tokens, w.local_tokens, tok, head)
        assert np.isfinite(ref).all()
        what = f"quantised chunk {dtype} {bits} bit two_way={two_way} {hist}->{list(now)}"
        assert_attention_close(out, ref.reshape(total_new, H, -1), what)
        assert_lse_close(lse.t().contiguous(), lse_ref.reshape(total_new, H), what + " lse", LSE_TOL_QUANT_HISTORY[dtype])
        L.lserve_append_kv(desc, kv, kd, vd, _pad4(cu_new, dev), _pad4(list(hist), dev), max(max(chunks), 1))
        hist = list(now)

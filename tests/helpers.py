"""Shared test helpers: gathering paged KV into contiguous arrays (indexing only)."""
import numpy as np
import torch


def gather_tokens(pool: torch.Tensor, page_table, b: int, length: int) -> np.ndarray:
    """[length, Hkv, D] float64 view of the first `length` tokens of sequence b."""
    NP = pool.shape[2]
    pt = np.asarray(page_table)[b]
    pos = np.arange(length)
    phys = pt[pos // NP]
    x = pool[torch.from_numpy(phys).long(), :, torch.from_numpy(pos % NP).long()]  # [length, Hkv, D]
    return x.to(torch.float64).numpy()


def small_decode_workload(**kw):
    from workloads import Workload

    base = dict(name="tiny", batch=2, num_q_heads=4, num_kv_heads=2, dtype="fp16",
                streaming_kv_heads=(0,), sink_tokens=64, local_tokens=128, budget_tokens=256,
                reuse_interval=2, decode_steps=2, lengths=(300, 777), seed=7, pool_slack=0.3)
    base.update(kw)
    return Workload(**base)


def sub_problem(inp, seqs):
    """CPU copy of the sequences `seqs` of a (possibly device-resident, large) decode problem.

    Only the pages those sequences own are gathered into a small pool with a renumbered page table,
    so that the oracle can check sampled sequences of a full-size run.  Pure indexing and copies.
    """
    from workloads import DecodeInputs
    from dataclasses import replace

    w = inp.workload
    steps = max(1, w.decode_steps)
    rows, tables, off = [], [], 0
    max_pages = inp.page_table.shape[1]
    for b in seqs:
        n_pages = (int(inp.prompt_lens[b]) + steps + w.page_size - 1) // w.page_size
        rows.append(inp.page_table[b, :n_pages].long())
        t = torch.zeros(max_pages, dtype=torch.int32)
        t[:n_pages] = torch.arange(off, off + n_pages, dtype=torch.int32)
        tables.append(t)
        off += n_pages
    idx = torch.cat(rows)
    sel = torch.tensor(list(seqs), dtype=torch.long, device=inp.q.device)
    return DecodeInputs(
        workload=replace(w, batch=len(seqs)),
        k_pool=inp.k_pool[idx].cpu(),
        v_pool=inp.v_pool[idx].cpu(),
        page_table=torch.stack(tables),
        prompt_lens=inp.prompt_lens[sel].cpu(),
        q=inp.q[:, sel].cpu(),
        needle_pos=None if inp.needle_pos is None else inp.needle_pos[list(seqs)],
        k_scale=inp.k_scale,
    )


def block_mask_csr(masks, lengths, tile=64):
    """CSR arrays of a list of block masks.

    masks[m](b, i) -> iterable of kept key tiles (each <= i) of query tile i of sequence b.  Returns
    (q_tile_start [B+1], row_ptr [M*R+1], cols, R) as int32 numpy arrays, rows ordered mask-major.
    """
    import numpy as np
    n_tiles = [-(-int(l) // tile) for l in lengths]
    q_tile_start = np.concatenate([[0], np.cumsum(n_tiles)]).astype(np.int32)
    R = int(q_tile_start[-1])
    row_ptr, cols = [0], []
    for fn in masks:
        for b, nt in enumerate(n_tiles):
            for i in range(nt):
                row = sorted(set(int(j) for j in fn(b, i)))
                assert all(0 <= j <= i for j in row)
                cols.extend(row)
                row_ptr.append(len(cols))
    return q_tile_start, np.asarray(row_ptr, dtype=np.int32), np.asarray(cols, dtype=np.int32), R

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

"""Comparison rules between the HIP path and the oracle.

Floating point: for fp16 storage with fp32 accumulation the attention output must satisfy
max |delta| <= 2e-3 over all elements and, per output row, ||delta||_2 / ||ref||_2 <= 1e-2.
bf16 storage has 8x coarser rounding of the stored output, so its absolute bound is 1.6e-2
with the same row-relative bound.  Integer results (selected page sets) must be identical,
except where the oracle's own scores show a near-tie at the cut (relative gap < 1e-6): those
are counted and reported, never hidden.
"""
import numpy as np
import torch

ABS_TOL = {torch.float16: 2e-3, torch.bfloat16: 1.6e-2}
ROW_REL_TOL = 1e-2
SCORE_REL_TOL = 1e-5
NEAR_TIE_REL = 1e-6


def assert_attention_close(got: torch.Tensor, ref: np.ndarray, what: str = ""):
    g = got.detach().to(torch.float64).cpu().numpy().reshape(ref.shape)
    assert np.isfinite(g).all(), f"{what}: non-finite values in the GPU output"
    delta = g - ref
    max_abs = np.abs(delta).max() if delta.size else 0.0
    rows = delta.reshape(-1, delta.shape[-1])
    refr = ref.reshape(-1, ref.shape[-1])
    rel = np.linalg.norm(rows, axis=1) / np.maximum(np.linalg.norm(refr, axis=1), 1e-30)
    max_rel = rel.max() if rel.size else 0.0
    assert max_abs <= ABS_TOL[got.dtype], f"{what}: max abs error {max_abs:.3e} > {ABS_TOL[got.dtype]}"
    assert max_rel <= ROW_REL_TOL, f"{what}: max row-relative error {max_rel:.3e} > {ROW_REL_TOL}"
    OBSERVED.append((what, "out", float(max_abs), float(max_rel)))
    return max_abs, max_rel


# Log-sum-exp.  Decode keeps the query exact: 2e-3.  Prefill rounds the query times the softmax scale to the
# storage type (unit roundoff u = 2^-11 for fp16, 2^-8 for bf16), which moves a logit of 128 N(0,1) products by
# about 0.58 u (one sigma) and the log-sum-exp by at most the largest logit move: four sigma is 1.1e-3 for fp16
# and 9e-3 for bf16, and the bound is that four-sigma figure (fp16 keeps the 2e-3 of the output bound).
LSE_TOL_DECODE = 2e-3
LSE_TOL_PREFILL = {"fp16": 2e-3, "bf16": 9e-3}

# Largest errors seen by the assertions of the running test: (what, kind, max abs, max row-relative or 0).
# tests/conftest.py prints them after each test so that a run's log records the margins, not only pass / fail.
OBSERVED = []


def assert_lse_close(got: torch.Tensor, ref: np.ndarray, what: str = "", tol: float = LSE_TOL_DECODE):
    g = got.detach().to(torch.float64).cpu().numpy().reshape(ref.shape)
    err = np.abs(g - ref).max() if ref.size else 0.0
    assert err <= tol, f"{what}: lse error {err:.3e} > {tol}"
    OBSERVED.append((what, "lse", float(err), 0.0))


def compare_selection(sel_gpu, cnt_gpu, sel_ref, cnt_ref, scores_ref, streaming_flags):
    """Bit-exact set comparison per (sequence, KV head); returns the number of near-tie rows.

    A row whose sets differ passes only if every page of the symmetric difference scores within
    NEAR_TIE_REL (relative) of the oracle's cut score, the lowest score the oracle selected among
    the non-forced pages.
    """
    sel_gpu, cnt_gpu = np.asarray(sel_gpu), np.asarray(cnt_gpu)
    near_ties = 0
    B, Hkv = cnt_ref.shape
    for b in range(B):
        for hk in range(Hkv):
            if streaming_flags[hk]:
                assert cnt_gpu[b, hk] == 0
                continue
            assert cnt_gpu[b, hk] == cnt_ref[b, hk], (b, hk, cnt_gpu[b, hk], cnt_ref[b, hk])
            a = sel_gpu[b, hk, :cnt_gpu[b, hk]]
            r = sel_ref[b, hk, :cnt_ref[b, hk]]
            assert (np.diff(a) > 0).all(), "GPU selection must be ascending and unique"
            assert (sel_gpu[b, hk, cnt_gpu[b, hk]:] == -1).all()
            if np.array_equal(a, r):
                continue
            diff = set(a.tolist()) ^ set(r.tolist())
            sc = scores_ref[b, hk]
            cut = min(sc[p] for p in r[:-1])  # the forced newest page is last and not ranked
            for p in diff:
                assert abs(sc[p] - cut) <= NEAR_TIE_REL * abs(cut), \
                    f"selection differs beyond a near-tie at b={b} hk={hk} page={p}: {sc[p]} vs cut {cut}"
            near_ties += 1
    return near_ties

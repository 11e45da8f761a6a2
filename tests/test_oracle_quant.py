"""Pins for the oracle's 8-bit and 4-bit KV quantiser (Sec. 3.2: one scale factor and zero point per token,
stored after the token features) and for decode over the values a quantised cache stands for.

The quantiser is a definition (an encoding), so it is pinned by rows whose codes are known by
construction, by a row worked by hand, by brute force over all codes, and by the error bound
the definition implies."""
import numpy as np
import pytest
import torch

import oracle


def _row(values, dtype=torch.float16, D=128, fill=None):
    x = torch.full((D,), float(values[0] if fill is None else fill), dtype=torch.float32)
    x[: len(values)] = torch.tensor(values, dtype=torch.float32)
    return x.to(dtype)


def test_a_row_on_the_code_lattice_gets_its_lattice_indices():
    # x_c = -1 + k_c / 64 with k = 0, 2, ..., 252 and 255: range 255 / 64, so scale = 1 / 64 and zero = -1
    # are both exact in fp16 and every feature sits on a code.
    k = np.concatenate([np.arange(0, 254, 2), [255]])
    x = torch.tensor(-1.0 + k / 64.0, dtype=torch.float32).to(torch.float16)
    codes, scale, zero = oracle.quantize_q8(x)
    assert float(scale) == 1.0 / 64.0 and float(zero) == -1.0
    assert np.array_equal(codes, k.astype(np.uint8))
    assert np.array_equal(oracle.dequantize_q8(codes, scale, zero), x.double().numpy())


def test_a_constant_row_keeps_its_value():
    for dtype in (torch.float16, torch.bfloat16):
        x = torch.full((2, 128), 0.7265625, dtype=dtype)  # exact in both storage types
        codes, scale, zero = oracle.quantize_q8(x)
        assert not codes.any() and float(scale[0]) == 0.0 and float(zero[1]) == 0.7265625
        assert np.array_equal(oracle.dequantize_q8(codes, scale, zero), x.double().numpy())


def test_a_row_worked_by_hand():
    # lo = 0, hi = 1: zero = 0; 1 / 255 = 0.0039215686... lies between the fp16 neighbours
    # 2^-8 (1 + 4 / 1024) = 0.00392150879 and 2^-8 (1 + 5 / 1024) = 0.00392532349 and is nearer the first.
    # fp16(0.3) = 0.300048828125 -> 76.51 -> 77;  0.5 -> 127.502 -> 128;  fp16(0.1) = 0.0999755859375 -> 25.49 -> 25;
    # fp16(0.9) = 0.89990234375 -> 229.48 -> 229;  1.0 -> 255.004 -> 255.
    x = _row([0.0, 1.0, 0.3, 0.5, 0.1, 0.9], fill=0.0)
    codes, scale, zero = oracle.quantize_q8(x)
    assert float(zero) == 0.0
    assert float(scale) == 2.0 ** -8 * (1 + 4 / 1024)
    assert codes[:6].tolist() == [0, 255, 77, 128, 25, 229]
    assert not codes[6:].any()


def test_four_bit_rows_known_by_construction_and_by_hand():
    # lattice: x_c = 2 + k_c / 8 with every k in 0 .. 15 present: scale = 1 / 8, zero = 2, codes = k
    k = np.arange(128) % 16
    x = torch.tensor(2.0 + k / 8.0, dtype=torch.float32).to(torch.bfloat16)
    codes, scale, zero = oracle.quantize_kv(x, 4)
    assert float(scale) == 0.125 and float(zero) == 2.0 and np.array_equal(codes, k.astype(np.uint8))
    assert np.array_equal(oracle.dequantize_q8(codes, scale, zero), x.double().numpy())
    # by hand: lo = 0, hi = 1: 1 / 15 = 0.0666... lies between the fp16 neighbours 2^-4 (1 + 68 / 1024) = 0.06665039
    # and 2^-4 (1 + 69 / 1024) = 0.06671143 and is nearer the first.  fp16(0.3) = 0.30004883 -> 4.502 -> 5 (the real
    # quotient 0.3 / (1 / 15) = 4.5 would tie); 0.5 -> 7.502 -> 8; fp16(0.1) = 1638 / 16384 over the scale 1092 / 16384
    # is exactly 1.5, a tie that goes to the even code 2; fp16(0.9) -> 13.502 -> 14.
    x = _row([0.0, 1.0, 0.3, 0.5, 0.1, 0.9], fill=0.0)
    codes, scale, zero = oracle.quantize_kv(x, 4)
    assert float(scale) == 2.0 ** -4 * (1 + 68 / 1024) and float(zero) == 0.0
    assert codes[:6].tolist() == [0, 15, 5, 8, 2, 14] and not codes[6:].any()


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
def test_codes_are_the_nearest_of_all_256_and_the_error_stays_inside_the_bound(dtype, bits):
    g = torch.Generator().manual_seed(5)
    top = 2 ** bits - 1
    x = (torch.randn((40, 3, 128), generator=g) * torch.rand((40, 3, 1), generator=g) * 6 + 2 * torch.randn((40, 3, 1), generator=g)).to(dtype)
    codes, scale, zero = oracle.quantize_kv(x, bits)
    xd = x.double().numpy()
    sc, ze = scale.astype(np.float64), zero.astype(np.float64)
    # brute force: distance of every feature to each of the 256 values a byte can stand for
    grid = np.arange(top + 1, dtype=np.float64)[None, None, None, :] * sc[..., None, None] + ze[..., None, None]
    dist = np.abs(xd[..., None] - grid)
    chosen = np.take_along_axis(dist, codes[..., None].astype(np.int64), axis=-1)[..., 0]
    # a tie between two neighbouring codes may go either way; fp32 rounding of the quotient can move a
    # feature that sits within 2^-23 of a tie
    assert np.all(chosen <= dist.min(axis=-1) + 1e-6 * sc[..., None])
    # the extremes take the end codes; the range is covered up to the fp16 rounding of the scale
    assert np.all(np.take_along_axis(codes, xd.argmin(-1)[..., None], -1) == 0)
    assert np.all(np.take_along_axis(codes, xd.argmax(-1)[..., None], -1) == top)
    span = xd.max(-1) - ze
    assert np.all(np.abs(top * sc - span) <= span * 2.0 ** -11)
    assert np.all(np.abs(ze - xd.min(-1)) <= np.abs(xd.min(-1)) * 2.0 ** -11)
    # error bound: half a step, plus the part of the range the rounded scale and zero point do not cover
    err = np.abs(oracle.dequantize_q8(codes, scale, zero) - xd)
    bound = 0.5 * sc + span * 2.0 ** -11 + np.abs(xd.min(-1)) * 2.0 ** -11
    assert np.all(err <= bound[..., None] * (1 + 1e-6))
    # order is kept
    order = np.argsort(xd, axis=-1, kind="stable")
    assert np.all(np.diff(np.take_along_axis(codes.astype(np.int32), order, -1), axis=-1) >= 0)


def test_decode_over_values_matches_a_direct_softmax_and_the_16_bit_decode():
    B, H, Hkv, NP, D = 2, 4, 2, 8, 16
    g = torch.Generator().manual_seed(9)
    k_pool = torch.randn((6, Hkv, NP, D), generator=g).to(torch.float16)
    v_pool = torch.randn((6, Hkv, NP, D), generator=g).to(torch.float16)
    q = torch.randn((B, H, D), generator=g).to(torch.float16)
    page_table = torch.tensor([[3, 0, 5], [1, 4, 2]], dtype=torch.int32)
    seq_lens = np.array([19, 24], np.int32)
    sel = np.array([[[0, 2], [1, -1]], [[0, 1], [2, -1]]], np.int32)
    cnt = np.array([[2, 1], [2, 1]], np.int32)
    flags = [0, 0]
    kc, ks, kz = oracle.quantize_q8(k_pool)
    vc, vs, vz = oracle.quantize_q8(v_pool)
    kval, vval = oracle.dequantize_q8(kc, ks, kz), oracle.dequantize_q8(vc, vs, vz)
    out, lse = oracle.sparse_decode_values(q, kval, vval, page_table, seq_lens, sel, cnt, seq_lens, flags, 8, 8)
    # direct: gather the attended tokens with numpy indexing and apply Eq. 1
    for b in range(B):
        for h in range(H):
            hk = h // (H // Hkv)
            rows_k, rows_v = [], []
            for p in sorted(sel[b, hk, : cnt[b, hk]].tolist()):
                n = min(NP, int(seq_lens[b]) - p * NP)
                rows_k.append(kval[int(page_table[b, p]), hk, :n])
                rows_v.append(vval[int(page_table[b, p]), hk, :n])
            K, V = np.concatenate(rows_k), np.concatenate(rows_v)
            s = K @ q[b, h].double().numpy() / np.sqrt(D)
            w = np.exp(s - s.max())
            np.testing.assert_allclose(out[b, h], (w / w.sum()) @ V, rtol=1e-12, atol=1e-13)
            np.testing.assert_allclose(lse[b, h], s.max() + np.log(w.sum()), rtol=1e-12)
    # a pool of doubles that holds exactly the 16-bit values gives the 16-bit decode
    o16, l16 = oracle.sparse_decode(q, k_pool, v_pool, page_table, seq_lens, sel, cnt, seq_lens, flags, 8, 8)
    o64, l64 = oracle.sparse_decode_values(q, k_pool.double().numpy(), v_pool.double().numpy(), page_table, seq_lens,
                                           sel, cnt, seq_lens, flags, 8, 8)
    assert np.array_equal(o16, o64) and np.array_equal(l16, l64)

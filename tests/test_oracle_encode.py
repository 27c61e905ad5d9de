"""Pins for the oracle's scales, quantiser and packing (Eq. (1), Section 3.2.1).

Closed forms: rows whose part maxima are exactly 127 / 7 make Q/amax == 1.0, so the
codes must be the round-half-even of the values themselves, including exact half-way
cases.  Invariants: disjoint support, half-step reconstruction bound, |code| == Q at
the maximum, k set bits per bank, pack/unpack identity.
"""
import numpy as np
import pytest

import oracle
from workloads import f32_to_bf16_bits, bf16_bits_to_f32, unpack_int4, make


def dense_hi(enc) -> np.ndarray:
    """Scatter hi_val back to [M, K] using the mask (test-side helper, python loops)."""
    out = np.zeros((enc.M, enc.K), np.int32)
    for m in range(enc.M):
        mk = enc.mask if enc.mode == 1 else enc.mask[m]
        pos = [j for j in range(enc.K) if (int(mk[j // 32]) >> (j % 32)) & 1]
        assert len(pos) == (enc.K // enc.bank) * enc.topk
        out[m, pos] = enc.hi_val[m].reshape(-1)
    return out


def mask_flags(enc) -> np.ndarray:
    mk = np.broadcast_to(enc.mask, (enc.M, enc.K // 32)) if enc.mode == 1 else enc.mask
    bits = (mk[:, :, None] >> np.arange(32, dtype=np.uint32)[None, None, :]) & 1
    return bits.reshape(enc.M, enc.K).astype(bool)


def test_unit_scale_row_gives_rne_of_values():
    hi = [127.0, -100.5, 63.5, 12.5, -11.5, 10.5, 9.5, 8.5]
    hi_codes = [127, -100, 64, 12, -12, 10, 10, 8]
    lo = [0.5, 1.5, 2.5, -0.5, -2.5, 3.5, -3.5, 6.5, 7.0, -7.0, 0.25, 0.75, 4.5, 5.5, -1.5, -4.5]
    lo_codes = [0, 2, 2, 0, -2, 4, -4, 6, 7, -7, 0, 1, 4, 6, -2, -4]
    x = np.zeros(64, np.float32)
    hi_pos = [3, 9, 17, 22, 31, 40, 50, 63]
    lo_pos = [j for j in range(64) if j not in hi_pos][:len(lo)]
    x[hi_pos] = hi
    x[lo_pos] = lo
    bits = f32_to_bf16_bits(x)
    assert np.array_equal(bf16_bits_to_f32(bits), x)  # every value is exact in bf16
    enc = oracle.encode(bits[None, :], 64, 8)
    assert enc.s_hi[0] == np.float32(1.0) and enc.s_lo[0] == np.float32(1.0)
    assert list(enc.hi_val[0, 0]) == hi_codes  # ascending channel order
    d = unpack_int4(enc.d_lo)[0]
    assert [int(d[j]) for j in lo_pos] == lo_codes
    assert all(d[j] == 0 for j in hi_pos)
    flags = mask_flags(enc)[0]
    assert list(np.flatnonzero(flags)) == hi_pos


def test_power_of_two_scales():
    # amax_hi = 254 -> s_hi = 2, codes = rne(x/2); amax_lo = 3.5 -> s_lo = 0.5, codes = rne(2x)
    x = np.zeros(32, np.float32)
    x[[0, 5]] = [254.0, -5.0]            # hi (k=2): 5/2 = 2.5 -> -2
    x[[1, 2, 3, 4]] = [3.5, 0.25, 0.75, -1.25]   # 2x = 7, 0.5->0, 1.5->2, -2.5->-2
    enc = oracle.encode(f32_to_bf16_bits(x)[None, :], 32, 2)
    assert enc.s_hi[0] == np.float32(2.0) and enc.s_lo[0] == np.float32(0.5)
    assert list(enc.hi_val[0, 0]) == [127, -2]
    d = unpack_int4(enc.d_lo)[0]
    assert list(d[:6]) == [0, 7, 0, 2, -2, 0]


@pytest.mark.parametrize("b,k", [(32, 4), (64, 8), (128, 16)])
def test_invariants_random(b, k):
    rng = np.random.default_rng(1234 + b)
    M, K = 12, 4 * b
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[:, rng.choice(K, 3, replace=False)] *= 30.0
    bits = f32_to_bf16_bits(x)
    xv = bf16_bits_to_f32(bits).astype(np.float64)
    enc = oracle.encode(bits, b, k)
    flags = mask_flags(enc)
    # exactly k per bank, every bank, every row
    assert (flags.reshape(M, K // b, b).sum(-1) == k).all()
    assert int(sum(bin(int(w)).count("1") for w in enc.mask.reshape(-1))) == M * (K // b) * k
    d = unpack_int4(enc.d_lo).astype(np.int32)
    h = dense_hi(enc)
    # disjoint support
    assert not (d[flags] != 0).any()
    assert not (h[~flags] != 0).any()
    # ranges: symmetric, -8 and -128 never appear
    assert d.min() >= -7 and d.max() <= 7 and h.min() >= -127 and h.max() <= 127
    # selection invariant per bank
    mag = np.abs(xv).reshape(M, K // b, b)
    fl = flags.reshape(M, K // b, b)
    assert (np.where(fl, mag, np.inf).min(-1) >= np.where(fl, -np.inf, mag).max(-1)).all()
    # reconstruction within half a step of the owning part
    s_lo = enc.s_lo.astype(np.float64)[:, None]
    s_hi = enc.s_hi.astype(np.float64)[:, None]
    rec = d * s_lo + h * s_hi
    step = np.where(flags, s_hi, s_lo)
    assert (np.abs(xv - rec) <= 0.5 * step * (1 + 1e-5)).all()
    # the maximum of each part maps to +-Q
    for m in range(M):
        assert np.abs(h[m]).max() == 127 and np.abs(d[m]).max() == 7
        assert enc.s_hi[m] == np.float32(np.float32(np.abs(xv[m][flags[m]]).max()) / np.float32(127.0))
        assert enc.s_lo[m] == np.float32(np.float32(np.abs(xv[m][~flags[m]]).max()) / np.float32(7.0))


def test_zero_row_and_all_high():
    bits = np.zeros((2, 64), np.uint16)
    bits[1] = f32_to_bf16_bits(np.linspace(-4, 4, 64).astype(np.float32))
    enc = oracle.encode(bits, 64, 8)
    assert enc.s_lo[0] == 1.0 and enc.s_hi[0] == 1.0
    assert not enc.d_lo[0].any() and not enc.hi_val[0].any()
    assert list(np.flatnonzero(mask_flags(enc)[0])) == list(range(8))  # all equal -> first k
    # k == b: every channel is high precision, the low part is empty
    enc2 = oracle.encode(bits, 64, 64)
    assert not enc2.d_lo.any() and enc2.s_lo[1] == 1.0
    assert (mask_flags(enc2)).all()
    xv = bf16_bits_to_f32(bits[1])
    inv = np.float32(127.0) / np.float32(np.abs(xv).max())
    want = np.rint((xv * inv).astype(np.float32)).astype(np.int32)
    assert np.array_equal(enc2.hi_val[1].reshape(-1).astype(np.int32), want)


def test_static_mask_mode():
    rng = np.random.default_rng(5)
    K, b, k = 128, 32, 4
    flags = np.zeros(K, bool)
    for g in range(K // b):
        flags[g * b + rng.choice(b, k, replace=False)] = True
    mask = np.zeros(K // 32, np.uint32)
    for j in np.flatnonzero(flags):
        mask[j // 32] |= np.uint32(1) << np.uint32(j % 32)
    x = rng.standard_normal((5, K)).astype(np.float32)
    bits = f32_to_bf16_bits(x)
    xv = bf16_bits_to_f32(bits)
    enc = oracle.encode(bits, b, k, static_mask=mask)
    assert enc.mode == 1
    for m in range(5):
        amax_hi = np.float32(np.abs(xv[m][flags]).max())
        inv = np.float32(127.0) / amax_hi
        want = np.clip(np.rint((xv[m][flags] * inv).astype(np.float32)), -127, 127).astype(np.int32)
        assert np.array_equal(enc.hi_val[m].reshape(-1).astype(np.int32), want)
        d = unpack_int4(enc.d_lo[m:m + 1])[0]
        assert not d[flags].any()
        # a static mask can leave larger values in the low part: they must clamp at +-7, not wrap
        assert d.min() >= -7 and d.max() <= 7
    # a mask whose bank counts are wrong is refused
    bad = mask.copy()
    bad[0] |= np.uint32(0xFFFF)
    with pytest.raises(ValueError):
        oracle.encode(bits, b, k, static_mask=bad)


def test_numpy_twin_on_config1():
    """Vectorised numpy restatement of the encoding on the tiny benchmark configuration."""
    w = make("c1_tiny", with_weights=False)
    enc = oracle.encode(w.x_bits, w.bank, w.topk)
    xv = bf16_bits_to_f32(w.x_bits)
    M, K, b, k = w.M, w.K, w.bank, w.topk
    mag = (w.x_bits & 0x7FFF).astype(np.int64).reshape(M, K // b, b)
    order = np.argsort(-mag, axis=-1, kind="stable")  # descending magnitude, stable -> lowest index first
    flags = np.zeros((M, K // b, b), bool)
    np.put_along_axis(flags, order[..., :k], True, axis=-1)
    flags = flags.reshape(M, K)
    assert np.array_equal(flags, mask_flags(enc))
    a = np.abs(xv)
    amax_hi = np.where(flags, a, 0).max(1).astype(np.float32)
    amax_lo = np.where(flags, 0, a).max(1).astype(np.float32)
    inv_hi = (np.float32(127.0) / amax_hi).astype(np.float32)
    inv_lo = (np.float32(7.0) / amax_lo).astype(np.float32)
    q_hi = np.rint((xv * inv_hi[:, None]).astype(np.float32)).astype(np.int32)
    q_lo = np.rint((xv * inv_lo[:, None]).astype(np.float32)).astype(np.int32)
    assert np.array_equal(np.where(flags, 0, q_lo), unpack_int4(enc.d_lo).astype(np.int32))
    assert np.array_equal(np.where(flags, q_hi, 0), dense_hi(enc))
    assert np.array_equal(enc.s_hi, (amax_hi / np.float32(127.0)).astype(np.float32))
    assert np.array_equal(enc.s_lo, (amax_lo / np.float32(7.0)).astype(np.float32))


def test_equivalent_bits_match_paper_table():
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "equivalent_bits_table3.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) == 14
    for hh, hl, s, y in rows:
        assert oracle.equivalent_bits(float(hh), float(hl), float(s)) == pytest.approx(float(y), abs=1e-12)
    # the layout stored here keeps the low part dense and adds an explicit mask bit
    assert oracle.stored_bits(8, 4, 0.875) == 6.0


def test_static_mask_storage_matches_paper_figure():
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "static_mask_storage.txt")
    layers, hidden, inter, printed = [l.split() for l in open(path) if l.strip() and not l.startswith("#")][0]
    channels = (6 * int(hidden) + int(inter)) * int(layers)
    assert round(channels / 2 ** 20, 2) == float(printed)  # one byte per input channel per linear layer

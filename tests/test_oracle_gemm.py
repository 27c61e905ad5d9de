"""Pins for the oracle's integer products, epilogue and static-mask calibrator.

The products are checked against numpy's int64 matmul of independently unpacked
operands, against one-hot weights that read the encoding back, and against the two
reductions to a textbook quantised matmul (k = b: plain per-token W4A8; emptied high
part: plain W4A4).  The epilogue is checked against an fp64 evaluation.
"""
import numpy as np
import pytest

import oracle
from workloads import f32_to_bf16_bits, bf16_bits_to_f32, pack_int4, unpack_int4, make
from test_oracle_encode import dense_hi, mask_flags


def small_case(seed, M=9, K=256, N=37, b=64, k=8):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[:, rng.choice(K, 4, replace=False)] *= 25.0
    w = rng.integers(-8, 8, size=(N, K)).astype(np.int8)
    sw = rng.uniform(0.005, 0.02, N).astype(np.float32)
    return f32_to_bf16_bits(x), w, sw


@pytest.mark.parametrize("b,k", [(32, 4), (64, 8), (64, 16), (128, 8)])
def test_products_match_numpy_int64_matmul(b, k):
    bits, w, sw = small_case(3 + b + k, b=b, k=k)
    enc = oracle.encode(bits, b, k)
    out = oracle.gemm(enc, pack_int4(w), sw)
    D = unpack_int4(enc.d_lo).astype(np.int64)
    H = dense_hi(enc).astype(np.int64)
    W = w.astype(np.int64)
    assert np.array_equal(out.acc_lo.astype(np.int64), D @ W.T)
    assert np.array_equal(out.acc_hi.astype(np.int64), H @ W.T)


def test_one_hot_weights_read_the_encoding_back():
    bits, _, _ = small_case(11, M=5, K=128, N=128)
    w = np.eye(128, dtype=np.int8)  # row n picks channel n
    enc = oracle.encode(bits, 64, 8)
    out = oracle.gemm(enc, pack_int4(w), np.ones(128, np.float32))
    assert np.array_equal(out.acc_lo, unpack_int4(enc.d_lo).astype(np.int32))
    assert np.array_equal(out.acc_hi, dense_hi(enc))


def test_linearity_in_weights():
    bits, w, sw = small_case(21)
    w1 = np.clip(w, -4, 3)
    w2 = (w - w1).astype(np.int8)
    assert w2.min() >= -8 and w2.max() <= 7
    enc = oracle.encode(bits, 64, 8)
    a = oracle.gemm(enc, pack_int4(w), sw)
    a1 = oracle.gemm(enc, pack_int4(w1), sw)
    a2 = oracle.gemm(enc, pack_int4(w2), sw)
    assert np.array_equal(a.acc_lo, a1.acc_lo + a2.acc_lo)
    assert np.array_equal(a.acc_hi, a1.acc_hi + a2.acc_hi)


def test_all_high_reduces_to_plain_w4a8():
    bits, w, sw = small_case(31, K=128, b=64)
    enc = oracle.encode(bits, 64, 64)  # k == b
    out = oracle.gemm(enc, pack_int4(w), sw)
    xv = bf16_bits_to_f32(bits)
    amax = np.abs(xv).max(1).astype(np.float32)
    q = np.rint((xv * (np.float32(127.0) / amax)[:, None]).astype(np.float32)).astype(np.int64)
    assert not out.acc_lo.any()
    assert np.array_equal(out.acc_hi.astype(np.int64), q @ w.astype(np.int64).T)
    y = (q @ w.astype(np.int64).T) * (amax.astype(np.float64) / 127.0)[:, None] * sw.astype(np.float64)[None, :]
    assert np.allclose(out.y64, y, rtol=1e-6, atol=0)


def test_emptied_high_part_reduces_to_plain_w4a4():
    bits, w, sw = small_case(41)
    enc = oracle.encode(bits, 64, 8)
    enc.hi_val[:] = 0
    out = oracle.gemm(enc, pack_int4(w), sw)
    assert not out.acc_hi.any()
    D = unpack_int4(enc.d_lo).astype(np.int64)
    assert np.array_equal(out.acc_lo.astype(np.int64), D @ w.astype(np.int64).T)
    y = (D @ w.astype(np.int64).T) * enc.s_lo.astype(np.float64)[:, None] * sw.astype(np.float64)[None, :]
    assert np.allclose(out.y32, y, rtol=1e-6, atol=0)


def test_epilogue_against_fp64_and_bf16_rounding():
    bits, w, sw = small_case(51, M=16, K=512, N=64)
    enc = oracle.encode(bits, 64, 8)
    out = oracle.gemm(enc, pack_int4(w), sw)
    want = (out.acc_lo.astype(np.float64) * enc.s_lo.astype(np.float64)[:, None]
            + out.acc_hi.astype(np.float64) * enc.s_hi.astype(np.float64)[:, None]) * sw.astype(np.float64)[None, :]
    assert np.array_equal(out.y64, want)
    # cancellation-safe relative error of the fp32 evaluation: three fp32 roundings
    denom = (np.abs(out.acc_lo * enc.s_lo.astype(np.float64)[:, None])
             + np.abs(out.acc_hi * enc.s_hi.astype(np.float64)[:, None])) * np.abs(sw.astype(np.float64))[None, :]
    err = np.abs(out.y32.astype(np.float64) - want)
    assert (err <= 1e-6 * np.maximum(np.abs(want), denom * 2.0 ** -20) + 1e-300).all() or (err <= 3 * 2.0 ** -24 * denom).all()
    assert np.array_equal(out.ybf16, f32_to_bf16_bits(out.y32))


def test_the_layer_approximates_the_real_product():
    """End to end sanity: the dequantised output is close to X @ (s_w * Wq)^T in fp64."""
    wl = make("c1_tiny")
    enc = oracle.encode(wl.x_bits, wl.bank, wl.topk)
    out = oracle.gemm(enc, wl.wq_packed, wl.w_scale)
    X = bf16_bits_to_f32(wl.x_bits).astype(np.float64)
    W = unpack_int4(wl.wq_packed).astype(np.float64) * wl.w_scale.astype(np.float64)[:, None]
    ref = X @ W.T
    rel = np.linalg.norm(out.y64 - ref) / np.linalg.norm(ref)
    assert rel < 0.05
    # and the high-precision part matters: dropping it is much worse
    enc0 = oracle.encode(wl.x_bits, wl.bank, wl.topk)
    enc0.hi_val[:] = 0
    rel0 = np.linalg.norm(oracle.gemm(enc0, wl.wq_packed, wl.w_scale).y64 - ref) / np.linalg.norm(ref)
    assert rel0 > 5 * rel


def test_static_mask_hand_built_bank():
    # One bank of 8 channels, k = 2, two calibration tokens, two output channels with scale 1.
    #  mean|A|  = [1, 2, 3, 4, 1, 1, 2, 0.5]
    #  col sums = [4,-3, 1, 0, 5,-5, 2.5->int, ..] chosen as small integers below
    A = np.array([[1, -2, 3, 4, 1, -1, 2, 0.5],
                  [-1, 2, -3, -4, 1, 1, -2, 0.5]], np.float32)
    W = np.array([[3, -1, 1, 0, 2, -2, 1, 7],
                  [1, -2, 0, 0, 3, -3, 2, 1]], np.int8)
    # I = |mean|A| * colsum| = [4, 6, 3, 0, 5, 5, 6, 4] -> top-2: channel 1 and 6 (6, 6)
    K = 32
    Ab = np.zeros((2, K), np.float32); Ab[:, :8] = A
    Wb = np.zeros((2, K), np.int8); Wb[:, :8] = W
    mask, imp = oracle.static_mask(f32_to_bf16_bits(Ab), pack_int4(Wb), np.ones(2, np.float32), 8, 2)
    assert list(imp[:8]) == [4, 6, 3, 0, 5, 5, 6, 4]
    assert (int(mask[0]) & 0xFF) == (1 << 1) | (1 << 6)
    # the other banks are all-zero importance: ties -> the first two channels of each bank
    assert (int(mask[0]) >> 8) & 0xFF == 0b11
    # tie between channels 4 and 5 (I = 5) at the boundary with k = 3 -> lower index 4 wins
    mask3, _ = oracle.static_mask(f32_to_bf16_bits(Ab), pack_int4(Wb), np.ones(2, np.float32), 8, 3)
    assert (int(mask3[0]) & 0xFF) == (1 << 1) | (1 << 6) | (1 << 4)


def test_static_mask_finds_outlier_channels():
    wl = make("c4_down7b_static", M=8, N=64)
    mask, imp = oracle.static_mask(wl.calib_bits, wl.wq_packed, wl.w_scale, wl.bank, wl.topk)
    flags = ((mask[:, None] >> np.arange(32, dtype=np.uint32)[None, :]) & 1).reshape(-1).astype(bool)
    assert (flags.reshape(-1, wl.bank).sum(1) == wl.topk).all()
    # outlier channels are x20-50 larger: nearly all must be selected (a channel can only miss
    # if its weight column sum happens to be ~0 or its bank holds more than k outliers)
    assert flags[wl.outlier_channels].mean() > 0.9
    enc = oracle.encode(wl.x_bits, wl.bank, wl.topk, static_mask=mask)
    out = oracle.gemm(enc, wl.wq_packed, wl.w_scale)
    D = unpack_int4(enc.d_lo).astype(np.int64)
    H = dense_hi(enc).astype(np.int64)
    Wi = unpack_int4(wl.wq_packed).astype(np.int64)
    assert np.array_equal(out.acc_lo, D @ Wi.T) and np.array_equal(out.acc_hi, H @ Wi.T)


def test_bf16_output_rounding_hand_computed_patterns():
    """The bf16 output is round-half-to-even of the fp32 output.  Each row's output is made to be a chosen
    fp32 bit pattern (accumulator 1 x per-token scale = that value, weight scale 1); the expected bf16
    patterns below are worked out by hand from the definition: keep the upper 16 bits, look at the lower 16;
    above 0x8000 round up, below round down, exactly 0x8000 round to the even upper half."""
    cases = [
        (0x3F808000, 0x3F80),  # 1 + 2^-8: half-way, 0x3F80 is even -> stays
        (0x3F818000, 0x3F82),  # 1 + 3*2^-8: half-way, 0x3F81 is odd -> up
        (0x3F808001, 0x3F81),  # just above half-way -> up
        (0x3F807FFF, 0x3F80),  # just below half-way -> down
        (0xBF808000, 0xBF80),  # the same magnitudes, negative (sign-magnitude: rounding is symmetric)
        (0xBF818000, 0xBF82),
        (0x3FFF8000, 0x4000),  # half-way with an odd, all-ones mantissa: the carry runs into the exponent -> 2.0
        (0x3FFFFFFF, 0x4000),  # just under 2.0 -> 2.0
        (0x3F800000, 0x3F80),  # exactly representable values are untouched
        (0x40490FDB, 0x4049),  # pi -> 3.140625
        (0x00000000, 0x0000),
    ]
    M, K = len(cases), 32
    d = np.zeros((M, K), np.int8)
    d[:, 1] = 1  # one low code of 1 in channel 1 (channel 0 is the bank's high channel, code 0)
    mask = np.zeros((M, 1), np.uint32)
    mask[:, 0] = 1
    s_lo = np.array([c[0] for c in cases], np.uint32).view(np.float32)
    enc = oracle.Encoded(M, K, 32, 1, 0, pack_int4(d), np.zeros((M, 1, 1), np.int8), mask, s_lo.copy(),
                         np.ones(M, np.float32))
    w = np.zeros((1, K), np.int8)
    w[0, 1] = 1
    out = oracle.gemm(enc, pack_int4(w), np.ones(1, np.float32))
    assert np.array_equal(out.acc_lo[:, 0], np.ones(M, np.int32)) and not out.acc_hi.any()
    assert [int(v) for v in out.y32.view(np.uint32)[:, 0]] == [c[0] for c in cases]
    assert [hex(int(v)) for v in out.ybf16[:, 0]] == [hex(c[1]) for c in cases]

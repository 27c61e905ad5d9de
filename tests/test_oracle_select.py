"""Pins for the oracle's per-bank selection (Sections 3.1, 3.2.2, 4.3).

The oracle orders a bank with a stable insertion sort; here the same set is obtained
with an independent k-pass arg-max (scan for the maximum with a strict '>' so the
earliest index wins, remove it, repeat) and by hand for the 2:4 special case.
"""
import numpy as np
import pytest

import oracle
from workloads import f32_to_bf16_bits, bf16_bits_to_f32


def kpass_argmax(mag: np.ndarray, k: int) -> np.ndarray:
    taken = np.zeros(len(mag), dtype=bool)
    for _ in range(k):
        best, best_i = -1.0, -1
        for i, v in enumerate(mag):
            if not taken[i] and v > best:
                best, best_i = v, i
        taken[best_i] = True
    return taken


@pytest.mark.parametrize("b,k", [(4, 2), (16, 4), (32, 2), (32, 8), (64, 8), (64, 4), (64, 16), (128, 16)])
def test_matches_kpass_argmax_random(b, k):
    rng = np.random.default_rng(7 + b * 131 + k)
    for trial in range(40):
        G = 3
        x = rng.standard_normal(G * b).astype(np.float32)
        bits = f32_to_bf16_bits(x)
        got = oracle.select_dynamic(bits, b, k).astype(bool)
        mag = np.abs(bf16_bits_to_f32(bits)).astype(np.float64)
        for g in range(G):
            want = kpass_argmax(mag[g * b:(g + 1) * b], k)
            assert np.array_equal(got[g * b:(g + 1) * b], want), (trial, g)


@pytest.mark.parametrize("b,k", [(8, 3), (32, 4), (64, 8)])
def test_heavy_ties_lowest_index_wins(b, k):
    # values from a 4-element set (both signs): almost every boundary is a tie
    rng = np.random.default_rng(99 + b)
    vals = np.array([0.0, 0.5, 1.0, 2.0], np.float32)
    for trial in range(200):
        x = vals[rng.integers(0, 4, size=b)] * rng.choice([-1.0, 1.0], size=b).astype(np.float32)
        bits = f32_to_bf16_bits(x)
        got = oracle.select_dynamic(bits, b, k).astype(bool)
        want = kpass_argmax(np.abs(x).astype(np.float64), k)
        assert np.array_equal(got, want)
        assert got.sum() == k
        # invariant: nothing left out is strictly larger than something taken
        assert np.abs(x)[got].min() >= np.abs(x)[~got].max()
        # among elements equal to the boundary magnitude the taken ones come first
        t = np.abs(x)[got].min()
        eq = np.flatnonzero(np.abs(x) == t)
        n_taken = got[eq].sum()
        assert got[eq[:n_taken]].all() and not got[eq[n_taken:]].any()


def test_all_equal_takes_first_k():
    bits = f32_to_bf16_bits(np.full(64, -3.0, np.float32))
    got = oracle.select_dynamic(bits, 64, 8)
    assert got[:8].all() and not got[8:].any()


def test_signed_zero_ties():
    x = np.zeros(16, np.float32)
    x[5] = -0.0
    bits = f32_to_bf16_bits(x)
    bits[5] = 0x8000
    got = oracle.select_dynamic(bits, 16, 3)
    assert list(np.flatnonzero(got)) == [0, 1, 2]


def test_two_of_four_special_case():
    # Section 3.1: 2:4 semi-structured sparsity is the case b=4, s=0.5 (h_low = 0):
    # in every group of four the two largest magnitudes survive.  Checked by hand.
    x = np.array([0.1, -0.9, 0.5, 0.2,    # -> idx 1, 2
                  1.0, 1.0, 1.0, 1.0,     # tie -> idx 0, 1
                  -4.0, 0.0, 0.0, 3.0,    # -> idx 0, 3
                  0.0, 0.0, 0.25, 0.0],   # -> idx 2 and the first zero (idx 0)
                 np.float32)
    got = oracle.select_dynamic(f32_to_bf16_bits(x), 4, 2)
    want = [0, 1, 1, 0, 1, 1, 0, 0, 1, 0, 0, 1, 1, 0, 1, 0]
    assert list(got) == want


def test_magnitude_order_uses_absolute_value_not_sign():
    x = np.array([-8.0, 7.0, -6.0, 5.0, 1.0, -1.0, 0.5, 0.25], np.float32)
    got = oracle.select_dynamic(f32_to_bf16_bits(x), 8, 3)
    assert list(np.flatnonzero(got)) == [0, 1, 2]


def test_bad_arguments():
    bits = np.zeros(64, np.uint16)
    with pytest.raises(ValueError):
        oracle.select_dynamic(bits, 48, 4)  # K % b != 0
    with pytest.raises(ValueError):
        oracle.select_dynamic(bits, 64, 0)  # k >= 1

"""CPU oracle for the tied-scale variant of the SQ-format linear layer.   *** TEST INFRASTRUCTURE ***

Plain numpy, fp32 where the layer is fp32, written from the definitions; it shares no code with the
GPU library and is only used by tests and the benchmark's checks.

What it follows (paper "SQ-format: A Unified Sparse-Quantized Hardware-friendly Data Format for LLMs"):
Section 3.1, Eq. (1) (banks, a fixed number of high-precision elements per bank, a mask); Section 3.2.1
(symmetric quantisation); Sections 3.2.2 / 4.3 (dynamic rule: the largest magnitudes of a bank, per token);
Section 3.3 and Section 5.2 (the product is worth splitting only if the low-precision path is cheaper than
the high-precision one).

Reading taken here (the paper gives each part a scale of its own and says nothing about tying them): on
hardware whose only integer matrix path is INT8 the two products of Section 3.3 cost the same, so this
variant ties the two scales of a token, s_lo = 16 * s_hi.  An INT4 low code d then stands for the INT8
value 16 * d on the high part's grid, the whole row becomes ONE INT8 operand
    c[j] = h[j] at the high channels,  16 * d[j] at the low channels,
and the layer needs one integer product and one accumulator:
    acc[m, n] = sum_j c[m, j] * Wq[n, j]            Y[m, n] = (acc * s_hi[m]) * s_w[n].
The stored format is unchanged (INT8 high codes, INT4 low codes, mask; 4.5 bits per element at k/b = 1/8).
Steps, per token row:
  1. selection: exactly as in the two-scale layer (per bank the k largest |x|, ties to the lower channel);
  2. A = max(amax_hi, fl32(amax_lo * fl32(127/112))): the smallest INT8 full-scale value for which neither
     the high codes (|h| <= 127) nor the low codes (|d| <= 7, i.e. 16*7 = 112 grid steps) clip;
     s_hi = fl32(A / 127), inv_hi = fl32(127 / A), s_lo = 16 * s_hi, inv_lo = inv_hi / 16 (both exact);
     A == 0: s_hi = 1, inv = 0;
  3. codes: h = clamp(rne(fl32(x * inv_hi)), +-127), d = clamp(rne(fl32(x * inv_lo)), +-7), d = 0 at the
     high channels; rne = round half to even.
  4. product in exact integers; epilogue t = fl32(float(acc) * s_hi), y = fl32(t * s_w[n]); bf16 = RNE(y).

Pins (tests/test_oracle_tied.py): hand-built rows with scale 1 and exact half-way cases, the row where the
low part sets the scale, s_lo == 16*s_hi bit for bit, agreement of the mask with the two-scale oracle's
(same rule), numpy int64 matmul, the identity acc == 16*acc_lo + acc_hi with the two-accumulator oracle run
on the same codes, k = b (plain per-token INT8), fp64 epilogue, and planted mistakes.
Parity unpinned: the paper prints no worked example, and this variant is a reading, not the paper's text.
"""
from __future__ import annotations

import numpy as np

from . import select_dynamic

F32 = np.float32


class EncodedTied:
    """SQ-format with tied scales: the usual arrays plus the combined INT8 codes of every channel."""

    def __init__(self, M, K, bank, topk, d_lo, hi_val, mask, s_lo, s_hi, codes):
        self.M, self.K, self.bank, self.topk, self.mode = M, K, bank, topk, 0
        self.d_lo, self.hi_val, self.mask, self.s_lo, self.s_hi, self.codes = d_lo, hi_val, mask, s_lo, s_hi, codes


def _bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rne_bf16(y: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(y, dtype=np.float32).view(np.uint32)
    keep = u >> np.uint32(16)
    rest = u & np.uint32(0xFFFF)
    up = (rest > 0x8000) | ((rest == 0x8000) & ((keep & np.uint32(1)) == 1))
    return (keep + up.astype(np.uint32)).astype(np.uint16)


def encode_tied(x_bits: np.ndarray, bank: int, topk: int) -> EncodedTied:
    x_bits = np.ascontiguousarray(x_bits, dtype=np.uint16)
    M, K = x_bits.shape
    assert K % bank == 0 and K % 32 == 0 and 1 <= topk <= bank
    G = K // bank
    x = _bf16_to_f32(x_bits)
    mag = np.abs(x)
    d_lo = np.zeros((M, K // 2), np.uint8)
    hi_val = np.zeros((M, G, topk), np.int8)
    mask = np.zeros((M, K // 32), np.uint32)
    s_lo = np.zeros(M, F32)
    s_hi = np.zeros(M, F32)
    codes = np.zeros((M, K), np.int8)
    for m in range(M):
        is_hi = select_dynamic(x_bits[m], bank, topk).astype(bool)                 # step 1
        amax_hi = F32(mag[m][is_hi].max()) if is_hi.any() else F32(0)
        amax_lo = F32(mag[m][~is_hi].max()) if (~is_hi).any() else F32(0)
        A = max(amax_hi, F32(amax_lo * (F32(127.0) / F32(112.0))))                 # step 2
        if A == 0:
            sc_hi, inv_hi = F32(1.0), F32(0.0)
        else:
            sc_hi, inv_hi = F32(A / F32(127.0)), F32(F32(127.0) / A)
        sc_lo, inv_lo = F32(sc_hi * F32(16.0)), F32(inv_hi * F32(0.0625))
        s_hi[m], s_lo[m] = sc_hi, sc_lo
        h = np.clip(np.rint((x[m] * inv_hi).astype(F32)), -127, 127).astype(np.int32)   # step 3
        d = np.clip(np.rint((x[m] * inv_lo).astype(F32)), -7, 7).astype(np.int32)
        d[is_hi] = 0
        codes[m] = np.where(is_hi, h, 16 * d).astype(np.int8)
        hi_val[m] = h[is_hi].reshape(G, topk)  # ascending channel order inside each bank
        d_lo[m] = ((d[0::2] & 0xF) | ((d[1::2] & 0xF) << 4)).astype(np.uint8)
        bits = is_hi.reshape(K // 32, 32).astype(np.uint64) << np.arange(32, dtype=np.uint64)[None, :]
        mask[m] = bits.sum(1).astype(np.uint32)
    return EncodedTied(M, K, bank, topk, d_lo, hi_val, mask, s_lo, s_hi, codes)


class ProductTied:
    def __init__(self, acc, y32, ybf16, y64):
        self.acc, self.y32, self.ybf16, self.y64 = acc, y32, ybf16, y64


def _unpack_weights(wq_packed: np.ndarray) -> np.ndarray:
    p = np.ascontiguousarray(wq_packed, dtype=np.uint8)
    w = np.empty((p.shape[0], p.shape[1] * 2), np.int64)
    lo, hi = (p & 0xF).astype(np.int64), (p >> 4).astype(np.int64)
    w[:, 0::2] = np.where(lo >= 8, lo - 16, lo)
    w[:, 1::2] = np.where(hi >= 8, hi - 16, hi)
    return w


def gemm_tied(enc: EncodedTied, wq_packed: np.ndarray, w_scale: np.ndarray) -> ProductTied:
    W = _unpack_weights(wq_packed)
    sw = np.ascontiguousarray(w_scale, dtype=F32)
    acc64 = enc.codes.astype(np.int64) @ W.T                                         # step 4
    assert np.abs(acc64).max(initial=0) < 2 ** 31
    acc = acc64.astype(np.int32)
    t = (acc.astype(F32) * enc.s_hi[:, None]).astype(F32)
    y32 = (t * sw[None, :]).astype(F32)
    y64 = acc64.astype(np.float64) * enc.s_hi.astype(np.float64)[:, None] * sw.astype(np.float64)[None, :]
    return ProductTied(acc, y32, _rne_bf16(y32), y64)

"""CPU oracle for SQ-format on WEIGHTS at run time (W(SQ)A8 / W(SQ)A4 linear layer).   *** TEST INFRASTRUCTURE ***

Plain numpy, written from the definitions; shares no code with the GPU library.

What it follows (paper "SQ-format: A Unified Sparse-Quantized Hardware-friendly Data Format for LLMs"):
Section 3.2.1 and Algorithm 1 (a weight matrix is represented by a high- and a low-precision part; inside every
bank the top (1-s) fraction of the weights of a column, ranked by the importance I = W'^2 / diag(H^-1)^2, is kept
in high precision; symmetric quantisation; the high part is stored compactly, the low part in its original
shape with the unused code v_mask at the high positions), its Figure 1 caption (every column of every bank is
quantised as a group of its own: one scale for its high part, one for its low part), Section 3.3 (the product
splits into a dense low-precision part and a sparse high-precision part), Section 4.1 (W(SQx)Ay: the other
operand, the activation, is plain INTy).

Conventions here: W is held as [N, K] (row n = output channel n = a "column" of the paper's K x N matrix), a bank
is b consecutive input channels of one output channel, G = K / b banks per row.
Readings where the paper is silent:
  - the smoothed weights W' and the Hessian come from calibration, which is out of scope: the layer takes the
    weights as given and an optional positive vector d[K] = diag(H^-1); importance I = fl32(fl32(w*w) / fl32(d*d)),
    ties to the lower channel; d = None means d = 1 (ranking by |w|);
  - scales per (n, bank) group: s_hi = amax_hi / Q_hi, s_lo = amax_lo / Q_lo (amax over the group's high / low
    weights; 1 when that part is all zero), codes rne(fl32(w * fl32(Q / amax))) clamped to +-Q, Q = 2^(h-1) - 1;
  - v_mask = -2^(h_low-1), the one code the symmetric low range leaves unused (as in the activation storage);
  - activations: plain per-token symmetric INT8 (or INT4): s_a = amax_row / Q_a, code rne(fl32(x * fl32(Q_a/amax)));
  - the integer products of one bank are exact; they are dequantised and added bank by bank in fp32, in this order:
        f = 0;  for g in banks:  t = fl(float(acc_lo_g) * s_lo[n,g]);  t = fma(float(acc_hi_g), s_hi[n,g], t);
                                 f = fl(f + t);          y = fl(f * s_a[m]);   bf16 output = RNE(y).
Pins (tests/test_oracle_wsq.py): hand-built groups (scale 1, half-way cases, a tie in importance, the effect of
d), invariants (exactly k high per group, sentinel exactly at the high positions, code ranges, reconstruction
within half a step), per-bank integer products against numpy, the fp64 evaluation of the sum, k = b (plain
per-group INT8 weights), and planted mistakes.
Parity unpinned: the paper prints no worked example (its Figure 1 is not in the text).
"""
from __future__ import annotations

import numpy as np

F32 = np.float32


def qmax(bits: int) -> int:
    return (1 << (bits - 1)) - 1


class WeightSQ:
    """lo: [N, K] int8 low codes with v_mask at the high positions; hi_val: [N, G, k] int8 (ascending channel);
    s_lo, s_hi: [N, G] fp32."""

    def __init__(self, N, K, bank, topk, h_high, h_low, lo, hi_val, s_lo, s_hi):
        self.N, self.K, self.bank, self.topk, self.h_high, self.h_low = N, K, bank, topk, h_high, h_low
        self.lo, self.hi_val, self.s_lo, self.s_hi = lo, hi_val, s_lo, s_hi

    @property
    def v_mask(self):
        return -(1 << (self.h_low - 1))

    def is_hi(self):
        return self.lo == self.v_mask

    def dense_hi(self):
        H = np.zeros((self.N, self.K), np.int32)
        flags = self.is_hi()
        for n in range(self.N):
            H[n, flags[n]] = self.hi_val[n].reshape(-1)
        return H

    def dense_lo(self):
        return np.where(self.is_hi(), 0, self.lo).astype(np.int32)


def encode_weights(w_bits: np.ndarray, bank: int, topk: int, h_high: int = 8, h_low: int = 4, d=None) -> WeightSQ:
    w_bits = np.ascontiguousarray(w_bits, dtype=np.uint16)
    N, K = w_bits.shape
    assert K % bank == 0 and 1 <= topk <= bank
    G = K // bank
    w = (w_bits.astype(np.uint32) << np.uint32(16)).view(np.float32)
    dd = np.ones(K, F32) if d is None else np.ascontiguousarray(d, dtype=F32)
    imp = ((w * w).astype(F32) / (dd * dd).astype(F32)[None, :]).astype(F32)
    q_hi, q_lo = F32(qmax(h_high)), F32(qmax(h_low))
    v_mask = -(1 << (h_low - 1))
    lo = np.zeros((N, K), np.int8)
    hi_val = np.zeros((N, G, topk), np.int8)
    s_lo, s_hi = np.ones((N, G), F32), np.ones((N, G), F32)
    for n in range(N):
        for g in range(G):
            sl = slice(g * bank, (g + 1) * bank)
            order = sorted(range(bank), key=lambda i: (-float(imp[n, sl][i]), i))  # importance descending, index ascending
            hi = np.zeros(bank, bool)
            hi[order[:topk]] = True
            wg = w[n, sl]
            a_hi = F32(np.abs(wg[hi]).max()) if hi.any() else F32(0)
            a_lo = F32(np.abs(wg[~hi]).max()) if (~hi).any() else F32(0)
            inv_hi = F32(q_hi / a_hi) if a_hi != 0 else F32(0)
            inv_lo = F32(q_lo / a_lo) if a_lo != 0 else F32(0)
            s_hi[n, g] = F32(a_hi / q_hi) if a_hi != 0 else F32(1)
            s_lo[n, g] = F32(a_lo / q_lo) if a_lo != 0 else F32(1)
            ch = np.clip(np.rint((wg * inv_hi).astype(F32)), -q_hi, q_hi).astype(np.int32)
            cl = np.clip(np.rint((wg * inv_lo).astype(F32)), -q_lo, q_lo).astype(np.int32)
            lo[n, sl] = np.where(hi, v_mask, cl)
            hi_val[n, g] = ch[hi]
    return WeightSQ(N, K, bank, topk, h_high, h_low, lo, hi_val, s_lo, s_hi)


def quantize_activations(x_bits: np.ndarray, bits: int = 8):
    """Plain per-token symmetric quantisation -> (codes [M, K] int8, scale [M] fp32)."""
    x = (np.ascontiguousarray(x_bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)
    q = F32(qmax(bits))
    amax = np.abs(x).max(1).astype(F32)
    nz = amax != 0
    inv = np.where(nz, q / np.where(nz, amax, 1), 0).astype(F32)
    scale = np.where(nz, amax / q, 1).astype(F32)
    codes = np.clip(np.rint((x * inv[:, None]).astype(F32)), -q, q).astype(np.int8)
    return codes, scale


class WsqProduct:
    def __init__(self, acc_lo, acc_hi, y32, ybf16, y64):
        self.acc_lo, self.acc_hi, self.y32, self.ybf16, self.y64 = acc_lo, acc_hi, y32, ybf16, y64


def _fma32(a: np.ndarray, b: np.ndarray, c: np.ndarray) -> np.ndarray:
    """fl32(a*b + c) with a single rounding (the C library's fmaf)."""
    from . import fma32
    return fma32(a, b, c)


def gemm(a_codes: np.ndarray, a_scale: np.ndarray, wsq: WeightSQ) -> WsqProduct:
    """acc_lo / acc_hi: [M, N, G] per-bank integer products; y: the bank-by-bank fp32 evaluation."""
    A = a_codes.astype(np.int64)
    M, K = A.shape
    G, b = wsq.K // wsq.bank, wsq.bank
    L, H = wsq.dense_lo().astype(np.int64), wsq.dense_hi().astype(np.int64)
    acc_lo = np.zeros((M, wsq.N, G), np.int64)
    acc_hi = np.zeros((M, wsq.N, G), np.int64)
    f = np.zeros((M, wsq.N), F32)
    f64 = np.zeros((M, wsq.N), np.float64)
    for g in range(G):
        sl = slice(g * b, (g + 1) * b)
        acc_lo[:, :, g] = A[:, sl] @ L[:, sl].T
        acc_hi[:, :, g] = A[:, sl] @ H[:, sl].T
        t = (acc_lo[:, :, g].astype(F32) * wsq.s_lo[None, :, g]).astype(F32)
        t = _fma32(acc_hi[:, :, g].astype(F32), np.broadcast_to(wsq.s_hi[None, :, g], t.shape), t)
        f = (f + t).astype(F32)
        f64 += acc_lo[:, :, g] * wsq.s_lo[None, :, g].astype(np.float64) + acc_hi[:, :, g] * wsq.s_hi[None, :, g].astype(np.float64)
    y32 = (f * a_scale.astype(F32)[:, None]).astype(F32)
    u = y32.view(np.uint32)
    keep, rest = u >> np.uint32(16), u & np.uint32(0xFFFF)
    up = (rest > 0x8000) | ((rest == 0x8000) & ((keep & np.uint32(1)) == 1))
    ybf16 = (keep + up.astype(np.uint32)).astype(np.uint16)
    return WsqProduct(acc_lo.astype(np.int32), acc_hi.astype(np.int32), y32, ybf16, f64 * a_scale.astype(np.float64)[:, None])

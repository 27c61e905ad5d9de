"""CPU oracle for the other precision pairs of the SQ-format and for its bit-packed storage.   *** TEST INFRASTRUCTURE ***

Plain numpy, written from the definitions; shares no code with the GPU library.

What it follows (paper "SQ-format: A Unified Sparse-Quantized Hardware-friendly Data Format for LLMs"):
Section 4.1 (Notation: a setting is B-(h_high/h_low)-s; an activation in SQ-format costs
y = (1-s)*h_high + s*h_low bits per element), Section 5.1 and Table 3 (the pairs (8/3), (8/2), (4/2) beside
(8/4)), Section 3.2.1 (symmetric quantisation; the INT2 example uses the codes -1, 0, 1), Section 3.1 Eq. (1).

encode_pair: the two-scale encoding with code ranges Q_hi = 2^(h_high-1) - 1 and Q_lo = 2^(h_low-1) - 1
(127 / 7 / 3 / 1), everything else as in the (8/4) layer: per-bank top-k by |x| (ties to the lower channel) or
a static channel mask, per-token scales amax/Q, codes rne(fl32(x * fl32(Q/amax))) clamped to +-Q.  The codes are
returned in the same containers as the (8/4) layer (INT8 high codes, 4-bit two's complement low codes), so the
products of Section 3.3 are those of the pinned C oracle, unchanged.

pack_storage / unpack_storage: the format at its equivalent bit width.  Reading (the paper gives the bit count,
not a layout): per token row, the high codes of the high channels at h_high bits each, then the low codes of
the LOW channels only at h_low bits each, both in ascending channel order, as one little-endian bit stream per
section (code t occupies bits [t*h, (t+1)*h) of its section; bit i of a section is bit i%8 of its byte i/8;
h-bit two's complement).  Row size = K * y / 8 bytes exactly; the mask and the two scales are stored beside it.

pack_storage_sentinel / unpack_storage_sentinel: the implicit-mask form of Section 3.1 / Section 3.2.1 ("the unused
largest value of the low-precision format is considered as a high-precision mask"): the low section covers ALL K
channels and holds, at the high channels, the code the symmetric range leaves unused, v_mask = -2^(h_low-1)
(bit pattern 10 = 2 for INT2, as in the paper's example; for INT4 the pattern is 1000 -- the figure caption's
"15" does not fit two's complement, reading taken: the one consistent with the INT2 example); no mask is stored,
unpacking recovers it from the sentinels.  Row size = K * x / 8 bytes with x = (1-s)*h_high + h_low, the
formula Section 4.1 gives for this form.

Pins (tests/test_oracle_pairs.py): for (8/4) encode_pair must equal the pinned C oracle bit for bit; hand-built
rows with scale 1 for Q = 3 and Q = 1 including half-way cases; code ranges; storage size against the y column
of the paper's Table 3 (tests/golden); pack/unpack round trip and a hand-packed 3-bit example; planted mistakes.
Parity unpinned: no worked example of these pairs is printed in the paper.
"""
from __future__ import annotations

import numpy as np

from . import Encoded, select_dynamic

F32 = np.float32


def qmax(bits: int) -> int:
    """Largest code magnitude of a symmetric h-bit integer format (Section 3.2.1)."""
    return (1 << (bits - 1)) - 1


def encode_pair(x_bits: np.ndarray, bank: int, topk: int, h_high: int, h_low: int, static_mask=None) -> Encoded:
    x_bits = np.ascontiguousarray(x_bits, dtype=np.uint16)
    M, K = x_bits.shape
    assert K % bank == 0 and K % 32 == 0 and 1 <= topk <= bank and 2 <= h_low <= 4 and h_low < h_high <= 8
    G = K // bank
    q_hi, q_lo = F32(qmax(h_high)), F32(qmax(h_low))
    x = (x_bits.astype(np.uint32) << np.uint32(16)).view(np.float32)
    mag = np.abs(x)
    d_lo = np.zeros((M, K // 2), np.uint8)
    hi_val = np.zeros((M, G, topk), np.int8)
    s_lo, s_hi = np.zeros(M, F32), np.zeros(M, F32)
    if static_mask is None:
        mask = np.zeros((M, K // 32), np.uint32)
    else:
        mask = np.ascontiguousarray(static_mask, dtype=np.uint32)
        static_hi = ((mask[:, None] >> np.arange(32, dtype=np.uint32)[None, :]) & 1).reshape(-1).astype(bool)
    for m in range(M):
        is_hi = select_dynamic(x_bits[m], bank, topk).astype(bool) if static_mask is None else static_hi
        amax_hi = F32(mag[m][is_hi].max()) if is_hi.any() else F32(0)
        amax_lo = F32(mag[m][~is_hi].max()) if (~is_hi).any() else F32(0)
        sc_hi, inv_hi = (F32(amax_hi / q_hi), F32(q_hi / amax_hi)) if amax_hi != 0 else (F32(1), F32(0))
        sc_lo, inv_lo = (F32(amax_lo / q_lo), F32(q_lo / amax_lo)) if amax_lo != 0 else (F32(1), F32(0))
        s_hi[m], s_lo[m] = sc_hi, sc_lo
        h = np.clip(np.rint((x[m] * inv_hi).astype(F32)), -q_hi, q_hi).astype(np.int32)
        d = np.clip(np.rint((x[m] * inv_lo).astype(F32)), -q_lo, q_lo).astype(np.int32)
        d[is_hi] = 0
        hi_val[m] = h[is_hi].reshape(G, topk)
        d_lo[m] = ((d[0::2] & 0xF) | ((d[1::2] & 0xF) << 4)).astype(np.uint8)
        if static_mask is None:
            bits = is_hi.reshape(K // 32, 32).astype(np.uint64) << np.arange(32, dtype=np.uint64)[None, :]
            mask[m] = bits.sum(1).astype(np.uint32)
    return Encoded(M, K, bank, topk, 0 if static_mask is None else 1, d_lo, hi_val, mask, s_lo, s_hi)


def storage_row_bytes(K: int, bank: int, topk: int, h_high: int, h_low: int) -> int:
    k_hi = K // bank * topk
    return (k_hi * h_high + (K - k_hi) * h_low) // 8


def _flags(enc: Encoded) -> np.ndarray:
    m = enc.mask if enc.mode == 0 else np.broadcast_to(enc.mask[None, :], (enc.M, enc.K // 32))
    return ((m[:, :, None] >> np.arange(32, dtype=np.uint32)[None, None, :]) & 1).reshape(enc.M, enc.K).astype(bool)


def _low_codes(enc: Encoded) -> np.ndarray:
    p = enc.d_lo
    lo, hi = (p & 0xF).astype(np.int32), (p >> 4).astype(np.int32)
    d = np.empty((enc.M, enc.K), np.int32)
    d[:, 0::2] = np.where(lo >= 8, lo - 16, lo)
    d[:, 1::2] = np.where(hi >= 8, hi - 16, hi)
    return d


def _pack_section(codes: np.ndarray, h: int) -> np.ndarray:
    """[n] integer codes -> little-endian bit stream of n*h bits (n*h a multiple of 8)."""
    u = (codes.astype(np.int64) & ((1 << h) - 1)).astype(np.uint8)
    bits = ((u[:, None] >> np.arange(h, dtype=np.uint8)[None, :]) & 1).reshape(-1)
    return np.packbits(bits, bitorder="little")


def _unpack_section(stream: np.ndarray, n: int, h: int) -> np.ndarray:
    bits = np.unpackbits(stream, bitorder="little")[: n * h].reshape(n, h).astype(np.int32)
    u = (bits << np.arange(h, dtype=np.int32)[None, :]).sum(1)
    return np.where(u >= (1 << (h - 1)), u - (1 << h), u)


def pack_storage(enc: Encoded, h_high: int, h_low: int) -> np.ndarray:
    """-> [M, K*y/8] bytes: per row the high section, then the low section (see the module header)."""
    flags = _flags(enc)
    d = _low_codes(enc)
    out = np.zeros((enc.M, storage_row_bytes(enc.K, enc.bank, enc.topk, h_high, h_low)), np.uint8)
    for m in range(enc.M):
        hs = _pack_section(enc.hi_val[m].reshape(-1), h_high)
        ls = _pack_section(d[m][~flags[m]], h_low)
        out[m, : len(hs)] = hs
        out[m, len(hs):] = ls
    return out


def sentinel_row_bytes(K: int, bank: int, topk: int, h_high: int, h_low: int) -> int:
    return (K // bank * topk * h_high + K * h_low) // 8


def pack_storage_sentinel(enc: Encoded, h_high: int, h_low: int) -> np.ndarray:
    """-> [M, K*x/8] bytes: high section, then K low codes with v_mask = -2^(h_low-1) at the high channels."""
    flags = _flags(enc)
    d = _low_codes(enc)
    v_mask = -(1 << (h_low - 1))
    out = np.zeros((enc.M, sentinel_row_bytes(enc.K, enc.bank, enc.topk, h_high, h_low)), np.uint8)
    for m in range(enc.M):
        hs = _pack_section(enc.hi_val[m].reshape(-1), h_high)
        ls = _pack_section(np.where(flags[m], v_mask, d[m]), h_low)
        out[m, : len(hs)] = hs
        out[m, len(hs):] = ls
    return out


def unpack_storage_sentinel(packed: np.ndarray, K: int, bank: int, topk: int, h_high: int, h_low: int,
                            s_lo: np.ndarray, s_hi: np.ndarray) -> Encoded:
    """The inverse; the (per-row) mask comes out of the sentinels."""
    M = packed.shape[0]
    G = K // bank
    k_hi = G * topk
    nh = k_hi * h_high // 8
    v_mask = -(1 << (h_low - 1))
    d_lo = np.zeros((M, K // 2), np.uint8)
    hi_val = np.zeros((M, G, topk), np.int8)
    mask = np.zeros((M, K // 32), np.uint32)
    for m in range(M):
        hi_val[m] = _unpack_section(packed[m, :nh], k_hi, h_high).reshape(G, topk)
        d = _unpack_section(packed[m, nh:], K, h_low)
        is_hi = d == v_mask
        d = np.where(is_hi, 0, d)
        d_lo[m] = ((d[0::2] & 0xF) | ((d[1::2] & 0xF) << 4)).astype(np.uint8)
        bits = is_hi.reshape(K // 32, 32).astype(np.uint64) << np.arange(32, dtype=np.uint64)[None, :]
        mask[m] = bits.sum(1).astype(np.uint32)
    return Encoded(M, K, bank, topk, 0, d_lo, hi_val, mask, s_lo, s_hi)


def unpack_storage(packed: np.ndarray, mask: np.ndarray, K: int, bank: int, topk: int, h_high: int, h_low: int,
                   s_lo: np.ndarray, s_hi: np.ndarray, static: bool = False) -> Encoded:
    M = packed.shape[0]
    G = K // bank
    k_hi = G * topk
    tmp = Encoded(M, K, bank, topk, 1 if static else 0, None, None, mask, s_lo, s_hi)
    flags = _flags(tmp)
    d_lo = np.zeros((M, K // 2), np.uint8)
    hi_val = np.zeros((M, G, topk), np.int8)
    nh = k_hi * h_high // 8
    for m in range(M):
        hi_val[m] = _unpack_section(packed[m, :nh], k_hi, h_high).reshape(G, topk)
        d = np.zeros(K, np.int32)
        d[~flags[m]] = _unpack_section(packed[m, nh:], K - k_hi, h_low)
        d_lo[m] = ((d[0::2] & 0xF) | ((d[1::2] & 0xF) << 4)).astype(np.uint8)
    return Encoded(M, K, bank, topk, tmp.mode, d_lo, hi_val, mask, s_lo, s_hi)

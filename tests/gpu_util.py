"""Helpers for the GPU parity tests: host<->device copies with guard bytes, and the comparison rules."""
from __future__ import annotations

import numpy as np
import torch

import paper_2512_05409_amd as sq

GUARD = 256  # bytes of canary on each side of an output buffer
CANARY = 0xA5


def dev(a: np.ndarray) -> torch.Tensor:
    """Host array -> device tensor of the same bytes (uint16/uint32 travel as int16/int32)."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    elif a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(a).cuda()


class Guarded:
    """A device byte buffer with canaries before and after the payload; ``t`` is the payload view."""

    def __init__(self, nbytes: int, dtype: torch.dtype):
        self.raw = torch.full((nbytes + 2 * GUARD,), CANARY, dtype=torch.uint8, device="cuda")
        self.nbytes = nbytes
        self.t = self.raw[GUARD:GUARD + nbytes].view(dtype)

    def check(self):
        r = self.raw.cpu().numpy()
        assert (r[:GUARD] == CANARY).all(), "write before the buffer"
        assert (r[GUARD + self.nbytes:] == CANARY).all(), "write past the buffer"

    def host(self, np_dtype) -> np.ndarray:
        return self.raw[GUARD:GUARD + self.nbytes].cpu().numpy().view(np_dtype)


class GuardedAct(sq.Act):
    """An sq.Act whose arrays sit between canaries."""

    def __init__(self, p, static_mask=None):
        nb = sq.sq_act_bytes(p)
        self.p = p
        self.g_d_lo = Guarded(nb.d_lo, torch.uint8)
        self.g_hi = Guarded(nb.hi_val, torch.int8)
        self.g_slo = Guarded(nb.scale, torch.float32)
        self.g_shi = Guarded(nb.scale, torch.float32)
        self.d_lo, self.hi_val = self.g_d_lo.t, self.g_hi.t
        self.scale_lo, self.scale_hi = self.g_slo.t, self.g_shi.t
        if p.mode != sq.SQ_STATIC:
            self.g_mask = Guarded(nb.mask, torch.int32)
            self.mask = self.g_mask.t
        else:
            self.g_mask = None
            self.mask = static_mask

    def check(self):
        for g in (self.g_d_lo, self.g_hi, self.g_slo, self.g_shi, self.g_mask):
            if g is not None:
                g.check()


def assert_encoding_equal(act: sq.Act, enc, rows=None):
    """Packed encodings must agree bit for bit (codes, mask, and the fp32 scales' bit patterns)."""
    p = act.p
    G = p.K // p.bank
    d_lo = act.d_lo.cpu().numpy().reshape(p.M, p.K // 2)
    hi = act.hi_val.cpu().numpy().reshape(p.M, G, p.topk)
    s_lo = act.scale_lo.cpu().numpy().view(np.uint32)
    s_hi = act.scale_hi.cpu().numpy().view(np.uint32)
    sel = slice(None) if rows is None else rows
    if p.mode != sq.SQ_STATIC:
        mask = act.mask.cpu().numpy().view(np.uint32).reshape(p.M, p.K // 32)
        bad = np.flatnonzero((mask[sel] != enc.mask).any(1))
        assert bad.size == 0, f"mask differs in rows {bad[:8]}"
    bad = np.flatnonzero(s_hi[sel] != enc.s_hi.view(np.uint32))
    assert bad.size == 0, f"scale_hi differs in rows {bad[:8]}"
    bad = np.flatnonzero(s_lo[sel] != enc.s_lo.view(np.uint32))
    assert bad.size == 0, f"scale_lo differs in rows {bad[:8]}"
    bad = np.flatnonzero((hi[sel] != enc.hi_val).reshape(enc.M, -1).any(1))
    assert bad.size == 0, f"hi_val differs in rows {bad[:8]}"
    bad = np.flatnonzero((d_lo[sel] != enc.d_lo).any(1))
    assert bad.size == 0, f"d_lo differs in rows {bad[:8]}"


def assert_outputs_close(y_gpu: np.ndarray, prod, enc, w_scale, rtol=1e-6):
    """Two checks of the fp32 output.
    (1) Against the oracle's fp32 evaluation (same three operations in the same order): relative
        error <= rtol element by element (bit-equality is what is expected).
    (2) Against the oracle's fp64 evaluation: |y - y64| <= 4 * 2^-24 * (|acc_lo*s_lo| + |acc_hi*s_hi|) * |s_w|,
        the bound three fp32 roundings allow; it is relative to the magnitudes of the two parts, not
        to their possibly cancelling sum."""
    y = y_gpu.astype(np.float64)
    y32 = prod.y32.astype(np.float64)
    err = np.abs(y - y32)
    ok = err <= rtol * np.abs(y32)
    worst = np.unravel_index(np.argmax(err - rtol * np.abs(y32)), err.shape)
    assert ok.all(), f"output differs from the fp32 oracle at {worst}: {y_gpu[worst]!r} vs {prod.y32[worst]!r}"
    lo = np.abs(prod.acc_lo.astype(np.float64) * enc.s_lo.astype(np.float64)[:, None])
    hi = np.abs(prod.acc_hi.astype(np.float64) * enc.s_hi.astype(np.float64)[:, None])
    bound = 4.0 * 2.0 ** -24 * (lo + hi) * np.abs(w_scale.astype(np.float64))[None, :]
    err64 = np.abs(y - prod.y64)
    worst = np.unravel_index(np.argmax(err64 - bound), err64.shape)
    assert (err64 <= bound).all(), f"output off the fp64 value at {worst}: {y_gpu[worst]!r} vs {prod.y64[worst]!r}"

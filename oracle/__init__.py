"""CPU oracle for the SQ-format linear layer.   *** TEST INFRASTRUCTURE ***

numpy-facing wrappers around ``sq_oracle.c`` (plain C, compiled with gcc), plus the
storage-accounting formula of Section 4.1.  Only tests, the smoke check and the
benchmark's CPU-baseline leg use this package; the GPU library never does, and this
package never touches the GPU library.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sq_oracle.c")
_LIB = os.path.join(_HERE, "libsq_oracle.so")
_lib = None

OK, ERR_ARG, ERR_MASK, ERR_OVERFLOW = 0, -1, -2, -3


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction, OpenMP over token rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c99", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-fPIC",
               "-shared", "-Wall", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def build_from_source(source_text: str, out_path: str) -> str:
    """Compile a given oracle source text with the oracle's own compiler flags (used by the test that plants
    mistakes in the oracle and checks that the pins notice)."""
    src = out_path + ".c"
    with open(src, "w") as f:
        f.write(source_text)
    cmd = ["gcc", "-std=c99", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-fPIC",
           "-shared", "-o", out_path, src, "-lm"]
    subprocess.run(cmd, check=True)
    return out_path


def _load():
    global _lib
    if _lib is None:
        # SQ_ORACLE_LIB: a substitute library (only the mutation test sets it, for its child processes)
        override = os.environ.get("SQ_ORACLE_LIB")
        if not override:
            build()
        L = ctypes.CDLL(override or _LIB)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
        L.sqo_num_threads.restype = i32
        L.sqo_select_dynamic.argtypes = [vp, i32, i32, i32, vp]
        L.sqo_select_dynamic.restype = i32
        L.sqo_encode.argtypes = [vp, i64, i32, i64, i32, i32, i32, vp, vp, vp, vp, vp, vp]
        L.sqo_encode.restype = i32
        L.sqo_gemm.argtypes = [i64, i32, i64, i32, i32, vp, vp, vp, i64, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.sqo_gemm.restype = i32
        L.sqo_static_mask.argtypes = [vp, i64, i32, vp, vp, i64, i32, i32, vp, vp]
        L.sqo_static_mask.restype = i32
        L.sqo_fma32.argtypes = [i64, vp, vp, vp, vp]
        L.sqo_fma32.restype = None
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    return int(_load().sqo_num_threads())


def select_dynamic(x_row_bits: np.ndarray, bank: int, topk: int) -> np.ndarray:
    """Per-bank top-k by |x| of one token row -> uint8 [K] flags (Sections 3.1, 3.2.2, 4.3)."""
    x = np.ascontiguousarray(x_row_bits, dtype=np.uint16)
    out = np.zeros(x.shape[0], dtype=np.uint8)
    rc = _load().sqo_select_dynamic(_p(x), x.shape[0], bank, topk, _p(out))
    if rc != OK:
        raise ValueError(f"sqo_select_dynamic: {rc}")
    return out


class Encoded:
    """The SQ-format of an activation matrix, Eq. (1): codes, scales, mask and (b, k)."""

    def __init__(self, M, K, bank, topk, mode, d_lo, hi_val, mask, s_lo, s_hi):
        self.M, self.K, self.bank, self.topk, self.mode = M, K, bank, topk, mode
        self.d_lo, self.hi_val, self.mask, self.s_lo, self.s_hi = d_lo, hi_val, mask, s_lo, s_hi

    def rows(self, idx) -> "Encoded":
        idx = np.asarray(idx)
        mask = self.mask if self.mode == 1 else np.ascontiguousarray(self.mask[idx])
        return Encoded(len(idx), self.K, self.bank, self.topk, self.mode,
                       np.ascontiguousarray(self.d_lo[idx]), np.ascontiguousarray(self.hi_val[idx]), mask,
                       np.ascontiguousarray(self.s_lo[idx]), np.ascontiguousarray(self.s_hi[idx]))


def encode(x_bits: np.ndarray, bank: int, topk: int, static_mask: Optional[np.ndarray] = None) -> Encoded:
    """X bf16 bits [M, K] -> SQ-format.  static_mask [K/32] uint32 selects the static rule (Algorithm 2)."""
    x = np.ascontiguousarray(x_bits, dtype=np.uint16)
    M, K = x.shape
    G = K // bank
    mode = 0 if static_mask is None else 1
    d_lo = np.zeros((M, K // 2), np.uint8)
    hi_val = np.zeros((M, G, topk), np.int8)
    s_lo = np.zeros(M, np.float32)
    s_hi = np.zeros(M, np.float32)
    if mode == 0:
        mask = np.zeros((M, K // 32), np.uint32)
        rc = _load().sqo_encode(_p(x), M, K, K, bank, topk, 0, None, _p(d_lo), _p(hi_val), _p(mask), _p(s_lo), _p(s_hi))
    else:
        mask = np.ascontiguousarray(static_mask, dtype=np.uint32)
        assert mask.shape == (K // 32,)
        rc = _load().sqo_encode(_p(x), M, K, K, bank, topk, 1, _p(mask), _p(d_lo), _p(hi_val), None, _p(s_lo), _p(s_hi))
    if rc != OK:
        raise ValueError(f"sqo_encode: {rc}")
    return Encoded(M, K, bank, topk, mode, d_lo, hi_val, mask, s_lo, s_hi)


class Product:
    def __init__(self, acc_lo, acc_hi, y32, ybf16, y64):
        self.acc_lo, self.acc_hi, self.y32, self.ybf16, self.y64 = acc_lo, acc_hi, y32, ybf16, y64


def gemm(enc: Encoded, wq_packed: np.ndarray, w_scale: np.ndarray, want_y64: bool = True) -> Product:
    """Both integer products and the dequantised output (Section 3.3) for every row of ``enc``."""
    wq = np.ascontiguousarray(wq_packed, dtype=np.uint8)
    sw = np.ascontiguousarray(w_scale, dtype=np.float32)
    N = wq.shape[0]
    assert wq.shape[1] == enc.K // 2 and sw.shape == (N,)
    M = enc.M
    acc_lo = np.zeros((M, N), np.int32)
    acc_hi = np.zeros((M, N), np.int32)
    y32 = np.zeros((M, N), np.float32)
    ybf = np.zeros((M, N), np.uint16)
    y64 = np.zeros((M, N), np.float64) if want_y64 else None
    stride = 0 if enc.mode == 1 else enc.K // 32
    rc = _load().sqo_gemm(M, enc.K, N, enc.bank, enc.topk, _p(enc.d_lo), _p(enc.hi_val), _p(enc.mask), stride,
                          _p(enc.s_lo), _p(enc.s_hi), _p(wq), _p(sw), _p(acc_lo), _p(acc_hi), _p(y32), _p(ybf), _p(y64))
    if rc != OK:
        raise ValueError(f"sqo_gemm: {rc}")
    return Product(acc_lo, acc_hi, y32, ybf, y64)


def static_mask(calib_bits: np.ndarray, wq_packed: np.ndarray, w_scale: np.ndarray, bank: int, topk: int
                ) -> Tuple[np.ndarray, np.ndarray]:
    """Calibrated channel mask [K/32] uint32 and the importance scores I_j [K] (Algorithm 2)."""
    c = np.ascontiguousarray(calib_bits, dtype=np.uint16)
    wq = np.ascontiguousarray(wq_packed, dtype=np.uint8)
    sw = np.ascontiguousarray(w_scale, dtype=np.float32)
    T, K = c.shape
    mask = np.zeros(K // 32, np.uint32)
    imp = np.zeros(K, np.float64)
    rc = _load().sqo_static_mask(_p(c), T, K, _p(wq), _p(sw), wq.shape[0], bank, topk, _p(mask), _p(imp))
    if rc != OK:
        raise ValueError(f"sqo_static_mask: {rc}")
    return mask, imp


def fma32(a: np.ndarray, b: np.ndarray, c: np.ndarray) -> np.ndarray:
    """Element-wise fmaf (one rounding), through the C library."""
    a = np.ascontiguousarray(np.broadcast_to(a, np.broadcast(a, b, c).shape), dtype=np.float32)
    b = np.ascontiguousarray(np.broadcast_to(b, a.shape), dtype=np.float32)
    c = np.ascontiguousarray(np.broadcast_to(c, a.shape), dtype=np.float32)
    out = np.empty_like(a)
    _load().sqo_fma32(a.size, _p(a), _p(b), _p(c), _p(out))
    return out


def equivalent_bits(h_high: float, h_low: float, s: float) -> float:
    """Equivalent bit width of an SQ-format activation, y = (1-s)*h_high + s*h_low (Section 4.1, Notation)."""
    return (1.0 - s) * h_high + s * h_low


def stored_bits(h_high: float, h_low: float, s: float, explicit_mask: bool = True) -> float:
    """Bits per element of the layout used here: the low part is kept dense (zeros at the
    high positions), the high part compact, plus one mask bit per element when the mask is explicit."""
    return h_low + (1.0 - s) * h_high + (1.0 if explicit_mask else 0.0)


# ---- tied-scale variant (oracle/tied.py, plain numpy) ----
_tied_mod = None


def _tied():
    """oracle.tied, or -- only for the test that plants mistakes in it -- the copy named by SQ_ORACLE_TIED_SRC."""
    global _tied_mod
    if _tied_mod is None:
        import importlib
        import importlib.util

        override = os.environ.get("SQ_ORACLE_TIED_SRC")
        if override:
            spec = importlib.util.spec_from_file_location(__name__ + ".tied_variant", override)
            mod = importlib.util.module_from_spec(spec)
            mod.__package__ = __name__
            spec.loader.exec_module(mod)
            _tied_mod = mod
        else:
            _tied_mod = importlib.import_module(__name__ + ".tied")
    return _tied_mod


def encode_tied(x_bits: np.ndarray, bank: int, topk: int):
    """X bf16 bits [M, K] -> SQ-format with tied scales (s_lo = 16 * s_hi); see oracle/tied.py."""
    return _tied().encode_tied(x_bits, bank, topk)


def gemm_tied(enc, wq_packed: np.ndarray, w_scale: np.ndarray):
    """The single integer product of the tied-scale layer and its dequantised output."""
    return _tied().gemm_tied(enc, wq_packed, w_scale)


# ---- other precision pairs and the bit-packed storage (oracle/pairs.py, plain numpy) ----
_pairs_mod = None


def _pairs():
    """oracle.pairs, or -- only for the test that plants mistakes in it -- the copy named by SQ_ORACLE_PAIRS_SRC."""
    global _pairs_mod
    if _pairs_mod is None:
        import importlib
        import importlib.util

        override = os.environ.get("SQ_ORACLE_PAIRS_SRC")
        if override:
            spec = importlib.util.spec_from_file_location(__name__ + ".pairs_variant", override)
            mod = importlib.util.module_from_spec(spec)
            mod.__package__ = __name__
            spec.loader.exec_module(mod)
            _pairs_mod = mod
        else:
            _pairs_mod = importlib.import_module(__name__ + ".pairs")
    return _pairs_mod


def encode_pair(x_bits, bank, topk, h_high, h_low, static_mask=None):
    """SQ-format with the precision pair (h_high/h_low) of Section 4.1 / Table 3; see oracle/pairs.py."""
    return _pairs().encode_pair(x_bits, bank, topk, h_high, h_low, static_mask)


def pack_storage(enc, h_high, h_low):
    """The encoding as a bit stream of exactly K*y/8 bytes per row, y = (1-s) h_high + s h_low (Section 4.1)."""
    return _pairs().pack_storage(enc, h_high, h_low)


def unpack_storage(packed, mask, K, bank, topk, h_high, h_low, s_lo, s_hi, static=False):
    return _pairs().unpack_storage(packed, mask, K, bank, topk, h_high, h_low, s_lo, s_hi, static)


def storage_row_bytes(K, bank, topk, h_high, h_low):
    return _pairs().storage_row_bytes(K, bank, topk, h_high, h_low)


def pack_storage_sentinel(enc, h_high, h_low):
    """The implicit-mask form: K*x/8 bytes per row, x = (1-s) h_high + h_low, sentinels at the high channels."""
    return _pairs().pack_storage_sentinel(enc, h_high, h_low)


def unpack_storage_sentinel(packed, K, bank, topk, h_high, h_low, s_lo, s_hi):
    return _pairs().unpack_storage_sentinel(packed, K, bank, topk, h_high, h_low, s_lo, s_hi)


def sentinel_row_bytes(K, bank, topk, h_high, h_low):
    return _pairs().sentinel_row_bytes(K, bank, topk, h_high, h_low)


# ---- SQ-format on weights at run time (oracle/wsq.py, plain numpy) ----
_wsq_mod = None


def wsq_module():
    """oracle.wsq, or -- only for the test that plants mistakes in it -- the copy named by SQ_ORACLE_WSQ_SRC."""
    global _wsq_mod
    if _wsq_mod is None:
        import importlib
        import importlib.util

        override = os.environ.get("SQ_ORACLE_WSQ_SRC")
        if override:
            spec = importlib.util.spec_from_file_location(__name__ + ".wsq_variant", override)
            mod = importlib.util.module_from_spec(spec)
            mod.__package__ = __name__
            spec.loader.exec_module(mod)
            _wsq_mod = mod
        else:
            _wsq_mod = importlib.import_module(__name__ + ".wsq")
    return _wsq_mod

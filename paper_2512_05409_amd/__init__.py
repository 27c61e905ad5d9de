"""Python binding of libsq (the SQ-format linear layer for MI355X).

Argument marshalling only: every function here has the name and the meaning of the C entry
point declared in ``include/sq.h`` and passes device pointers of torch tensors straight
through.  No arithmetic of the method happens in Python, and there is no fallback: if the
HIP library is missing or no GPU is present the calls raise.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libsq.so")

SQ_DYNAMIC, SQ_STATIC, SQ_DYNAMIC_TIED = 0, 1, 2
SQ_OUT_F32, SQ_OUT_BF16 = 0, 1

EXPORTS = (
    "sq_act_bytes", "sq_gemm_workspace_bytes", "sq_linear_workspace_bytes", "sq_weight_prepack_bytes",
    "sq_weight_prepack", "sq_encode", "sq_gemm", "sq_linear", "sq_dense_w4a8_prepack", "sq_dense_w4a8_gemm",
    "sq_calibrate_workspace_bytes", "sq_calibrate_static", "sq_probe_mfma_i8", "sq_probe_stream", "sq_status_string", "sq_version",
    "sq_init", "sq_gemm_variant", "sq_linear_noalloc", "sq_lo_compact_bytes",
    "sq_storage_row_bytes", "sq_pack_storage", "sq_unpack_storage", "sq_probe_mfma_alt", "sq_probe_fp6_tile",
    "sq_storage_row_bytes_sentinel", "sq_pack_storage_sentinel", "sq_unpack_storage_sentinel",
    "sq_wsq_bytes", "sq_wsq_encode", "sq_wsq_prepack_bytes", "sq_wsq_prepack", "sq_quantize_act", "sq_wsq_gemm",
    "sq_wsq_linear_workspace_bytes", "sq_wsq_linear",
)
SQ_NOALLOC_SCRATCH_BYTES = 8 << 20


class SqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


class sq_params(ctypes.Structure):
    _fields_ = [("M", ctypes.c_int32), ("K", ctypes.c_int32), ("N", ctypes.c_int32), ("bank", ctypes.c_int32),
                ("topk", ctypes.c_int32), ("mode", ctypes.c_int32), ("out_dtype", ctypes.c_int32),
                ("h_high", ctypes.c_int32), ("h_low", ctypes.c_int32)]


class sq_act(ctypes.Structure):
    _fields_ = [("d_lo", ctypes.c_void_p), ("hi_val", ctypes.c_void_p), ("mask", ctypes.c_void_p),
                ("scale_lo", ctypes.c_void_p), ("scale_hi", ctypes.c_void_p), ("hi_dense", ctypes.c_void_p),
                ("lo_compact", ctypes.c_void_p)]


class sq_wsq(ctypes.Structure):
    _fields_ = [("lo", ctypes.c_void_p), ("hi_val", ctypes.c_void_p), ("scale_lo", ctypes.c_void_p),
                ("scale_hi", ctypes.c_void_p)]


class sq_weight(ctypes.Structure):
    _fields_ = [("wq", ctypes.c_void_p), ("scale", ctypes.c_void_p), ("prepacked", ctypes.c_void_p)]


_lib = None


def lib() -> ctypes.CDLL:
    """Load libsq.so (built in-tree by ``paper_2512_05409_amd.build``); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2512_05409_amd.build` (needs hipcc)")
        L = ctypes.CDLL(LIB_PATH)
        P, vp, sz, i64 = ctypes.POINTER, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int64
        L.sq_act_bytes.argtypes = [P(sq_params), P(sz), P(sz), P(sz), P(sz)]
        L.sq_act_bytes.restype = sz
        for f in (L.sq_gemm_workspace_bytes, L.sq_linear_workspace_bytes, L.sq_weight_prepack_bytes, L.sq_lo_compact_bytes):
            f.argtypes = [P(sq_params)]
            f.restype = sz
        L.sq_weight_prepack.argtypes = [P(sq_params), vp, vp, vp, vp, vp, vp]
        L.sq_encode.argtypes = [P(sq_params), vp, i64, vp, P(sq_act), vp]
        L.sq_gemm.argtypes = [P(sq_params), P(sq_act), P(sq_weight), vp, i64, vp, vp, vp, sz, vp]
        L.sq_linear.argtypes = [P(sq_params), vp, i64, vp, P(sq_weight), vp, i64, vp, sz, vp]
        L.sq_linear_noalloc.argtypes = [P(sq_params), vp, i64, vp, P(sq_weight), vp, i64, vp]
        L.sq_linear_noalloc.restype = ctypes.c_int
        L.sq_dense_w4a8_prepack.argtypes = [P(sq_params), vp, vp, vp]
        L.sq_dense_w4a8_gemm.argtypes = [P(sq_params), vp, vp, P(sq_weight), vp, i64, vp]
        L.sq_calibrate_workspace_bytes.argtypes = [P(sq_params), i64]
        L.sq_calibrate_workspace_bytes.restype = sz
        L.sq_calibrate_static.argtypes = [P(sq_params), vp, i64, i64, P(sq_weight), vp, vp, vp, sz, vp]
        L.sq_calibrate_static.restype = ctypes.c_int
        L.sq_probe_mfma_i8.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, vp]
        L.sq_probe_stream.argtypes = [vp, sz, vp, sz, vp]
        L.sq_probe_mfma_alt.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, vp]
        L.sq_probe_mfma_alt.restype = ctypes.c_int
        L.sq_probe_fp6_tile.argtypes = [vp, vp, vp, ctypes.c_float, ctypes.c_int, vp]
        L.sq_probe_fp6_tile.restype = ctypes.c_int
        for f in (L.sq_weight_prepack, L.sq_encode, L.sq_gemm, L.sq_linear, L.sq_dense_w4a8_prepack,
                  L.sq_dense_w4a8_gemm, L.sq_probe_mfma_i8, L.sq_probe_stream):
            f.restype = ctypes.c_int
        L.sq_status_string.argtypes = [ctypes.c_int]
        L.sq_status_string.restype = ctypes.c_char_p
        L.sq_version.restype = ctypes.c_char_p
        L.sq_storage_row_bytes.argtypes = [P(sq_params)]
        L.sq_storage_row_bytes.restype = sz
        L.sq_pack_storage.argtypes = [P(sq_params), P(sq_act), vp, vp]
        L.sq_unpack_storage.argtypes = [P(sq_params), vp, P(sq_act), vp]
        L.sq_storage_row_bytes_sentinel.argtypes = [P(sq_params)]
        L.sq_storage_row_bytes_sentinel.restype = sz
        L.sq_pack_storage_sentinel.argtypes = [P(sq_params), P(sq_act), vp, vp]
        L.sq_unpack_storage_sentinel.argtypes = [P(sq_params), vp, P(sq_act), vp]
        L.sq_pack_storage_sentinel.restype = ctypes.c_int
        L.sq_unpack_storage_sentinel.restype = ctypes.c_int
        L.sq_pack_storage.restype = ctypes.c_int
        L.sq_unpack_storage.restype = ctypes.c_int
        L.sq_wsq_bytes.argtypes = [P(sq_params), P(sz), P(sz), P(sz)]
        L.sq_wsq_bytes.restype = sz
        L.sq_wsq_encode.argtypes = [P(sq_params), vp, i64, vp, P(sq_wsq), vp]
        L.sq_wsq_prepack_bytes.argtypes = [P(sq_params)]
        L.sq_wsq_prepack_bytes.restype = sz
        L.sq_wsq_prepack.argtypes = [P(sq_params), P(sq_wsq), vp, vp]
        L.sq_quantize_act.argtypes = [P(sq_params), vp, i64, ctypes.c_int, vp, vp, vp]
        L.sq_wsq_gemm.argtypes = [P(sq_params), vp, vp, P(sq_wsq), vp, vp, i64, vp, vp, vp]
        L.sq_wsq_linear_workspace_bytes.argtypes = [P(sq_params)]
        L.sq_wsq_linear_workspace_bytes.restype = sz
        L.sq_wsq_linear.argtypes = [P(sq_params), vp, i64, ctypes.c_int, P(sq_wsq), vp, vp, i64, vp, sz, vp]
        for f in (L.sq_wsq_encode, L.sq_wsq_prepack, L.sq_quantize_act, L.sq_wsq_gemm, L.sq_wsq_linear):
            f.restype = ctypes.c_int
        L.sq_init.argtypes = []
        L.sq_init.restype = ctypes.c_int
        L.sq_gemm_variant.argtypes = [P(sq_params)]
        L.sq_gemm_variant.restype = ctypes.c_char_p
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().sq_status_string(int(status)).decode()


def version() -> str:
    return lib().sq_version().decode()


def sq_init() -> None:
    _check(lib().sq_init(), "sq_init")


def sq_gemm_variant(p: "sq_params") -> str:
    return lib().sq_gemm_variant(ctypes.byref(p)).decode()


def params(M: int, K: int, N: int, bank: int = 64, topk: int = 8, mode: int = SQ_DYNAMIC,
           out_dtype: int = SQ_OUT_BF16, h_high: int = 0, h_low: int = 0) -> sq_params:
    return sq_params(int(M), int(K), int(N), int(bank), int(topk), int(mode), int(out_dtype), int(h_high), int(h_low))


def _check(rc: int, where: str) -> None:
    if rc != 0:
        raise SqError(rc, where)


def _ptr(t) -> Optional[int]:
    """Device address of a torch tensor (None -> NULL)."""
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("libsq takes device tensors")
    if not t.is_contiguous():
        raise ValueError("libsq takes contiguous tensors")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    import torch

    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream or None


@dataclass
class ActBytes:
    d_lo: int
    hi_val: int
    mask: int
    scale: int
    total: int


def sq_act_bytes(p: sq_params) -> ActBytes:
    a, b, c, d = (ctypes.c_size_t() for _ in range(4))
    tot = lib().sq_act_bytes(ctypes.byref(p), ctypes.byref(a), ctypes.byref(b), ctypes.byref(c), ctypes.byref(d))
    if tot == 0:
        raise SqError(-3, "sq_act_bytes (invalid parameters)")
    return ActBytes(a.value, b.value, c.value, d.value, tot)


def sq_gemm_workspace_bytes(p: sq_params) -> int:
    return int(lib().sq_gemm_workspace_bytes(ctypes.byref(p)))


def sq_linear_workspace_bytes(p: sq_params) -> int:
    return int(lib().sq_linear_workspace_bytes(ctypes.byref(p)))


def sq_weight_prepack_bytes(p: sq_params) -> int:
    return int(lib().sq_weight_prepack_bytes(ctypes.byref(p)))


def sq_lo_compact_bytes(p: sq_params) -> int:
    return int(lib().sq_lo_compact_bytes(ctypes.byref(p)))


class Act:
    """Device buffers of one SQ-format activation matrix (torch tensors, caller-visible)."""

    def __init__(self, p: sq_params, device="cuda", static_mask=None, with_hi_dense=False, with_lo_compact=False):
        import torch

        nb = sq_act_bytes(p)
        self.p = p
        self.hi_dense = None
        self.lo_compact = None
        if with_lo_compact and p.mode == SQ_STATIC:
            self.lo_compact = torch.empty(sq_lo_compact_bytes(p), dtype=torch.uint8, device=device)
        if with_hi_dense and p.mode != SQ_STATIC:
            self.hi_dense = torch.empty(p.M * p.K, dtype=torch.int8, device=device)
        self.d_lo = torch.empty(nb.d_lo, dtype=torch.uint8, device=device)
        self.hi_val = torch.empty(nb.hi_val, dtype=torch.int8, device=device)
        if p.mode != SQ_STATIC:
            self.mask = torch.empty(nb.mask // 4, dtype=torch.int32, device=device)
        else:
            assert static_mask is not None and static_mask.numel() == p.K // 32
            self.mask = static_mask
        self.scale_lo = torch.empty(p.M, dtype=torch.float32, device=device)
        self.scale_hi = torch.empty(p.M, dtype=torch.float32, device=device)

    def c(self) -> sq_act:
        return sq_act(_ptr(self.d_lo), _ptr(self.hi_val), _ptr(self.mask), _ptr(self.scale_lo), _ptr(self.scale_hi),
                      _ptr(getattr(self, "hi_dense", None)), _ptr(getattr(self, "lo_compact", None)))


def weight(wq, scale, prepacked=None) -> sq_weight:
    return sq_weight(_ptr(wq), _ptr(scale), _ptr(prepacked))


def sq_weight_prepack(p: sq_params, wq, static_mask_host, static_mask, out, bad_banks=None, stream=None) -> None:
    """static_mask_host: numpy uint32 [K/32] (host) or None; the rest are device tensors (bad_banks: int32[1] or None)."""
    import numpy as np

    mh = None if static_mask_host is None else np.ascontiguousarray(static_mask_host, dtype=np.uint32)
    _check(lib().sq_weight_prepack(ctypes.byref(p), _ptr(wq), None if mh is None else mh.ctypes.data, _ptr(static_mask),
                                   _ptr(out), _ptr(bad_banks), _stream(stream)), "sq_weight_prepack")


def sq_encode(p: sq_params, x_bf16, out: Act, static_mask=None, ldx: Optional[int] = None, stream=None) -> None:
    a = out.c()
    _check(lib().sq_encode(ctypes.byref(p), _ptr(x_bf16), p.K if ldx is None else ldx, _ptr(static_mask),
                           ctypes.byref(a), _stream(stream)), "sq_encode")


def sq_gemm(p: sq_params, a: Act, w: sq_weight, y, workspace, acc_lo_dbg=None, acc_hi_dbg=None,
            ldy: Optional[int] = None, stream=None) -> None:
    ac = a.c()
    _check(lib().sq_gemm(ctypes.byref(p), ctypes.byref(ac), ctypes.byref(w), _ptr(y), p.N if ldy is None else ldy,
                         _ptr(acc_lo_dbg), _ptr(acc_hi_dbg), _ptr(workspace),
                         0 if workspace is None else workspace.numel() * workspace.element_size(), _stream(stream)),
           "sq_gemm")


def sq_linear(p: sq_params, x_bf16, w: sq_weight, y, workspace, static_mask=None, ldx: Optional[int] = None,
              ldy: Optional[int] = None, stream=None) -> None:
    _check(lib().sq_linear(ctypes.byref(p), _ptr(x_bf16), p.K if ldx is None else ldx, _ptr(static_mask),
                           ctypes.byref(w), _ptr(y), p.N if ldy is None else ldy, _ptr(workspace),
                           workspace.numel() * workspace.element_size(), _stream(stream)), "sq_linear")


def sq_linear_noalloc(p: sq_params, x_bf16, w: sq_weight, y, static_mask=None, ldx: Optional[int] = None,
                      ldy: Optional[int] = None, stream=None) -> None:
    _check(lib().sq_linear_noalloc(ctypes.byref(p), _ptr(x_bf16), p.K if ldx is None else ldx, _ptr(static_mask),
                                   ctypes.byref(w), _ptr(y), p.N if ldy is None else ldy, _stream(stream)),
           "sq_linear_noalloc")


def sq_storage_row_bytes(p: sq_params) -> int:
    return int(lib().sq_storage_row_bytes(ctypes.byref(p)))


def sq_pack_storage(p: sq_params, a: Act, packed, stream=None) -> None:
    ac = a.c()
    _check(lib().sq_pack_storage(ctypes.byref(p), ctypes.byref(ac), _ptr(packed), _stream(stream)), "sq_pack_storage")


def sq_unpack_storage(p: sq_params, packed, a: Act, stream=None) -> None:
    ac = a.c()
    _check(lib().sq_unpack_storage(ctypes.byref(p), _ptr(packed), ctypes.byref(ac), _stream(stream)), "sq_unpack_storage")


def sq_storage_row_bytes_sentinel(p: sq_params) -> int:
    return int(lib().sq_storage_row_bytes_sentinel(ctypes.byref(p)))


def sq_pack_storage_sentinel(p: sq_params, a: Act, packed, stream=None) -> None:
    ac = a.c()
    _check(lib().sq_pack_storage_sentinel(ctypes.byref(p), ctypes.byref(ac), _ptr(packed), _stream(stream)),
           "sq_pack_storage_sentinel")


def sq_unpack_storage_sentinel(p: sq_params, packed, a: Act, stream=None) -> None:
    ac = a.c()
    _check(lib().sq_unpack_storage_sentinel(ctypes.byref(p), _ptr(packed), ctypes.byref(ac), _stream(stream)),
           "sq_unpack_storage_sentinel")


class WeightSQ:
    """Device buffers of a weight matrix in SQ-format (torch tensors)."""

    def __init__(self, p: sq_params, device="cuda"):
        import torch

        a, b, c = (ctypes.c_size_t() for _ in range(3))
        tot = lib().sq_wsq_bytes(ctypes.byref(p), ctypes.byref(a), ctypes.byref(b), ctypes.byref(c))
        if tot == 0:
            raise SqError(-3, "sq_wsq_bytes (invalid parameters)")
        self.p = p
        self.lo = torch.empty(a.value, dtype=torch.uint8, device=device)
        self.hi_val = torch.empty(b.value, dtype=torch.int8, device=device)
        self.scale_lo = torch.empty(c.value // 4, dtype=torch.float32, device=device)
        self.scale_hi = torch.empty(c.value // 4, dtype=torch.float32, device=device)

    def c(self) -> sq_wsq:
        return sq_wsq(_ptr(self.lo), _ptr(self.hi_val), _ptr(self.scale_lo), _ptr(self.scale_hi))


def sq_wsq_encode(p: sq_params, w_bf16, out: WeightSQ, hinv_diag=None, ldw: Optional[int] = None, stream=None) -> None:
    oc = out.c()
    _check(lib().sq_wsq_encode(ctypes.byref(p), _ptr(w_bf16), p.K if ldw is None else ldw, _ptr(hinv_diag), ctypes.byref(oc),
                               _stream(stream)), "sq_wsq_encode")


def sq_wsq_prepack_bytes(p: sq_params) -> int:
    return int(lib().sq_wsq_prepack_bytes(ctypes.byref(p)))


def sq_wsq_prepack(p: sq_params, w: WeightSQ, out, stream=None) -> None:
    wc = w.c()
    _check(lib().sq_wsq_prepack(ctypes.byref(p), ctypes.byref(wc), _ptr(out), _stream(stream)), "sq_wsq_prepack")


def sq_quantize_act(p: sq_params, x_bf16, a8, a_scale, bits: int = 8, ldx: Optional[int] = None, stream=None) -> None:
    _check(lib().sq_quantize_act(ctypes.byref(p), _ptr(x_bf16), p.K if ldx is None else ldx, int(bits), _ptr(a8),
                                 _ptr(a_scale), _stream(stream)), "sq_quantize_act")


def sq_wsq_gemm(p: sq_params, a8, a_scale, w: WeightSQ, prepacked, y, acc_lo_dbg=None, acc_hi_dbg=None,
                ldy: Optional[int] = None, stream=None) -> None:
    wc = w.c()
    _check(lib().sq_wsq_gemm(ctypes.byref(p), _ptr(a8), _ptr(a_scale), ctypes.byref(wc), _ptr(prepacked), _ptr(y),
                             p.N if ldy is None else ldy, _ptr(acc_lo_dbg), _ptr(acc_hi_dbg), _stream(stream)), "sq_wsq_gemm")


def sq_wsq_linear_workspace_bytes(p: sq_params) -> int:
    return int(lib().sq_wsq_linear_workspace_bytes(ctypes.byref(p)))


def sq_wsq_linear(p: sq_params, x_bf16, w: WeightSQ, prepacked, y, workspace, act_bits: int = 8, ldx: Optional[int] = None,
                  ldy: Optional[int] = None, stream=None) -> None:
    wc = w.c()
    _check(lib().sq_wsq_linear(ctypes.byref(p), _ptr(x_bf16), p.K if ldx is None else ldx, int(act_bits), ctypes.byref(wc),
                               _ptr(prepacked), _ptr(y), p.N if ldy is None else ldy, _ptr(workspace),
                               workspace.numel() * workspace.element_size(), _stream(stream)), "sq_wsq_linear")


def sq_dense_w4a8_prepack(p: sq_params, wq, out, stream=None) -> None:
    _check(lib().sq_dense_w4a8_prepack(ctypes.byref(p), _ptr(wq), _ptr(out), _stream(stream)), "sq_dense_w4a8_prepack")


def sq_calibrate_workspace_bytes(p: sq_params, T: int) -> int:
    return int(lib().sq_calibrate_workspace_bytes(ctypes.byref(p), int(T)))


def sq_calibrate_static(p: sq_params, x_calib, T: int, w: sq_weight, mask_out, importance_out, workspace,
                        ldx: Optional[int] = None, stream=None) -> None:
    _check(lib().sq_calibrate_static(ctypes.byref(p), _ptr(x_calib), p.K if ldx is None else ldx, int(T),
                                     ctypes.byref(w), _ptr(mask_out), _ptr(importance_out), _ptr(workspace),
                                     0 if workspace is None else workspace.numel() * workspace.element_size(),
                                     _stream(stream)), "sq_calibrate_static")


def sq_probe_mfma_i8(blocks: int, iters: int, sink, random_operands: bool = False, stream=None) -> None:
    _check(lib().sq_probe_mfma_i8(int(blocks), int(iters), int(bool(random_operands)), _ptr(sink), _stream(stream)),
           "sq_probe_mfma_i8")


def sq_probe_mfma_alt(kind: int, blocks: int, iters: int, sink, stream=None) -> None:
    _check(lib().sq_probe_mfma_alt(int(kind), int(blocks), int(iters), _ptr(sink), _stream(stream)), "sq_probe_mfma_alt")


def sq_probe_fp6_tile(a, b, c, c0: float = 0.0, reps: int = 1, stream=None) -> None:
    _check(lib().sq_probe_fp6_tile(_ptr(a), _ptr(b), _ptr(c), float(c0), int(reps), _stream(stream)), "sq_probe_fp6_tile")


def sq_probe_stream(src, read_bytes: int, dst, write_bytes: int, stream=None) -> None:
    _check(lib().sq_probe_stream(_ptr(src), int(read_bytes), _ptr(dst), int(write_bytes), _stream(stream)),
           "sq_probe_stream")


def sq_dense_w4a8_gemm(p: sq_params, a_i8, a_scale, w: sq_weight, y, ldy: Optional[int] = None, stream=None) -> None:
    _check(lib().sq_dense_w4a8_gemm(ctypes.byref(p), _ptr(a_i8), _ptr(a_scale), ctypes.byref(w), _ptr(y),
                                    p.N if ldy is None else ldy, _stream(stream)), "sq_dense_w4a8_gemm")

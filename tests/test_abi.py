"""Host-side checks of the C ABI: the library loads, exports what include/sq.h declares, and
turns every kind of bad argument into an error code before anything is launched (no GPU needed)."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2512_05409_amd as sq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(sq.LIB_PATH):
        from paper_2512_05409_amd import build
        build.build()
    return sq.lib()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "sq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sq_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(L):
    names = declared_functions()
    assert set(names) == set(sq.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_status_strings(L):
    assert sq.status_string(0) == "SQ_OK"
    for code in range(-8, 0):
        assert sq.status_string(code).startswith("SQ_ERR_")
    assert "unknown" in sq.status_string(-99)
    assert sq.version()


def test_sizes(L):
    p = sq.params(4096, 4096, 22016, 64, 8)
    nb = sq.sq_act_bytes(p)
    assert (nb.d_lo, nb.hi_val, nb.mask, nb.scale) == (4096 * 2048, 4096 * 512, 4096 * 512, 4096 * 4)
    # 0.75 bytes per element + two scales per row (dense low part, compact high part, explicit mask)
    assert nb.total == 4096 * 4096 * 3 // 4 + 2 * 4096 * 4
    assert sq.sq_gemm_workspace_bytes(p) == 4096 * 4096
    assert sq.sq_linear_workspace_bytes(p) >= nb.total + 4096 * 4096  # an sq_act plus its hi_dense image
    assert sq.sq_weight_prepack_bytes(p) == 0
    ps = sq.params(4096, 11008, 4096, 64, 8, mode=sq.SQ_STATIC)
    assert sq.sq_weight_prepack_bytes(ps) == 4096 * 11008 // 2          # every column once: high ones, then low ones
    assert sq.sq_lo_compact_bytes(ps) == 4096 * (11008 - 11008 // 64 * 8) // 2 and sq.sq_lo_compact_bytes(p) == 0
    # static sq_linear keeps only what sq_gemm multiplies: the reordered low part, the high codes, the scales
    assert sq.sq_linear_workspace_bytes(ps) < 4096 * (11008 // 2) + 4096 * (11008 // 8)  # less than dense low + high
    assert sq.sq_gemm_workspace_bytes(ps) == 16
    assert sq.sq_act_bytes(ps).mask == 11008 // 32 * 4


FAKE = 0x10000  # aligned, never dereferenced: every call below must fail before any launch


def _encode(L, p, x=FAKE, ldx=None, mask=None, act=None):
    a = act if act is not None else sq.sq_act(FAKE, FAKE, FAKE, FAKE, FAKE, None)
    return L.sq_encode(ctypes.byref(p), x, p.K if ldx is None else ldx, mask, ctypes.byref(a), None)


@pytest.mark.parametrize("kw,code", [
    (dict(M=0), -2), (dict(K=0), -2), (dict(N=-1), -2),
    (dict(K=4096 + 32), -2),            # K % 64
    (dict(K=64 * 3, bank=128), -2),     # K % bank
    (dict(K=262144), -2),               # K too large
    (dict(K=32768, bank=32), -2),       # more than 512 banks per row
    (dict(bank=48), -3), (dict(bank=256), -3),
    (dict(topk=0), -3), (dict(topk=3), -3), (dict(topk=64, bank=128), -3), (dict(topk=2, bank=64), -3),
    (dict(mode=3), -3), (dict(out_dtype=5), -3),
    (dict(mode=2, K=64 * 5), -3),       # tied scales: K / bank must be a power of two
    (dict(mode=2, K=32768, bank=64), -3),  # tied scales: at most 256 banks per row
    (dict(mode=1, K=64 * 5, bank=64, topk=4), -3),   # static: compact high width not a multiple of 32
])
def test_bad_params_are_refused(L, kw, code):
    base = dict(M=16, K=512, N=512, bank=64, topk=8, mode=0, out_dtype=0)
    base.update(kw)
    p = sq.params(**base)
    assert _encode(L, p) == code
    assert L.sq_act_bytes(ctypes.byref(p), None, None, None, None) == 0
    w = sq.sq_weight(FAKE, FAKE, FAKE)
    a = sq.sq_act(FAKE, FAKE, FAKE, FAKE, FAKE, None)
    assert L.sq_gemm(ctypes.byref(p), ctypes.byref(a), ctypes.byref(w), FAKE, base["N"], None, None, FAKE, 1 << 40, None) == code
    assert L.sq_linear(ctypes.byref(p), FAKE, base["K"], None, ctypes.byref(w), FAKE, base["N"], FAKE, 1 << 40, None) == code


def test_null_alignment_and_leading_dimension(L):
    p = sq.params(16, 512, 512, 64, 8, out_dtype=0)
    assert _encode(L, p, x=None) == -1
    assert _encode(L, p, act=sq.sq_act(FAKE, None, FAKE, FAKE, FAKE, None)) == -1
    assert _encode(L, p, x=FAKE + 2) == -4
    assert _encode(L, p, act=sq.sq_act(FAKE + 4, FAKE, FAKE, FAKE, FAKE, None)) == -4
    assert _encode(L, p, ldx=511) == -2
    assert _encode(L, p, ldx=516) == -4  # rows would not stay 16-byte aligned
    ps = sq.params(16, 512, 512, 64, 8, mode=1)
    assert _encode(L, ps, mask=None) == -3  # static mode needs a mask
    w = sq.sq_weight(FAKE, FAKE, None)
    a = sq.sq_act(FAKE, FAKE, FAKE, FAKE, FAKE, None)
    args = (ctypes.byref(a), ctypes.byref(w), FAKE, 512, None, None)
    assert L.sq_gemm(ctypes.byref(p), *args, None, 0, None) == -7   # no hi_dense and no workspace
    a_hd = sq.sq_act(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE + 8)
    assert L.sq_gemm(ctypes.byref(p), ctypes.byref(a_hd), ctypes.byref(w), FAKE, 512, None, None, None, 0, None) == -4
    assert L.sq_gemm(ctypes.byref(p), *args, FAKE, 16 * 512 - 1, None) == -7
    assert L.sq_gemm(ctypes.byref(p), ctypes.byref(a), ctypes.byref(w), FAKE, 511, None, None, FAKE, 1 << 30, None) == -2
    assert L.sq_gemm(ctypes.byref(p), ctypes.byref(a), ctypes.byref(w), None, 512, None, None, FAKE, 1 << 30, None) == -1
    assert L.sq_gemm(ctypes.byref(ps), ctypes.byref(a), ctypes.byref(w), FAKE, 512, None, None, FAKE, 1 << 30, None) == -1  # static needs prepacked
    assert L.sq_linear(ctypes.byref(p), FAKE, 512, None, ctypes.byref(w), FAKE, 512, FAKE, 16, None) == -7
    assert L.sq_linear(ctypes.byref(p), FAKE, 512, None, ctypes.byref(w), FAKE, 512, FAKE + 16, 1 << 30, None) == -4
    assert L.sq_dense_w4a8_gemm(ctypes.byref(p), FAKE, FAKE, ctypes.byref(w), FAKE, 512, None) == -1  # needs prepacked


def test_calibrate_arguments(L):
    ps = sq.params(1, 512, 64, 64, 8, mode=1)
    pd = sq.params(1, 512, 64, 64, 8, mode=0)
    w = sq.sq_weight(FAKE, FAKE, None)
    need = L.sq_calibrate_workspace_bytes(ctypes.byref(ps), 100)
    assert need >= (2 + 1) * 512 * 8 and need % 8 == 0
    assert L.sq_calibrate_workspace_bytes(ctypes.byref(pd), 100) == 0   # dynamic mode has no mask to calibrate
    assert L.sq_calibrate_workspace_bytes(ctypes.byref(ps), 0) == 0
    call = lambda p, x=FAKE, ldx=512, T=100, wt=w, m=FAKE, imp=None, ws=FAKE, nb=need: L.sq_calibrate_static(
        ctypes.byref(p), x, ldx, T, ctypes.byref(wt), m, imp, ws, nb, None)
    assert call(pd) == -3
    assert call(ps, x=None) == -1
    assert call(ps, m=None) == -1
    assert call(ps, wt=sq.sq_weight(None, FAKE, None)) == -1
    assert call(ps, T=0) == -2
    assert call(ps, ldx=256) == -2
    assert call(ps, ldx=516) == -4
    assert call(ps, x=FAKE + 2) == -4
    assert call(ps, imp=FAKE + 8) == -4
    assert call(ps, ws=None) == -7
    assert call(ps, nb=need - 1) == -7


def test_probe_arguments(L):
    assert L.sq_probe_mfma_i8(4, 16, 0, None, None) == -1
    assert L.sq_probe_mfma_i8(0, 16, 1, FAKE, None) == -2
    assert L.sq_probe_mfma_i8(4, 10, 0, FAKE, None) == -2
    assert L.sq_probe_mfma_i8(4, 0, 0, FAKE, None) == -2
    assert L.sq_probe_mfma_i8(1 << 20, 8, 1, FAKE, None) == -2
    assert L.sq_probe_stream(None, 1024, FAKE, 1024, None) == -1
    assert L.sq_probe_stream(FAKE, 1024, None, 1024, None) == -1
    assert L.sq_probe_stream(FAKE, 1000, FAKE, 1024, None) == -2
    assert L.sq_probe_stream(FAKE, 0, FAKE, 0, None) == -2
    assert L.sq_probe_stream(FAKE + 4, 1024, FAKE, 1024, None) == -4


def test_prepack_checks_the_mask_on_the_host(L):
    ps = sq.params(16, 512, 512, 64, 8, mode=1)
    good = np.zeros(512 // 32, np.uint32)
    good[0::2] = 0xFF  # 8 bits in every bank of 64
    bad = good.copy()
    bad[2] = 0x7F
    assert L.sq_weight_prepack(ctypes.byref(ps), FAKE, bad.ctypes.data, FAKE, FAKE, None, None) == -6
    pd = sq.params(16, 512, 512, 64, 8, mode=0)
    assert L.sq_weight_prepack(ctypes.byref(pd), FAKE, good.ctypes.data, FAKE, FAKE, None, None) == -3
    assert L.sq_weight_prepack(ctypes.byref(ps), None, good.ctypes.data, FAKE, FAKE, None, None) == -1
    assert L.sq_weight_prepack(ctypes.byref(ps), FAKE, None, None, FAKE, None, None) == -1   # the device mask is required
    assert L.sq_weight_prepack(ctypes.byref(ps), FAKE, None, FAKE + 4, FAKE, None, None) == -4


def test_binding_refuses_host_tensors():
    import torch
    with pytest.raises(ValueError):
        sq._ptr(torch.zeros(4))


def test_gemm_variant_names(L):
    """Which kernel a shape runs on (the GPU tests use this to state what they cover)."""
    assert sq.sq_gemm_variant(sq.params(4096, 4096, 22016)) == "tile128x256"      # 32 x 86 tiles
    assert sq.sq_gemm_variant(sq.params(1500, 320, 6100)) == "tile128x256"        # 12 x 24 tiles
    assert sq.sq_gemm_variant(sq.params(200, 1024, 300)) == "tile128x128"
    assert sq.sq_gemm_variant(sq.params(64, 8192, 28672)) == "tile64x128"
    assert sq.sq_gemm_variant(sq.params(64, 8192, 4096)) == "tile64x64"
    assert sq.sq_gemm_variant(sq.params(20, 8192 + 64, 28672)) == "tile64x64"
    assert sq.sq_gemm_variant(sq.params(8, 8192, 28672)) == "stream32"
    assert sq.sq_gemm_variant(sq.params(8, 8192 + 64, 28672)) == "tile64x64"      # K % 128 != 0
    assert sq.sq_gemm_variant(sq.params(8, 8192, 28672, mode=sq.SQ_STATIC)) == "tile64x64"
    assert sq.sq_gemm_variant(sq.params(8, 100, 64)) == "invalid"
    assert sq.sq_gemm_variant(sq.params(4096, 4096, 22016, mode=sq.SQ_DYNAMIC_TIED)) == "tile256x256"   # 16 x 86 tiles
    assert sq.sq_gemm_variant(sq.params(1500, 512, 6100, mode=sq.SQ_DYNAMIC_TIED)) == "tile128x256"
    assert sq.sq_gemm_variant(sq.params(8, 8192, 28672, mode=sq.SQ_DYNAMIC_TIED)) == "tile64x64"

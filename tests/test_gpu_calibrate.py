"""GPU parity of the device-side static calibration (Algorithm 2 up to the mask) against the oracle.

Both sides work in fp64.  The oracle adds each sum sequentially; the device adds per-chunk partial sums in
chunk order.  On these inputs every partial sum is exactly representable (bf16 magnitudes; an fp32 scale of
limited range times a 4-bit integer), so the importance scores must agree bit for bit and the masks with
them.  Independently of that, every mask is checked for validity against the oracle's scores: exactly k
bits per bank, and no unselected channel scoring above a selected one.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2512_05409_amd as sq
import workloads
from gpu_util import Guarded, dev

pytestmark = pytest.mark.gpu


def run_device(calib_bits, wq_packed, w_scale, bank, topk, ldx=None, want_importance=True):
    T, K = calib_bits.shape
    N = wq_packed.shape[0]
    p = sq.params(1, K, N, bank, topk, mode=sq.SQ_STATIC)
    ldx = K if ldx is None else ldx
    xh = np.zeros((T, ldx), np.uint16)
    xh[:, :K] = calib_bits
    if ldx > K:
        xh[:, K:] = 0x7F80  # +inf in the padding: must never be read
    x = dev(xh)
    wqd, swd = dev(wq_packed), dev(w_scale)  # sq.weight keeps raw addresses: the tensors must stay alive
    w = sq.weight(wqd, swd, None)
    ws_bytes = sq.sq_calibrate_workspace_bytes(p, T)
    assert ws_bytes > 0
    ws = Guarded(ws_bytes, torch.uint8)
    gm = Guarded(K // 32 * 4, torch.int32)
    gi = Guarded(K * 8, torch.float64) if want_importance else None
    sq.sq_calibrate_static(p, x, T, w, gm.t, gi.t if gi else None, ws.t, ldx=ldx)
    torch.cuda.synchronize()
    ws.check(), gm.check()
    if gi:
        gi.check()
    return gm.host(np.uint32).copy(), (gi.host(np.float64).copy() if gi else None)


def check_valid(mask, imp, bank, topk):
    K = imp.shape[0]
    flags = ((mask[np.arange(K) // 32] >> (np.arange(K) % 32)) & 1).astype(bool).reshape(-1, bank)
    assert (flags.sum(axis=1) == topk).all()
    s = imp.reshape(-1, bank)
    lo_sel = np.where(flags, s, np.inf).min(axis=1)
    hi_unsel = np.where(flags, -np.inf, s).max(axis=1)
    assert (lo_sel >= hi_unsel).all()


def small_case(seed, T, K, N, scale_kind="uniform"):
    rng = np.random.Generator(np.random.PCG64([seed, 77]))
    x = rng.standard_normal((T, K)).astype(np.float32)
    x[:, rng.choice(K, size=max(1, K // 100), replace=False)] *= 30.0
    wq = workloads.pack_int4(rng.integers(-8, 8, size=(N, K), dtype=np.int8))
    sw = rng.uniform(0.005, 0.02, size=N).astype(np.float32)
    return workloads.f32_to_bf16_bits(x), wq, sw


@pytest.mark.parametrize("T,K,N,bank,topk", [
    (1, 64, 1, 64, 32),        # one token, one weight row
    (7, 256, 33, 64, 8),       # ragged row chunks on both sides
    (100, 512, 200, 32, 4),
    (513, 1024, 1000, 128, 16),
    (64, 2048, 129, 128, 32),
    (300, 4096, 777, 64, 16),
])
def test_small_shapes(T, K, N, bank, topk):
    calib, wq, sw = small_case(T * 31 + K, T, K, N)
    m_ref, i_ref = oracle.static_mask(calib, wq, sw, bank, topk)
    m, i = run_device(calib, wq, sw, bank, topk)
    np.testing.assert_array_equal(i.view(np.uint64), i_ref.view(np.uint64))
    np.testing.assert_array_equal(m, m_ref)
    check_valid(m, i_ref, bank, topk)


def test_ties_go_to_the_lower_channel():
    T, K, N, bank, topk = 16, 256, 8, 64, 8
    calib = workloads.f32_to_bf16_bits(np.ones((T, K), np.float32))
    wq = workloads.pack_int4(np.full((N, K), 3, np.int8))
    sw = np.full(N, 0.5, np.float32)
    m, i = run_device(calib, wq, sw, bank, topk)
    assert (i == 12.0).all()  # 1 * (8 * 0.5 * 3)
    m_ref, _ = oracle.static_mask(calib, wq, sw, bank, topk)
    np.testing.assert_array_equal(m, m_ref)
    assert (m.reshape(-1, 2)[:, 0] == 0xFF).all() and (m.reshape(-1, 2)[:, 1] == 0).all()
    # all-zero column sums: every score is zero, still the first k channels
    wq0 = workloads.pack_int4(np.zeros((N, K), np.int8))
    m0, i0 = run_device(calib, wq0, sw, bank, topk)
    assert (i0 == 0).all()
    np.testing.assert_array_equal(m0, m)


def test_leading_dimension_and_optional_importance():
    calib, wq, sw = small_case(5, 40, 512, 64)
    m_ref, _ = oracle.static_mask(calib, wq, sw, 64, 8)
    m, i = run_device(calib, wq, sw, 64, 8, ldx=512 + 64, want_importance=False)
    assert i is None
    np.testing.assert_array_equal(m, m_ref)


def test_config4_calibration_full_size():
    wl = workloads.make("c4_down7b_static")
    m_ref, i_ref = oracle.static_mask(wl.calib_bits, wl.wq_packed, wl.w_scale, wl.bank, wl.topk)
    m, i = run_device(wl.calib_bits, wl.wq_packed, wl.w_scale, wl.bank, wl.topk)
    check_valid(m, i_ref, wl.bank, wl.topk)
    np.testing.assert_array_equal(i.view(np.uint64), i_ref.view(np.uint64))
    np.testing.assert_array_equal(m, m_ref)
    # the calibrated mask names the outlier channels the workload planted
    flags = (m[wl.outlier_channels // 32] >> (wl.outlier_channels % 32)) & 1
    assert flags.mean() > 0.9


def test_calibrated_mask_feeds_the_layer():
    """Device mask -> prepack -> sq_linear equals the oracle run with the oracle's mask."""
    rng_case = small_case(11, 128, 512, 256)
    calib, wq, sw = rng_case
    x = workloads.f32_to_bf16_bits(np.random.Generator(np.random.PCG64(5)).standard_normal((48, 512)).astype(np.float32))
    bank, topk = 64, 8
    m_ref, _ = oracle.static_mask(calib, wq, sw, bank, topk)
    m, _ = run_device(calib, wq, sw, bank, topk)
    enc = oracle.encode(x, bank, topk, static_mask=m_ref)
    ref = oracle.gemm(enc, wq, sw)
    p = sq.params(48, 512, 256, bank, topk, mode=sq.SQ_STATIC, out_dtype=sq.SQ_OUT_F32)
    wqd, swd, md = dev(wq), dev(sw), dev(m)
    pre = torch.empty(sq.sq_weight_prepack_bytes(p), dtype=torch.uint8, device="cuda")
    sq.sq_weight_prepack(p, wqd, m, md, pre)
    w = sq.weight(wqd, swd, pre)
    y = torch.empty(48 * 256, dtype=torch.float32, device="cuda")
    ws = torch.empty(sq.sq_linear_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    sq.sq_linear(p, dev(x), w, y, ws, static_mask=md)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(y.cpu().numpy().view(np.uint32), ref.y32.reshape(-1).view(np.uint32))

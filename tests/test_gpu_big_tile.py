"""Full-coverage parity for the 128 x 256 workgroup tile (the kernel the benchmark configurations run).

The tile is picked only for shapes with more than 128 such tiles, so these cases have many tiles (12 x 24 and
more: several rounds of workgroups over the chip, ragged last tile row and tile column, the XCD-aware
workgroup-to-tile mapping on a large grid) and a short K, which lets the oracle compute EVERY row and column.
Both accumulators, the fp32 and the bf16 output are compared element by element, in all three modes of the
kernel: dynamic (low + zero-padded high in one loop), static (low loop, then the compact high loop) and the
plain W4A8 reference (high loop only).  Outputs go into buffers pre-filled with a canary between guard bytes.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2512_05409_amd as sq
from workloads import pack_int4
from gpu_util import Guarded, dev
from test_gpu_parity import make_static_mask, random_case, run_gemm

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def check_all(p, enc, wq, sw, prepacked=None, static_mask=None):
    prod = oracle.gemm(enc, wq, sw)
    p.out_dtype = sq.SQ_OUT_F32
    y, alo, ahi = run_gemm(p, enc, wq, sw, sq.SQ_OUT_F32, prepacked=prepacked, static_mask=static_mask)
    assert np.array_equal(alo, prod.acc_lo), "acc_lo"
    assert np.array_equal(ahi, prod.acc_hi), "acc_hi"
    assert np.array_equal(y.view(np.uint32), prod.y32.view(np.uint32)), "fp32 output"
    p.out_dtype = sq.SQ_OUT_BF16
    y16, _, _ = run_gemm(p, enc, wq, sw, sq.SQ_OUT_BF16, prepacked=prepacked, static_mask=static_mask)
    assert np.array_equal(y16, prod.ybf16), "bf16 output"


@pytest.mark.parametrize("M,K,N,bank,topk", [(1500, 320, 6100, 64, 8),    # 3 K steps, the last one partial
                                             (1409, 256, 5900, 32, 4),    # 2 K steps: no steady-state iteration
                                             (1300, 640, 6200, 64, 8),    # 5 K steps: steady state + every peeled tail
                                             (1537, 1024, 8200, 128, 16)])  # 8 K steps, M one row past a tile edge
def test_big_tile_dynamic_every_element(M, K, N, bank, topk):
    _say(f"big tile dynamic M={M} K={K} N={N} bank={bank} topk={topk}")
    p = sq.params(M, K, N, bank, topk, out_dtype=sq.SQ_OUT_F32)
    assert sq.sq_gemm_variant(p) == "tile128x256"
    bits, wq, sw = random_case(5000 + M + K + N, M, K, N, outliers=4)
    check_all(p, oracle.encode(bits, bank, topk), wq, sw)


@pytest.mark.parametrize("M,K,N,bank,topk", [(1500, 256, 6100, 64, 8),    # K_hi = 32: one partial high step
                                             (1409, 512, 5900, 32, 4),    # K_hi = 64
                                             (1300, 1024, 6200, 64, 16)])  # K_hi = 256: two high steps
def test_big_tile_static_every_element(M, K, N, bank, topk):
    _say(f"big tile static M={M} K={K} N={N} bank={bank} topk={topk}")
    p = sq.params(M, K, N, bank, topk, mode=sq.SQ_STATIC, out_dtype=sq.SQ_OUT_F32)
    assert sq.sq_gemm_variant(p) == "tile128x256"
    bits, wq, sw = random_case(6000 + M + K + N, M, K, N, outliers=4)
    mask = make_static_mask(K, bank, topk, seed=K + N)
    enc = oracle.encode(bits, bank, topk, static_mask=mask)
    pre = torch.empty(sq.sq_weight_prepack_bytes(p), dtype=torch.uint8, device="cuda")
    sq.sq_weight_prepack(p, dev(wq), mask, dev(mask), pre)
    check_all(p, enc, wq, sw, prepacked=pre, static_mask=mask)


@pytest.mark.parametrize("M,K,N", [(1500, 320, 6100), (1300, 640, 6200)])
@pytest.mark.parametrize("out_dtype", [sq.SQ_OUT_F32, sq.SQ_OUT_BF16])
def test_big_tile_dense_w4a8_every_element(M, K, N, out_dtype):
    """The plain W4A8 reference of the benchmark on the same tile, against an exact integer matmul (float64 BLAS
    on integers below 2^53 is exact) and the two-multiplication epilogue written out in numpy."""
    _say(f"big tile dense w4a8 M={M} K={K} N={N} out={out_dtype}")
    p = sq.params(M, K, N, out_dtype=out_dtype)
    assert sq.sq_gemm_variant(p) == "tile128x256"
    rng = np.random.default_rng(M + K + N)
    a = rng.integers(-127, 128, size=(M, K)).astype(np.int8)
    sa = rng.uniform(0.01, 0.1, M).astype(np.float32)
    w = rng.integers(-8, 8, size=(N, K)).astype(np.int8)
    sw = rng.uniform(0.005, 0.02, N).astype(np.float32)
    wqd, swd = dev(pack_int4(w)), dev(sw)
    pre = torch.empty(N * K // 2, dtype=torch.uint8, device="cuda")
    sq.sq_dense_w4a8_prepack(p, wqd, pre)
    esz = 4 if out_dtype == sq.SQ_OUT_F32 else 2
    y = Guarded(M * N * esz, torch.float32 if esz == 4 else torch.int16)
    sq.sq_dense_w4a8_gemm(p, dev(a), dev(sa), sq.weight(wqd, swd, pre), y.t)
    torch.cuda.synchronize()
    y.check()
    acc = (a.astype(np.float64) @ w.astype(np.float64).T).astype(np.int64)
    want = (acc.astype(np.float32) * sa[:, None]).astype(np.float32) * sw[None, :]
    if esz == 4:
        assert np.array_equal(y.host(np.float32).reshape(M, N), want)
    else:
        from workloads import f32_to_bf16_bits
        assert np.array_equal(y.host(np.uint16).reshape(M, N), f32_to_bf16_bits(want))


# ---- leading dimension of Y: padded rows (vector stores when the rows stay 16-byte aligned, element stores
# otherwise), on every kernel variant; the padding columns must keep their canary ----
@pytest.mark.parametrize("M,K,N,variant", [(1300, 256, 6100, "tile128x256"), (200, 512, 300, "tile128x128"),
                                           (50, 512, 200, "tile64x64"), (8, 512, 200, "stream32")])
@pytest.mark.parametrize("pad", [8, 3])
@pytest.mark.parametrize("out_dtype", [sq.SQ_OUT_F32, sq.SQ_OUT_BF16])
def test_output_leading_dimension(M, K, N, variant, pad, out_dtype):
    _say(f"ldy M={M} K={K} N={N} pad={pad} out={out_dtype} ({variant})")
    bank, topk = 64, 8
    p = sq.params(M, K, N, bank, topk, out_dtype=out_dtype)
    assert sq.sq_gemm_variant(p) == variant
    bits, wq, sw = random_case(7000 + M + N + pad, M, K, N, outliers=4)
    enc = oracle.encode(bits, bank, topk)
    prod = oracle.gemm(enc, wq, sw)
    act = sq.Act(p)
    act.d_lo.copy_(dev(enc.d_lo).view(-1))
    act.hi_val.copy_(dev(enc.hi_val).view(-1))
    act.mask.copy_(dev(enc.mask).view(-1))
    act.scale_lo.copy_(dev(enc.s_lo))
    act.scale_hi.copy_(dev(enc.s_hi))
    ldy = N + pad
    esz = 4 if out_dtype == sq.SQ_OUT_F32 else 2
    y = Guarded(M * ldy * esz, torch.float32 if esz == 4 else torch.int16)
    ws = torch.empty(sq.sq_gemm_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    sq.sq_gemm(p, act, sq.weight(dev(wq), dev(sw)), y.t, ws, ldy=ldy)
    torch.cuda.synchronize()
    y.check()
    if esz == 4:
        got = y.host(np.uint32).reshape(M, ldy)
        assert np.array_equal(got[:, :N], prod.y32.view(np.uint32))
        assert (got[:, N:] == 0xA5A5A5A5).all(), "padding columns were written"
    else:
        got = y.host(np.uint16).reshape(M, ldy)
        assert np.array_equal(got[:, :N], prod.ybf16)
        assert (got[:, N:] == 0xA5A5).all(), "padding columns were written"


@pytest.mark.parametrize("M,N,variant", [(1300, 6100, "tile128x256"), (200, 300, "tile128x128"), (50, 200, "tile64x64"),
                                         (8, 200, "stream32")])
def test_tiny_magnitude_rows(M, N, variant):
    """Rows whose values are around 1e-30 (per-token scales near 2^-103 and 2^-107): the epilogue must still
    give the oracle's bits, i.e. no intermediate of the dequantisation may leave the normal fp32 range."""
    _say(f"tiny magnitudes M={M} N={N} ({variant})")
    K, bank, topk = 256, 64, 8
    p = sq.params(M, K, N, bank, topk, out_dtype=sq.SQ_OUT_F32)
    assert sq.sq_gemm_variant(p) == variant
    rng = np.random.default_rng(M + N)
    from workloads import f32_to_bf16_bits
    x = rng.standard_normal((M, K)).astype(np.float32)
    x = (np.sign(x) * np.maximum(np.abs(x), 1e-3)).astype(np.float32)  # every element stays a normal bf16 below
    x[0::2] *= np.float32(1e-30)
    x[1::10] *= np.float32(3e-33)
    bits = f32_to_bf16_bits(x)
    w = rng.integers(-8, 8, size=(N, K)).astype(np.int8)
    sw = rng.uniform(0.5, 2.0, N).astype(np.float32)
    enc = oracle.encode(bits, bank, topk)
    assert enc.s_lo.min() < 2.0 ** -108
    prod = oracle.gemm(enc, pack_int4(w), sw)
    y, alo, ahi = run_gemm(p, enc, pack_int4(w), sw, sq.SQ_OUT_F32)
    assert np.array_equal(alo, prod.acc_lo) and np.array_equal(ahi, prod.acc_hi)
    assert np.array_equal(y.view(np.uint32), prod.y32.view(np.uint32))


@pytest.mark.parametrize("mode", ["dynamic", "static"])
@pytest.mark.parametrize("M,K,N", [(50, 256, 25700), (64, 384, 26000)])
def test_wide_small_tile_every_element(M, K, N, mode):
    """The 64 x 128 tile (33-64 tokens on very wide layers), every element, both accumulators."""
    bank, topk = 64, 8
    static = mode == "static"
    if static and (K // bank * topk) % 32:
        K = 512
    p = sq.params(M, K, N, bank, topk, mode=sq.SQ_STATIC if static else sq.SQ_DYNAMIC, out_dtype=sq.SQ_OUT_F32)
    assert sq.sq_gemm_variant(p) == "tile64x128"
    _say(f"wide small tile {mode} M={M} K={K} N={N}")
    bits, wq, sw = random_case(8000 + M + K + N, M, K, N, outliers=4)
    if static:
        mask = make_static_mask(K, bank, topk, seed=K + N)
        enc = oracle.encode(bits, bank, topk, static_mask=mask)
        pre = torch.empty(sq.sq_weight_prepack_bytes(p), dtype=torch.uint8, device="cuda")
        sq.sq_weight_prepack(p, dev(wq), mask, dev(mask), pre)
        check_all(p, enc, wq, sw, prepacked=pre, static_mask=mask)
    else:
        check_all(p, oracle.encode(bits, bank, topk), wq, sw)

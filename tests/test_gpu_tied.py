"""GPU parity for the tied-scale variant (mode SQ_DYNAMIC_TIED: s_lo = 16 * s_hi, one INT8 operand, one
accumulator) against oracle/tied.py: packed encoding and scale bit patterns, the combined INT8 operand, the
accumulator, fp32 outputs bit for bit (tolerance 1e-6 relative is what is required), bf16 outputs identical."""
import numpy as np
import pytest
import torch

import oracle
import paper_2512_05409_amd as sq
import workloads
from gpu_util import Guarded, GuardedAct, assert_encoding_equal, dev
from test_gpu_parity import random_case

pytestmark = pytest.mark.gpu
torch.backends.cuda.matmul.allow_tf32 = False


def _say(msg):
    print(msg, flush=True)


def consumer_order(codes):
    """[M, K] codes in channel order -> the byte order of sq_act::hi_dense (per 8 channels: evens, then odds)."""
    M, K = codes.shape
    g = codes.reshape(M, K // 8, 8)
    return np.concatenate([g[:, :, 0::2], g[:, :, 1::2]], axis=2).reshape(M, K)


@pytest.mark.parametrize("bank,topk", [(64, 8), (32, 2), (32, 4), (32, 8), (32, 16), (64, 4), (64, 16), (64, 32),
                                       (128, 8), (128, 16), (128, 32)])
@pytest.mark.parametrize("M,K", [(37, 1024), (5, 8192), (130, 512)])
def test_encode_tied_bit_exact(M, K, bank, topk):
    if K // bank > (128 if bank == 128 else 256):
        pytest.skip("row longer than the tied encoder takes")
    _say(f"encode tied M={M} K={K} bank={bank} topk={topk}")
    bits, _, _ = random_case(900 + bank + topk + M, M=M, K=K, N=8, outliers=min(6, K // 16))
    p = sq.params(M, K, 64, bank, topk, mode=sq.SQ_DYNAMIC_TIED)
    enc = oracle.encode_tied(bits, bank, topk)
    act = GuardedAct(p)
    image = Guarded(M * K, torch.int8)
    act.hi_dense = image.t
    sq.sq_encode(p, dev(bits), act)
    torch.cuda.synchronize()
    act.check()
    image.check()
    assert_encoding_equal(act, enc)
    assert np.array_equal(image.host(np.int8).reshape(M, K), consumer_order(enc.codes))


def run_gemm_tied(p, enc, wq, sw, out_dtype, with_image):
    M, N = p.M, p.N
    p.out_dtype = out_dtype
    act = sq.Act(p, with_hi_dense=with_image)
    act.d_lo.copy_(dev(enc.d_lo).view(-1))
    act.hi_val.copy_(dev(enc.hi_val).view(-1))
    act.mask.copy_(dev(enc.mask).view(-1))
    act.scale_lo.copy_(dev(enc.s_lo))
    act.scale_hi.copy_(dev(enc.s_hi))
    if with_image:
        act.hi_dense.copy_(dev(consumer_order(enc.codes)).view(-1))
    esz = 4 if out_dtype == sq.SQ_OUT_F32 else 2
    y = Guarded(M * N * esz, torch.float32 if esz == 4 else torch.int16)
    acc = Guarded(M * N * 4, torch.int32)
    ws = torch.empty(sq.sq_gemm_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    sq.sq_gemm(p, act, sq.weight(dev(wq), dev(sw)), y.t, ws, acc_hi_dbg=acc.t)
    torch.cuda.synchronize()
    y.check()
    acc.check()
    return y.host(np.float32 if esz == 4 else np.uint16).reshape(M, N), acc.host(np.int32).reshape(M, N)


@pytest.mark.parametrize("M,K,N,bank,topk", [(16, 512, 512, 64, 8), (200, 1024, 300, 64, 8), (129, 256, 130, 32, 4),
                                             (64, 2048, 256, 128, 16), (1, 512, 128, 64, 8), (33, 2048, 70, 64, 16),
                                             (1500, 512, 6100, 64, 8), (1300, 1024, 6200, 32, 8)])
@pytest.mark.parametrize("with_image", [True, False])
def test_gemm_tied_every_element(M, K, N, bank, topk, with_image):
    """with_image: the combined operand comes from the caller; otherwise sq_gemm builds it from the format."""
    p = sq.params(M, K, N, bank, topk, mode=sq.SQ_DYNAMIC_TIED, out_dtype=sq.SQ_OUT_F32)
    _say(f"gemm tied M={M} K={K} N={N} bank={bank} topk={topk} image={with_image} ({sq.sq_gemm_variant(p)})")
    bits, wq, sw = random_case(1200 + M + K + N, M, K, N, outliers=4)
    enc = oracle.encode_tied(bits, bank, topk)
    prod = oracle.gemm_tied(enc, wq, sw)
    y, acc = run_gemm_tied(p, enc, wq, sw, sq.SQ_OUT_F32, with_image)
    assert np.array_equal(acc, prod.acc), "accumulator"
    assert (np.abs(y.astype(np.float64) - prod.y32.astype(np.float64)) <= 1e-6 * np.abs(prod.y32.astype(np.float64))).all()
    assert np.array_equal(y.view(np.uint32), prod.y32.view(np.uint32)), "fp32 outputs are expected to be bit-identical"
    y16, _ = run_gemm_tied(p, enc, wq, sw, sq.SQ_OUT_BF16, with_image)
    assert np.array_equal(y16, prod.ybf16)


@pytest.mark.parametrize("M", [70, 8])
def test_linear_tied_end_to_end(M):
    _say(f"linear tied M={M}")
    K, N, bank, topk = 1024, 192, 64, 8
    bits, wq, sw = random_case(3100 + M, M, K, N)
    prod = oracle.gemm_tied(oracle.encode_tied(bits, bank, topk), wq, sw)
    p = sq.params(M, K, N, bank, topk, mode=sq.SQ_DYNAMIC_TIED, out_dtype=sq.SQ_OUT_BF16)
    y = Guarded(M * N * 2, torch.int16)
    ws = Guarded(sq.sq_linear_workspace_bytes(p), torch.uint8)
    sq.sq_linear(p, dev(bits), sq.weight(dev(wq), dev(sw)), y.t, ws.t)
    torch.cuda.synchronize()
    y.check()
    ws.check()
    assert np.array_equal(y.host(np.uint16).reshape(M, N), prod.ybf16)
    y2 = Guarded(M * N * 2, torch.int16)
    sq.sq_linear_noalloc(p, dev(bits), sq.weight(dev(wq), dev(sw)), y2.t)
    torch.cuda.synchronize()
    assert torch.equal(y.t, y2.t)


def test_tied_at_the_benchmark_shape():
    """c3 at full size: encoding of every row against the oracle; the accumulator of the whole matrix against an
    fp32 library matmul of the oracle's combined codes (exact: every partial sum is an integer below 2^24);
    outputs of sampled rows (one per band of 128) bit for bit, of all rows within the rounding bound."""
    wl = workloads.make("c3_mlp7b")
    M, K, N = wl.M, wl.K, wl.N
    p = sq.params(M, K, N, wl.bank, wl.topk, mode=sq.SQ_DYNAMIC_TIED, out_dtype=sq.SQ_OUT_BF16)
    _say(f"tied c3: oracle encode ({sq.sq_gemm_variant(p)})")
    enc = oracle.encode_tied(wl.x_bits, wl.bank, wl.topk)
    xd, wqd, swd = dev(wl.x_bits), dev(wl.wq_packed), dev(wl.w_scale)
    act = sq.Act(p, with_hi_dense=True)
    sq.sq_encode(p, xd, act)
    torch.cuda.synchronize()
    assert_encoding_equal(act, enc)
    assert np.array_equal(act.hi_dense.cpu().numpy().reshape(M, K), consumer_order(enc.codes))
    y = torch.full((M * N,), -23131, dtype=torch.int16, device="cuda")
    acc = torch.full((M * N,), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
    sq.sq_gemm(p, act, sq.weight(wqd, swd), y, None, acc_hi_dbg=acc)
    torch.cuda.synchronize()
    from test_gpu_configs import unpack_int4_device, sample_rows
    Wf = unpack_int4_device(wqd, N, K)
    want = dev(enc.codes).to(torch.float32) @ Wf.T
    assert float(want.abs().max()) < 2 ** 24
    assert torch.equal(acc.view(M, N), want.to(torch.int32)), "accumulator differs somewhere in the whole matrix"
    y64 = acc.view(M, N).double() * dev(enc.s_hi).double()[:, None] * swd.double()[None, :]
    yv = (y.view(M, N).to(torch.int32) << 16).view(torch.float32).double()
    assert bool(((yv - y64).abs() <= (2.0 ** -8 + 3 * 2.0 ** -24) * y64.abs()).all())
    rows = sample_rows(M, 8, seed=5)
    sub = oracle.tied.EncodedTied(len(rows), K, wl.bank, wl.topk, None, None, None, enc.s_lo[rows], enc.s_hi[rows], enc.codes[rows])
    prod = oracle.gemm_tied(sub, wl.wq_packed, wl.w_scale)
    rd = torch.from_numpy(rows).cuda()
    assert np.array_equal(y.view(M, N)[rd].cpu().numpy().view(np.uint16), prod.ybf16)
    # the fused entry point gives the same bytes
    y2 = torch.full_like(y, 1)
    ws = torch.empty(sq.sq_linear_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    sq.sq_linear(p, xd, sq.weight(wqd, swd), y2, ws)
    torch.cuda.synchronize()
    assert torch.equal(y, y2)


@pytest.mark.parametrize("M,K,N", [(4100, 256, 8200), (4353, 1024, 7950)])
def test_huge_tile_single_product_every_element(M, K, N):
    """The 256 x 256 tile of the single-product modes (at least 512 such tiles): tied-scale layer and the plain
    W4A8 reference, every element.  Expected accumulators: float64 BLAS matmul of the oracle's integer codes
    (exact below 2^53); the epilogue's two fp32 multiplications written out in numpy; sampled rows also through
    the oracle's own product."""
    bank, topk = 64, 8
    p = sq.params(M, K, N, bank, topk, mode=sq.SQ_DYNAMIC_TIED, out_dtype=sq.SQ_OUT_F32)
    assert sq.sq_gemm_variant(p) == "tile256x256"
    _say(f"huge tile tied M={M} K={K} N={N}")
    bits, wq, sw = random_case(1700 + M + K + N, M, K, N, outliers=4)
    enc = oracle.encode_tied(bits, bank, topk)
    W = workloads.unpack_int4(wq).astype(np.float64)
    acc_want = (enc.codes.astype(np.float64) @ W.T).astype(np.int64)
    y_want = ((acc_want.astype(np.float32) * enc.s_hi[:, None]).astype(np.float32) * sw[None, :]).astype(np.float32)
    y, acc = run_gemm_tied(p, enc, wq, sw, sq.SQ_OUT_F32, True)
    assert np.array_equal(acc.astype(np.int64), acc_want)
    assert np.array_equal(y.view(np.uint32), y_want.view(np.uint32))
    rows = np.array([0, 255, 256, M // 2, M - 1])
    sub = oracle.tied.EncodedTied(len(rows), K, bank, topk, None, None, None, enc.s_lo[rows], enc.s_hi[rows], enc.codes[rows])
    prod = oracle.gemm_tied(sub, wq, sw)
    assert np.array_equal(y[rows].view(np.uint32), prod.y32.view(np.uint32)) and np.array_equal(acc[rows], prod.acc)
    y16, _ = run_gemm_tied(p, enc, wq, sw, sq.SQ_OUT_BF16, True)
    assert np.array_equal(y16, workloads.f32_to_bf16_bits(y_want))
    # plain W4A8 reference on the same tile
    _say("huge tile dense w4a8")
    rng = np.random.default_rng(M + N)
    a = rng.integers(-127, 128, size=(M, K)).astype(np.int8)
    sa = rng.uniform(0.01, 0.1, M).astype(np.float32)
    pd = sq.params(M, K, N, out_dtype=sq.SQ_OUT_F32)
    wqd, swd = dev(wq), dev(sw)
    pre = torch.empty(N * K // 2, dtype=torch.uint8, device="cuda")
    sq.sq_dense_w4a8_prepack(pd, wqd, pre)
    yd = Guarded(M * N * 4, torch.float32)
    sq.sq_dense_w4a8_gemm(pd, dev(a), dev(sa), sq.weight(wqd, swd, pre), yd.t)
    torch.cuda.synchronize()
    yd.check()
    accd = (a.astype(np.float64) @ W.T).astype(np.int64)
    want = (accd.astype(np.float32) * sa[:, None]).astype(np.float32) * sw[None, :]
    assert np.array_equal(yd.host(np.float32).reshape(M, N), want.astype(np.float32))

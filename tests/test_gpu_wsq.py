"""GPU parity for SQ-format on weights at run time (sq_wsq_encode / sq_wsq_prepack / sq_quantize_act / sq_wsq_gemm /
sq_wsq_linear) against oracle/wsq.py: the weight encoding (codes, sentinels, per-group scale bit patterns), the
activation codes, the exact per-bank integer products, fp32 outputs bit for bit (1e-6 relative is what is required)
and bf16 outputs."""
import numpy as np
import pytest
import torch

import oracle
import paper_2512_05409_amd as sq
from workloads import f32_to_bf16_bits, pack_int4
from gpu_util import Guarded, dev

pytestmark = pytest.mark.gpu
W = oracle.wsq_module()


def _say(msg):
    print(msg, flush=True)


def case(seed, M, K, N):
    rng = np.random.default_rng(seed)
    w = (rng.standard_normal((N, K)) * 0.04).astype(np.float32)
    w[:, rng.choice(K, 5, replace=False)] *= 6.0          # a few heavy input channels
    w[0] = 0.0                                            # an all-zero output channel: scales 1, codes 0
    if N > 2:
        w[2] = 0.125                                      # all-equal magnitudes: ties go to the lower channels
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[:, rng.choice(K, 4, replace=False)] *= 25.0
    if M > 1:
        x[1] = 0.0
    d = rng.uniform(0.5, 2.0, K).astype(np.float32)
    return f32_to_bf16_bits(w), f32_to_bf16_bits(x), d


def consumer_order(codes):
    M, K = codes.shape
    g = codes.reshape(M, K // 8, 8)
    return np.concatenate([g[:, :, 0::2], g[:, :, 1::2]], axis=2).reshape(M, K)


@pytest.mark.parametrize("N,K,bank,topk,h_high,h_low,with_d", [(37, 256, 64, 8, 8, 4, False), (20, 512, 128, 16, 8, 4, True),
                                                              (9, 256, 64, 16, 8, 2, True), (11, 128, 64, 4, 4, 2, False),
                                                              (5, 256, 64, 1, 8, 3, False), (70, 1024, 64, 8, 8, 4, True)])
def test_weight_encoding_bit_exact(N, K, bank, topk, h_high, h_low, with_d):
    _say(f"wsq encode N={N} K={K} bank={bank} topk={topk} ({h_high}/{h_low}) d={with_d}")
    wb, _, d = case(100 + N + K, 4, K, N)
    want = W.encode_weights(wb, bank, topk, h_high, h_low, d=d if with_d else None)
    p = sq.params(1, K, N, bank, topk, h_high=h_high, h_low=h_low)
    ws = sq.WeightSQ(p)
    sq.sq_wsq_encode(p, dev(wb), ws, hinv_diag=dev(d) if with_d else None)
    torch.cuda.synchronize()
    G = K // bank
    lo_want = pack_int4(want.lo)       # same 4-bit containers (the sentinel is -2^(h_low-1), sign-extended)
    assert np.array_equal(ws.lo.cpu().numpy().reshape(N, K // 2), lo_want)
    assert np.array_equal(ws.hi_val.cpu().numpy().reshape(N, G, topk), want.hi_val)
    assert np.array_equal(ws.scale_lo.cpu().numpy().view(np.uint32).reshape(N, G), want.s_lo.view(np.uint32))
    assert np.array_equal(ws.scale_hi.cpu().numpy().view(np.uint32).reshape(N, G), want.s_hi.view(np.uint32))


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("M,K", [(9, 256), (70, 4096), (1, 128)])
def test_activation_quantiser(M, K, bits):
    _say(f"quantize act M={M} K={K} bits={bits}")
    _, xb, _ = case(300 + M + K, M, K, 4)
    codes, scale = W.quantize_activations(xb, bits)
    p = sq.params(M, K, 64)
    a8 = Guarded(M * K, torch.int8)
    sa = Guarded(M * 4, torch.float32)
    sq.sq_quantize_act(p, dev(xb), a8.t, sa.t, bits=bits)
    torch.cuda.synchronize()
    a8.check()
    sa.check()
    assert np.array_equal(a8.host(np.int8).reshape(M, K), consumer_order(codes))
    assert np.array_equal(sa.host(np.uint32), scale.view(np.uint32))


@pytest.mark.parametrize("M,K,N,bank,topk,h_high,h_low,bits", [(16, 256, 64, 64, 8, 8, 4, 8), (70, 512, 130, 64, 8, 8, 4, 8),
                                                              (33, 512, 200, 128, 16, 8, 4, 8), (5, 1024, 65, 64, 16, 8, 2, 8),
                                                              (100, 256, 96, 64, 8, 4, 2, 4), (129, 384, 64, 128, 32, 8, 3, 8),
                                                              (300, 1024, 390, 64, 8, 8, 4, 8), (257, 512, 129, 128, 16, 8, 4, 8)])
def test_layer_against_the_oracle(M, K, N, bank, topk, h_high, h_low, bits):
    _say(f"wsq linear M={M} K={K} N={N} bank={bank} topk={topk} ({h_high}/{h_low}) A{bits}")
    wb, xb, d = case(500 + M + K + N, M, K, N)
    want_w = W.encode_weights(wb, bank, topk, h_high, h_low, d=d)
    codes, scale = W.quantize_activations(xb, bits)
    prod = W.gemm(codes, scale, want_w)
    G = K // bank
    p = sq.params(M, K, N, bank, topk, out_dtype=sq.SQ_OUT_F32, h_high=h_high, h_low=h_low)
    ws = sq.WeightSQ(p)
    sq.sq_wsq_encode(p, dev(wb), ws, hinv_diag=dev(d))
    pre = Guarded(sq.sq_wsq_prepack_bytes(p), torch.uint8)
    sq.sq_wsq_prepack(p, ws, pre.t)
    a8 = torch.empty(M * K, dtype=torch.int8, device="cuda")
    sa = torch.empty(M, dtype=torch.float32, device="cuda")
    sq.sq_quantize_act(p, dev(xb), a8, sa, bits=bits)
    y = Guarded(M * N * 4, torch.float32)
    alo, ahi = Guarded(M * N * G * 4, torch.int32), Guarded(M * N * G * 4, torch.int32)
    sq.sq_wsq_gemm(p, a8, sa, ws, pre.t, y.t, acc_lo_dbg=alo.t, acc_hi_dbg=ahi.t)
    torch.cuda.synchronize()
    for g_ in (pre, y, alo, ahi):
        g_.check()
    assert np.array_equal(alo.host(np.int32).reshape(M, N, G), prod.acc_lo), "per-bank low products"
    assert np.array_equal(ahi.host(np.int32).reshape(M, N, G), prod.acc_hi), "per-bank high products"
    got = y.host(np.float32).reshape(M, N)
    err = np.abs(got.astype(np.float64) - prod.y32.astype(np.float64))
    assert (err <= 1e-6 * np.abs(prod.y32.astype(np.float64))).all()
    assert np.array_equal(got.view(np.uint32), prod.y32.view(np.uint32)), "fp32 outputs are expected to be bit-identical"
    # without the per-bank dump (large shapes then take the throughput kernel): the same fp32 bits
    y2 = Guarded(M * N * 4, torch.float32)
    sq.sq_wsq_gemm(p, a8, sa, ws, pre.t, y2.t)
    torch.cuda.synchronize()
    y2.check()
    assert np.array_equal(y2.host(np.uint32).reshape(M, N), prod.y32.view(np.uint32))
    # the fused entry point, bf16 output
    p16 = sq.params(M, K, N, bank, topk, out_dtype=sq.SQ_OUT_BF16, h_high=h_high, h_low=h_low)
    y16 = Guarded(M * N * 2, torch.int16)
    wsb = Guarded(sq.sq_wsq_linear_workspace_bytes(p16), torch.uint8)
    sq.sq_wsq_linear(p16, dev(xb), ws, pre.t, y16.t, wsb.t, act_bits=bits)
    torch.cuda.synchronize()
    y16.check()
    wsb.check()
    assert np.array_equal(y16.host(np.uint16).reshape(M, N), prod.ybf16)


def test_bad_arguments_are_refused():
    p = sq.params(8, 256, 64, 32, 4)          # bank 32 is not a weight bank size here
    assert sq.sq_wsq_prepack_bytes(p) == 0
    with pytest.raises(sq.SqError):
        sq.WeightSQ(p)
    p = sq.params(8, 256, 64, 64, 8, h_high=8, h_low=5)
    assert sq.sq_wsq_prepack_bytes(p) == 0

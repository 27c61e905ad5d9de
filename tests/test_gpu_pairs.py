"""GPU parity for the precision pairs (8/3), (8/2), (4/2) of Section 4.1 / Table 3 and for the bit-packed storage
of the format, against oracle/pairs.py (encoding, storage stream) and the pinned C oracle (products on the codes)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2512_05409_amd as sq
from gpu_util import Guarded, GuardedAct, assert_encoding_equal, dev
from test_gpu_parity import make_static_mask, random_case, run_gemm

pytestmark = pytest.mark.gpu
PAIRS = [(8, 4), (8, 3), (8, 2), (4, 2)]


def _say(msg):
    print(msg, flush=True)


@pytest.mark.parametrize("h_high,h_low", PAIRS)
@pytest.mark.parametrize("M,K,bank,topk", [(37, 1024, 64, 8), (9, 4096, 32, 4), (5, 320, 64, 16), (130, 512, 128, 16)])
def test_encode_dynamic_pairs(M, K, bank, topk, h_high, h_low):
    _say(f"encode dynamic ({h_high}/{h_low}) M={M} K={K} bank={bank} topk={topk}")
    bits, _, _ = random_case(4100 + M + K + h_low, M=M, K=K, N=8, outliers=4)
    p = sq.params(M, K, 64, bank, topk, h_high=h_high, h_low=h_low)
    act = GuardedAct(p)
    sq.sq_encode(p, dev(bits), act)
    torch.cuda.synchronize()
    act.check()
    assert_encoding_equal(act, oracle.encode_pair(bits, bank, topk, h_high, h_low))


@pytest.mark.parametrize("h_high,h_low", PAIRS)
@pytest.mark.parametrize("M,K,bank,topk", [(21, 1024, 64, 8), (6, 11008, 64, 8), (12, 2048, 32, 4)])
def test_encode_static_pairs(M, K, bank, topk, h_high, h_low):
    _say(f"encode static ({h_high}/{h_low}) M={M} K={K} bank={bank} topk={topk}")
    bits, _, _ = random_case(4300 + M + K + h_low, M=M, K=K, N=8, outliers=4)
    mask = make_static_mask(K, bank, topk, seed=K + h_low)
    p = sq.params(M, K, 64, bank, topk, mode=sq.SQ_STATIC, h_high=h_high, h_low=h_low)
    md = dev(mask)
    act = GuardedAct(p, static_mask=md)
    sq.sq_encode(p, dev(bits), act, static_mask=md)
    torch.cuda.synchronize()
    act.check()
    assert_encoding_equal(act, oracle.encode_pair(bits, bank, topk, h_high, h_low, static_mask=mask))


@pytest.mark.parametrize("h_high,h_low", [(8, 3), (8, 2), (4, 2)])
@pytest.mark.parametrize("M,K,N", [(200, 1024, 300), (8, 1024, 200), (1300, 256, 6100)])
def test_gemm_on_pair_encodings(M, K, N, h_high, h_low):
    """The products and the epilogue are the same kernels whatever the pair: accumulators and outputs must be the
    pinned oracle's on the pair's codes."""
    _say(f"gemm ({h_high}/{h_low}) M={M} K={K} N={N}")
    bank, topk = 64, 8
    bits, wq, sw = random_case(4500 + M + N + h_low, M, K, N, outliers=4)
    enc = oracle.encode_pair(bits, bank, topk, h_high, h_low)
    prod = oracle.gemm(enc, wq, sw)
    p = sq.params(M, K, N, bank, topk, out_dtype=sq.SQ_OUT_F32, h_high=h_high, h_low=h_low)
    y, alo, ahi = run_gemm(p, enc, wq, sw, sq.SQ_OUT_F32)
    assert np.array_equal(alo, prod.acc_lo) and np.array_equal(ahi, prod.acc_hi)
    assert np.array_equal(y.view(np.uint32), prod.y32.view(np.uint32))
    # the whole layer through sq_linear
    pl = sq.params(M, K, N, bank, topk, out_dtype=sq.SQ_OUT_BF16, h_high=h_high, h_low=h_low)
    yl = Guarded(M * N * 2, torch.int16)
    ws = torch.empty(sq.sq_linear_workspace_bytes(pl), dtype=torch.uint8, device="cuda")
    sq.sq_linear(pl, dev(bits), sq.weight(dev(wq), dev(sw)), yl.t, ws)
    torch.cuda.synchronize()
    yl.check()
    assert np.array_equal(yl.host(np.uint16).reshape(M, N), prod.ybf16)


@pytest.mark.parametrize("h_high,h_low", PAIRS)
@pytest.mark.parametrize("mode", ["dynamic", "static"])
@pytest.mark.parametrize("M,K,bank,topk", [(19, 1024, 64, 8), (7, 512, 32, 4), (5, 2048, 128, 32), (3, 512, 64, 4)])
def test_storage_stream(M, K, bank, topk, mode, h_high, h_low):
    """sq_pack_storage writes exactly K*y/8 bytes per row, equal to the oracle's stream; sq_unpack_storage is its
    inverse."""
    if mode == "static" and (K // bank * topk) % 32:
        pytest.skip("static mode needs a compact high width that is a multiple of 32")
    _say(f"storage ({h_high}/{h_low}) {mode} M={M} K={K} bank={bank} topk={topk}")
    bits, _, _ = random_case(4700 + M + K + h_low + bank, M=M, K=K, N=8, outliers=4)
    mask = make_static_mask(K, bank, topk, seed=K + 1) if mode == "static" else None
    enc = oracle.encode_pair(bits, bank, topk, h_high, h_low, static_mask=mask)
    want = oracle.pack_storage(enc, h_high, h_low)
    p = sq.params(M, K, 64, bank, topk, mode=sq.SQ_STATIC if mask is not None else sq.SQ_DYNAMIC, h_high=h_high, h_low=h_low)
    s = 1 - topk / bank
    assert sq.sq_storage_row_bytes(p) * 8 == K * ((1 - s) * h_high + s * h_low) == want.shape[1] * 8
    md = None if mask is None else dev(mask)
    act = sq.Act(p, static_mask=md)
    sq.sq_encode(p, dev(bits), act, static_mask=md)
    packed = Guarded(M * sq.sq_storage_row_bytes(p), torch.uint8)
    sq.sq_pack_storage(p, act, packed.t)
    torch.cuda.synchronize()
    packed.check()
    assert np.array_equal(packed.host(np.uint8).reshape(M, -1), want)
    back = GuardedAct(p, static_mask=md)
    if mask is None:
        back.mask.copy_(act.mask)
    back.d_lo.fill_(0x5A)
    back.hi_val.fill_(0x5A)
    sq.sq_unpack_storage(p, packed.t, back)
    torch.cuda.synchronize()
    back.check()
    assert torch.equal(back.d_lo, act.d_lo) and torch.equal(back.hi_val, act.hi_val)


def test_unsupported_pairs_are_refused():
    for hh, hl in [(8, 5), (4, 3), (6, 4), (8, 1), (2, 2)]:
        assert sq.sq_gemm_variant(sq.params(16, 512, 512, h_high=hh, h_low=hl)) == "invalid"
    assert sq.sq_gemm_variant(sq.params(16, 512, 512, mode=sq.SQ_DYNAMIC_TIED, h_high=8, h_low=3)) == "invalid"
    assert sq.sq_gemm_variant(sq.params(16, 512, 512, h_high=8, h_low=3)) != "invalid"


@pytest.mark.parametrize("h_high,h_low", PAIRS)
@pytest.mark.parametrize("M,K,bank,topk", [(19, 1024, 64, 8), (7, 512, 32, 4), (5, 2048, 128, 32)])
def test_sentinel_storage_stream(M, K, bank, topk, h_high, h_low):
    """The implicit-mask form: sq_pack_storage_sentinel writes K*x/8 bytes per row equal to the oracle's stream;
    sq_unpack_storage_sentinel recovers codes AND the mask from it."""
    _say(f"sentinel storage ({h_high}/{h_low}) M={M} K={K} bank={bank} topk={topk}")
    bits, _, _ = random_case(4900 + M + K + h_low + bank, M=M, K=K, N=8, outliers=4)
    enc = oracle.encode_pair(bits, bank, topk, h_high, h_low)
    want = oracle.pack_storage_sentinel(enc, h_high, h_low)
    p = sq.params(M, K, 64, bank, topk, h_high=h_high, h_low=h_low)
    s = 1 - topk / bank
    assert sq.sq_storage_row_bytes_sentinel(p) * 8 == K * ((1 - s) * h_high + h_low) == want.shape[1] * 8
    act = sq.Act(p)
    sq.sq_encode(p, dev(bits), act)
    packed = Guarded(M * sq.sq_storage_row_bytes_sentinel(p), torch.uint8)
    sq.sq_pack_storage_sentinel(p, act, packed.t)
    torch.cuda.synchronize()
    packed.check()
    assert np.array_equal(packed.host(np.uint8).reshape(M, -1), want)
    back = GuardedAct(p)
    for t in (back.d_lo, back.hi_val, back.mask):
        t.fill_(0x5A)
    sq.sq_unpack_storage_sentinel(p, packed.t, back)
    torch.cuda.synchronize()
    back.check()
    assert torch.equal(back.mask, act.mask), "the mask must come back out of the sentinels"
    assert torch.equal(back.d_lo, act.d_lo) and torch.equal(back.hi_val, act.hi_val)
    ps = sq.params(M, K, 64, bank, topk, mode=sq.SQ_STATIC, h_high=h_high, h_low=h_low)
    assert sq.sq_storage_row_bytes_sentinel(ps) == 0

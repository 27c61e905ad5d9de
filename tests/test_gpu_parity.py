"""GPU parity: libsq (through its C ABI) against the CPU oracle on the same seeded inputs.

Bit-exact: packed encodings (codes, mask, scale bit patterns) and both INT32 accumulators.
fp32 outputs: relative error <= 1e-6 against the oracle's fp32 evaluation and within three
roundings of its fp64 evaluation; bf16 outputs: identical bit patterns.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2512_05409_amd as sq
import workloads
from workloads import f32_to_bf16_bits, pack_int4
from gpu_util import Guarded, GuardedAct, assert_encoding_equal, assert_outputs_close, dev

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def random_case(seed, M, K, N, outliers=6):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[:, rng.choice(K, outliers, replace=False)] *= rng.uniform(20, 50, outliers).astype(np.float32)
    # a few rows with heavy ties and a zero row, to exercise the tie-break and the degenerate scales
    if M > 3:
        x[1] = rng.choice(np.array([0.0, 0.5, -0.5, 1.0, 2.0, -2.0], np.float32), size=K)
        x[2] = 0.0
        x[3] = 1.0
    w = rng.integers(-8, 8, size=(N, K)).astype(np.int8)
    sw = rng.uniform(0.005, 0.02, N).astype(np.float32)
    return f32_to_bf16_bits(x), pack_int4(w), sw


def run_encode(bits, bank, topk, static_mask=None, ldx=None):
    M, K = bits.shape
    mode = sq.SQ_DYNAMIC if static_mask is None else sq.SQ_STATIC
    p = sq.params(M, K, 64, bank, topk, mode=mode)
    if ldx is None:
        xd = dev(bits)
    else:
        padded = np.full((M, ldx), 0x7F80, np.uint16)  # +inf in the padding: must never be read as data
        padded[:, :K] = bits
        xd = dev(padded)
    md = None if static_mask is None else dev(static_mask)
    act = GuardedAct(p, static_mask=md)
    sq.sq_encode(p, xd, act, static_mask=md, ldx=ldx)
    torch.cuda.synchronize()
    act.check()
    return p, act


@pytest.mark.parametrize("bank,topk", [(64, 8), (32, 2), (32, 4), (32, 8), (32, 16), (64, 4), (64, 16), (64, 32),
                                       (128, 8), (128, 16), (128, 32)])
def test_encode_dynamic_bit_exact(bank, topk):
    _say(f"encode dynamic bank={bank} topk={topk}")
    bits, _, _ = random_case(100 + bank + topk, M=37, K=1024, N=8)
    p, act = run_encode(bits, bank, topk)
    assert_encoding_equal(act, oracle.encode(bits, bank, topk))


@pytest.mark.parametrize("bank,topk", [(64, 8), (32, 2), (32, 4), (32, 8), (32, 16), (64, 4), (64, 16), (64, 32),
                                       (128, 8), (128, 16), (128, 32)])
@pytest.mark.parametrize("M,K", [(7, 1024), (32, 4096), (1, 8192)])
def test_encode_dynamic_few_rows(M, K, bank, topk):
    """A handful of rows (decode shapes), every format."""
    _say(f"encode dynamic few rows M={M} K={K} bank={bank} topk={topk}")
    bits, _, _ = random_case(3 * bank + topk + M + K, M=M, K=K, N=8)
    p, act = run_encode(bits, bank, topk)
    assert_encoding_equal(act, oracle.encode(bits, bank, topk))


@pytest.mark.parametrize("M,K,bank,topk", [(1, 64, 64, 8), (3, 128, 128, 8), (5, 8192, 64, 8), (2, 11008, 64, 8),
                                           (2, 11008, 32, 4), (3, 16384, 32, 8), (130, 512, 64, 8), (9, 4096, 128, 16)])
def test_encode_dynamic_shapes(M, K, bank, topk):
    _say(f"encode dynamic shape M={M} K={K} bank={bank} topk={topk}")
    bits, _, _ = random_case(7 * M + K, M=M, K=K, N=8, outliers=min(6, K // 16))
    p, act = run_encode(bits, bank, topk)
    assert_encoding_equal(act, oracle.encode(bits, bank, topk))


@pytest.mark.parametrize("K,bank,topk", [(32768, 64, 8), (65536, 128, 16), (16384, 32, 4)])
def test_encode_dynamic_longest_rows(K, bank, topk):
    """K / bank = 512 banks per row: the most the encoder takes (one workgroup of 512 lanes per row)."""
    _say(f"encode dynamic longest row K={K} bank={bank}")
    bits, _, _ = random_case(K + bank, M=5, K=K, N=8, outliers=40)
    p, act = run_encode(bits, bank, topk)
    assert_encoding_equal(act, oracle.encode(bits, bank, topk))


def test_encode_leading_dimension_and_determinism():
    _say("encode ldx / determinism")
    bits, _, _ = random_case(5, M=20, K=512, N=8)
    p, a1 = run_encode(bits, 64, 8, ldx=512 + 64)
    enc = oracle.encode(bits, 64, 8)
    assert_encoding_equal(a1, enc)
    p, a2 = run_encode(bits, 64, 8)
    for f in ("d_lo", "hi_val", "mask", "scale_lo", "scale_hi"):
        assert torch.equal(getattr(a1, f), getattr(a2, f))


def make_static_mask(K, bank, topk, seed):
    rng = np.random.default_rng(seed)
    mask = np.zeros(K // 32, np.uint32)
    for g in range(K // bank):
        for i in rng.choice(bank, topk, replace=False):
            j = g * bank + int(i)
            mask[j // 32] |= np.uint32(1 << (j % 32))
    return mask


@pytest.mark.parametrize("K,bank,topk", [(512, 64, 8), (1024, 32, 4), (2048, 128, 16), (11008, 64, 8), (512, 64, 4)])
def test_encode_static_bit_exact(K, bank, topk):
    _say(f"encode static K={K} bank={bank} topk={topk}")
    bits, _, _ = random_case(300 + K + bank, M=21, K=K, N=8)
    mask = make_static_mask(K, bank, topk, seed=K + topk)
    p, act = run_encode(bits, bank, topk, static_mask=mask)
    assert_encoding_equal(act, oracle.encode(bits, bank, topk, static_mask=mask))


def run_gemm(p, enc_host, wq, sw, out_dtype, prepacked=None, static_mask=None):
    """Upload an oracle encoding and run sq_gemm on it; returns (y, acc_lo, acc_hi) host arrays."""
    M, N = p.M, p.N
    md = None if static_mask is None else dev(static_mask)
    act = sq.Act(p, static_mask=md)
    act.d_lo.copy_(dev(enc_host.d_lo).view(-1))
    act.hi_val.copy_(dev(enc_host.hi_val).view(-1))
    if p.mode == sq.SQ_DYNAMIC:
        act.mask.copy_(dev(enc_host.mask).view(-1))
    act.scale_lo.copy_(dev(enc_host.s_lo))
    act.scale_hi.copy_(dev(enc_host.s_hi))
    wqd, swd = dev(wq), dev(sw)
    w = sq.weight(wqd, swd, prepacked)
    esz = 4 if out_dtype == sq.SQ_OUT_F32 else 2
    y = Guarded(M * N * esz, torch.float32 if esz == 4 else torch.int16)
    alo = Guarded(M * N * 4, torch.int32)
    ahi = Guarded(M * N * 4, torch.int32)
    ws = torch.empty(sq.sq_gemm_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    sq.sq_gemm(p, act, w, y.t, ws, acc_lo_dbg=alo.t, acc_hi_dbg=ahi.t)
    torch.cuda.synchronize()
    for g in (y, alo, ahi):
        g.check()
    yh = y.host(np.float32 if esz == 4 else np.uint16).reshape(M, N)
    return yh, alo.host(np.int32).reshape(M, N), ahi.host(np.int32).reshape(M, N)


# shapes chosen to reach the small kernel variants: the 128x128 tile (M > 64 with few tiles), the 64x64 tile
# (32 < M <= 64, or M <= 32 with K % 128 != 0), the weight-streaming kernel (M <= 32, K % 128 == 0) with
# 1 ... 26 K steps (fewer than its rings hold, exactly as many, the first trip of the steady state, several
# tail lengths), ragged M / N / K edges.  The 128x256 tile needs more than 128 tiles: test_gpu_big_tile.py.
@pytest.mark.parametrize("M,K,N,bank,topk", [(16, 512, 512, 64, 8), (200, 1024, 300, 64, 8), (129, 320, 130, 32, 4),
                                             (64, 2048, 256, 128, 16), (1, 512, 128, 64, 8), (257, 64, 5, 64, 16),
                                             (5, 384, 130, 64, 8), (32, 2048, 70, 64, 16), (8, 320, 96, 32, 8),
                                             (33, 1152, 200, 128, 32), (3, 128, 64, 64, 8),
                                             (4, 256, 64, 64, 8), (7, 768, 100, 64, 8), (12, 1024, 64, 64, 8),
                                             (2, 1280, 70, 64, 8), (9, 2304, 64, 64, 8), (17, 2560, 40, 64, 8),
                                             (3, 2816, 64, 64, 8), (20, 3072, 130, 64, 8), (6, 3328, 64, 64, 8)])
def test_gemm_dynamic_accumulators_and_outputs(M, K, N, bank, topk):
    _say(f"gemm dynamic M={M} K={K} N={N} bank={bank} topk={topk}")
    bits, wq, sw = random_case(1000 + M + K + N, M, K, N, outliers=min(6, K // 16))
    enc = oracle.encode(bits, bank, topk)
    prod = oracle.gemm(enc, wq, sw)
    p = sq.params(M, K, N, bank, topk, out_dtype=sq.SQ_OUT_F32)
    y, alo, ahi = run_gemm(p, enc, wq, sw, sq.SQ_OUT_F32)
    assert np.array_equal(alo, prod.acc_lo), "acc_lo"
    assert np.array_equal(ahi, prod.acc_hi), "acc_hi"
    assert_outputs_close(y, prod, enc, sw)
    assert np.array_equal(y.view(np.uint32), prod.y32.view(np.uint32)), "fp32 outputs are expected to be bit-identical"
    p16 = sq.params(M, K, N, bank, topk, out_dtype=sq.SQ_OUT_BF16)
    y16, _, _ = run_gemm(p16, enc, wq, sw, sq.SQ_OUT_BF16)
    assert np.array_equal(y16, prod.ybf16)


def test_gemm_extreme_codes_do_not_overflow():
    # every low code +-7, every high code +-127, every weight -8: the largest accumulators K allows
    _say("gemm extreme codes")
    M, K, N, bank, topk = 8, 2048, 64, 64, 16
    x = np.full((M, K), 1.0, np.float32)
    x[:, ::4] = 64.0  # k/b = 1/4 of the channels are the high ones
    x[1::2] *= -1
    bits = f32_to_bf16_bits(x)
    wq = pack_int4(np.full((N, K), -8, np.int8))
    sw = np.full(N, 0.01, np.float32)
    enc = oracle.encode(bits, bank, topk)
    prod = oracle.gemm(enc, wq, sw)
    assert abs(int(prod.acc_lo[0, 0])) == 7 * 8 * (K * 3 // 4) and abs(int(prod.acc_hi[0, 0])) == 127 * 8 * (K // 4)
    p = sq.params(M, K, N, bank, topk, out_dtype=sq.SQ_OUT_F32)
    y, alo, ahi = run_gemm(p, enc, wq, sw, sq.SQ_OUT_F32)
    assert np.array_equal(alo, prod.acc_lo) and np.array_equal(ahi, prod.acc_hi)


def test_gemm_largest_k_extreme_codes():
    """K = 65536 with bank 128 (the longest row the encoder takes), every code at its extreme: the widened
    accumulators reach 7*8*K*3/4*256 = 7.0e8 and 127*8*K/4*16 = 2.7e8, inside INT32."""
    _say("gemm largest K")
    M, K, N, bank, topk = 3, 65536, 40, 128, 32
    x = np.full((M, K), 1.0, np.float32)
    x[:, ::4] = 64.0
    x[1] *= -1
    bits = f32_to_bf16_bits(x)
    wq = pack_int4(np.full((N, K), -8, np.int8))
    sw = np.full(N, 0.01, np.float32)
    enc = oracle.encode(bits, bank, topk)
    prod = oracle.gemm(enc, wq, sw)
    assert abs(int(prod.acc_lo[0, 0])) == 7 * 8 * (K * 3 // 4) and abs(int(prod.acc_hi[0, 0])) == 127 * 8 * (K // 4)
    p = sq.params(M, K, N, bank, topk, out_dtype=sq.SQ_OUT_F32)
    y, alo, ahi = run_gemm(p, enc, wq, sw, sq.SQ_OUT_F32)
    assert np.array_equal(alo, prod.acc_lo) and np.array_equal(ahi, prod.acc_hi)
    assert np.array_equal(y.view(np.uint32), prod.y32.view(np.uint32))


@pytest.mark.parametrize("M,K,N,bank,topk", [(16, 512, 512, 64, 8), (150, 1024, 200, 32, 4), (40, 11008, 64, 64, 8)])
def test_gemm_static(M, K, N, bank, topk):
    _say(f"gemm static M={M} K={K} N={N} bank={bank} topk={topk}")
    bits, wq, sw = random_case(2000 + M + K + N, M, K, N)
    mask = make_static_mask(K, bank, topk, seed=K + 3)
    enc = oracle.encode(bits, bank, topk, static_mask=mask)
    prod = oracle.gemm(enc, wq, sw)
    p = sq.params(M, K, N, bank, topk, mode=sq.SQ_STATIC, out_dtype=sq.SQ_OUT_F32)
    pre = torch.empty(sq.sq_weight_prepack_bytes(p), dtype=torch.uint8, device="cuda")
    wqd, md = dev(wq), dev(mask)
    sq.sq_weight_prepack(p, wqd, mask, md, pre)
    y, alo, ahi = run_gemm(p, enc, wq, sw, sq.SQ_OUT_F32, prepacked=pre, static_mask=mask)
    assert np.array_equal(alo, prod.acc_lo), "acc_lo"
    assert np.array_equal(ahi, prod.acc_hi), "acc_hi"
    assert_outputs_close(y, prod, enc, sw)


def compact_low(enc):
    """The oracle's low codes of the low channels only, ascending channel order, two per byte."""
    flags = ((enc.mask[:, None] >> np.arange(32, dtype=np.uint32)[None, :]) & 1).reshape(-1).astype(bool)
    d = workloads.unpack_int4(enc.d_lo)[:, ~flags]
    return pack_int4(d)


@pytest.mark.parametrize("M,K,N,bank,topk", [(16, 512, 512, 64, 8), (150, 1024, 200, 32, 4), (40, 11008, 64, 64, 8),
                                             (70, 2048, 130, 128, 16), (33, 1024, 96, 64, 2)])
def test_static_reordered_operands(M, K, N, bank, topk):
    """Static mode with both operands reordered by the mask (Algorithm 2's last step; Section 3.3): sq_encode
    writes the low codes of the low channels only, sq_weight_prepack -- from the device copy of the mask alone --
    makes the matching weight columns contiguous, and the low product runs over K - K_hi channels.  The
    accumulators must be the oracle's (disjoint supports: skipping the zeros changes nothing)."""
    _say(f"static reordered M={M} K={K} N={N} bank={bank} topk={topk}")
    bits, wq, sw = random_case(2500 + M + K + N, M, K, N)
    mask = make_static_mask(K, bank, topk, seed=K + 5)
    enc = oracle.encode(bits, bank, topk, static_mask=mask)
    prod = oracle.gemm(enc, wq, sw)
    p = sq.params(M, K, N, bank, topk, mode=sq.SQ_STATIC, out_dtype=sq.SQ_OUT_F32)
    wqd, md = dev(wq), dev(mask)
    pre = torch.empty(sq.sq_weight_prepack_bytes(p), dtype=torch.uint8, device="cuda")
    bad = torch.full((1,), 77, dtype=torch.int32, device="cuda")
    sq.sq_weight_prepack(p, wqd, None, md, pre, bad_banks=bad)   # no host copy of the mask
    # the reordered weights: high columns, then low columns
    flags = ((mask[:, None] >> np.arange(32, dtype=np.uint32)[None, :]) & 1).reshape(-1).astype(bool)
    wfull = workloads.unpack_int4(wq)
    K_hi = K // bank * topk
    pre_h = pre.cpu().numpy()
    assert int(bad.item()) == 0
    assert np.array_equal(pre_h[N * K_hi // 2:].reshape(N, (K - K_hi) // 2), pack_int4(wfull[:, ~flags]))
    # encoder: reordered low part next to the format's arrays
    act = GuardedAct(p, static_mask=md)
    lo = Guarded(sq.sq_lo_compact_bytes(p), torch.uint8)
    act.lo_compact = lo.t
    sq.sq_encode(p, dev(bits), act, static_mask=md)
    torch.cuda.synchronize()
    act.check()
    lo.check()
    assert_encoding_equal(act, enc)
    assert np.array_equal(lo.host(np.uint8).reshape(M, -1), compact_low(enc))
    # product on the reordered operands
    y = Guarded(M * N * 4, torch.float32)
    alo, ahi = Guarded(M * N * 4, torch.int32), Guarded(M * N * 4, torch.int32)
    sq.sq_gemm(p, act, sq.weight(wqd, dev(sw), pre), y.t, None, acc_lo_dbg=alo.t, acc_hi_dbg=ahi.t)
    torch.cuda.synchronize()
    for g in (y, alo, ahi):
        g.check()
    assert np.array_equal(alo.host(np.int32).reshape(M, N), prod.acc_lo), "acc_lo"
    assert np.array_equal(ahi.host(np.int32).reshape(M, N), prod.acc_hi), "acc_hi"
    assert np.array_equal(y.host(np.uint32).reshape(M, N), prod.y32.view(np.uint32))
    # a malformed device mask is reported through bad_banks
    broken = mask.copy()
    broken[0] ^= np.uint32(1 << 5)
    broken[K // 32 - 1] ^= np.uint32(1 << 7)
    sq.sq_weight_prepack(p, wqd, None, dev(broken), pre, bad_banks=bad)
    torch.cuda.synchronize()
    assert int(bad.item()) == 2


@pytest.mark.parametrize("mode", ["dynamic", "static"])
def test_linear_end_to_end(mode):
    _say(f"linear {mode}")
    M, K, N, bank, topk = 70, 1024, 192, 64, 8
    bits, wq, sw = random_case(3000, M, K, N)
    mask = make_static_mask(K, bank, topk, seed=9) if mode == "static" else None
    enc = oracle.encode(bits, bank, topk, static_mask=mask)
    prod = oracle.gemm(enc, wq, sw)
    p = sq.params(M, K, N, bank, topk, mode=sq.SQ_STATIC if mask is not None else sq.SQ_DYNAMIC, out_dtype=sq.SQ_OUT_BF16)
    xd, wqd, swd = dev(bits), dev(wq), dev(sw)
    md = None if mask is None else dev(mask)
    pre = None
    if mask is not None:
        pre = torch.empty(sq.sq_weight_prepack_bytes(p), dtype=torch.uint8, device="cuda")
        sq.sq_weight_prepack(p, wqd, mask, md, pre)
    w = sq.weight(wqd, swd, pre)
    y = Guarded(M * N * 2, torch.int16)
    ws = Guarded(sq.sq_linear_workspace_bytes(p), torch.uint8)
    sq.sq_linear(p, xd, w, y.t, ws.t, static_mask=md)
    torch.cuda.synchronize()
    y.check()
    ws.check()
    assert np.array_equal(y.host(np.uint16).reshape(M, N), prod.ybf16)


def test_dense_w4a8_reference_kernel():
    _say("dense w4a8")
    rng = np.random.default_rng(77)
    M, K, N = 100, 768, 140
    a = rng.integers(-127, 128, size=(M, K)).astype(np.int8)
    sa = rng.uniform(0.01, 0.1, M).astype(np.float32)
    w = rng.integers(-8, 8, size=(N, K)).astype(np.int8)
    sw = rng.uniform(0.005, 0.02, N).astype(np.float32)
    p = sq.params(M, K, N, out_dtype=sq.SQ_OUT_F32)
    wqd, swd = dev(pack_int4(w)), dev(sw)
    pre = torch.empty(N * K // 2, dtype=torch.uint8, device="cuda")
    sq.sq_dense_w4a8_prepack(p, wqd, pre)
    y = Guarded(M * N * 4, torch.float32)
    sq.sq_dense_w4a8_gemm(p, dev(a), dev(sa), sq.weight(wqd, swd, pre), y.t)
    torch.cuda.synchronize()
    y.check()
    acc = a.astype(np.int64) @ w.astype(np.int64).T
    want = (acc.astype(np.float32) * sa[:, None]).astype(np.float32) * sw[None, :]
    assert np.array_equal(y.host(np.float32).reshape(M, N), want.astype(np.float32))


def expected_hi_dense(enc):
    """The documented image: INT8 codes at their channels, zero elsewhere; inside every group of
    8 channels the even channels come first, then the odd ones."""
    M, K = enc.M, enc.K
    dense = np.zeros((M, K), np.int8)
    flags = ((enc.mask[:, :, None] >> np.arange(32, dtype=np.uint32)[None, None, :]) & 1).reshape(M, K).astype(bool)
    for m in range(M):
        dense[m, flags[m]] = enc.hi_val[m].reshape(-1)
    g = dense.reshape(M, K // 8, 8)
    return np.concatenate([g[:, :, 0::2], g[:, :, 1::2]], axis=2).reshape(M, K)


@pytest.mark.parametrize("K,bank,topk", [(1024, 64, 8), (512, 32, 4), (2048, 128, 32), (11008, 64, 8)])
def test_hi_dense_image_from_encoder_and_from_gemm_workspace(K, bank, topk):
    _say(f"hi_dense K={K} bank={bank} topk={topk}")
    M, N = 19, 64
    bits, wq, sw = random_case(4000 + K, M, K, N)
    enc = oracle.encode(bits, bank, topk)
    want = expected_hi_dense(enc)
    p = sq.params(M, K, N, bank, topk, out_dtype=sq.SQ_OUT_F32)
    # written by the encoder
    act = sq.Act(p, with_hi_dense=True)
    sq.sq_encode(p, dev(bits), act)
    torch.cuda.synchronize()
    assert_encoding_equal(act, enc)
    assert np.array_equal(act.hi_dense.cpu().numpy().reshape(M, K), want)
    # built by sq_gemm in its workspace when the caller has none
    act2 = sq.Act(p)
    sq.sq_encode(p, dev(bits), act2)
    ws = torch.empty(sq.sq_gemm_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    y1 = torch.empty(M * N, dtype=torch.float32, device="cuda")
    y2 = torch.empty(M * N, dtype=torch.float32, device="cuda")
    w = sq.weight(dev(wq), dev(sw))
    sq.sq_gemm(p, act2, w, y1, ws)
    sq.sq_gemm(p, act, w, y2, None)
    torch.cuda.synchronize()
    assert np.array_equal(ws[:M * K].cpu().numpy().view(np.int8).reshape(M, K), want)
    assert torch.equal(y1, y2)
    assert np.array_equal(y1.cpu().numpy().reshape(M, N).view(np.uint32), oracle.gemm(enc, wq, sw).y32.view(np.uint32))


@pytest.mark.parametrize("mode", ["dynamic", "tied", "static"])
def test_encode_padded_rows_of_x_on_the_streaming_kernels(mode):
    """ldx > K on the kernels that copy rows into LDS (K = 4096: a unit of the streaming kernel lies inside one
    row; the static kernel stages whole rows): the padding holds +inf and must never be read as data."""
    _say(f"encode ldx {mode}")
    M, K, bank, topk, ldx = 70, 4096, 64, 8, 4096 + 24
    bits, _, _ = random_case(77, M=M, K=K, N=8)
    if mode == "static":
        mask = make_static_mask(K, bank, topk, seed=3)
        p, act = run_encode(bits, bank, topk, static_mask=mask, ldx=ldx)
        assert_encoding_equal(act, oracle.encode(bits, bank, topk, static_mask=mask))
        return
    padded = np.full((M, ldx), 0x7F80, np.uint16)
    padded[:, :K] = bits
    lib_mode = sq.SQ_DYNAMIC if mode == "dynamic" else sq.SQ_DYNAMIC_TIED
    p = sq.params(M, K, 64, bank, topk, mode=lib_mode)
    act = GuardedAct(p)
    sq.sq_encode(p, dev(padded), act, ldx=ldx)
    torch.cuda.synchronize()
    act.check()
    assert_encoding_equal(act, oracle.encode(bits, bank, topk) if mode == "dynamic" else oracle.encode_tied(bits, bank, topk))


@pytest.mark.parametrize("K,bank,topk", [(28672, 64, 8), (49152, 128, 16)])
def test_static_long_rows(K, bank, topk):
    """Static mode on long rows: 28672 channels take the row-staged encoder's larger instantiation and the reordered
    operands; 49152 channels do not fit in LDS, so sq_linear falls back to the dense low part (and sq_encode
    refuses lo_compact)."""
    _say(f"static long rows K={K}")
    M, N = 9, 96
    bits, wq, sw = random_case(5100 + K, M, K, N, outliers=8)
    mask = make_static_mask(K, bank, topk, seed=K)
    enc = oracle.encode(bits, bank, topk, static_mask=mask)
    prod = oracle.gemm(enc, wq, sw)
    p = sq.params(M, K, N, bank, topk, mode=sq.SQ_STATIC, out_dtype=sq.SQ_OUT_F32)
    xd, wqd, swd, md = dev(bits), dev(wq), dev(sw), dev(mask)
    pre = torch.empty(sq.sq_weight_prepack_bytes(p), dtype=torch.uint8, device="cuda")
    sq.sq_weight_prepack(p, wqd, None, md, pre)
    act = GuardedAct(p, static_mask=md)
    sq.sq_encode(p, xd, act, static_mask=md)
    torch.cuda.synchronize()
    act.check()
    assert_encoding_equal(act, enc)
    if K > 40000:
        act.lo_compact = torch.empty(sq.sq_lo_compact_bytes(p), dtype=torch.uint8, device="cuda")
        with pytest.raises(sq.SqError) as e:
            sq.sq_encode(p, xd, act, static_mask=md)
        assert e.value.status == -3
    y = Guarded(M * N * 4, torch.float32)
    ws = Guarded(sq.sq_linear_workspace_bytes(p), torch.uint8)
    sq.sq_linear(p, xd, sq.weight(wqd, swd, pre), y.t, ws.t, static_mask=md)
    torch.cuda.synchronize()
    y.check()
    ws.check()
    assert np.array_equal(y.host(np.uint32).reshape(M, N), prod.y32.view(np.uint32))


@pytest.mark.parametrize("M,K,N", [(1, 1024, 200), (8, 2048, 130), (32, 1280, 96)])
def test_static_decode_shapes_take_the_streaming_kernel(M, K, N):
    """Static mode with at most 32 tokens: given a workspace, sq_gemm builds the image of the high part from
    hi_val and the channel mask and runs the weight-streaming kernel on the dense low part: same accumulators,
    same outputs as the oracle; without a workspace the generic tile gives the same bytes."""
    _say(f"static decode M={M} K={K} N={N}")
    bank, topk = 64, 8
    bits, wq, sw = random_case(2700 + M + K + N, M, K, N, outliers=4)
    mask = make_static_mask(K, bank, topk, seed=K + 7)
    enc = oracle.encode(bits, bank, topk, static_mask=mask)
    prod = oracle.gemm(enc, wq, sw)
    p = sq.params(M, K, N, bank, topk, mode=sq.SQ_STATIC, out_dtype=sq.SQ_OUT_F32)
    assert sq.sq_gemm_workspace_bytes(p) >= M * K
    wqd, md = dev(wq), dev(mask)
    pre = torch.empty(sq.sq_weight_prepack_bytes(p), dtype=torch.uint8, device="cuda")
    sq.sq_weight_prepack(p, wqd, None, md, pre)
    y, alo, ahi = run_gemm(p, enc, wq, sw, sq.SQ_OUT_F32, prepacked=pre, static_mask=mask)   # passes a workspace
    assert np.array_equal(alo, prod.acc_lo) and np.array_equal(ahi, prod.acc_hi)
    assert np.array_equal(y.view(np.uint32), prod.y32.view(np.uint32))
    act = sq.Act(p, static_mask=md)
    act.d_lo.copy_(dev(enc.d_lo).view(-1))
    act.hi_val.copy_(dev(enc.hi_val).view(-1))
    act.scale_lo.copy_(dev(enc.s_lo))
    act.scale_hi.copy_(dev(enc.s_hi))
    y2 = Guarded(M * N * 4, torch.float32)
    sq.sq_gemm(p, act, sq.weight(wqd, dev(sw), pre), y2.t, None)
    torch.cuda.synchronize()
    y2.check()
    assert np.array_equal(y2.host(np.uint32).reshape(M, N), prod.y32.view(np.uint32))

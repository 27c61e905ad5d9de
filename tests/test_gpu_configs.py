"""GPU parity at the benchmark configurations' full sizes, in the launch configuration bench.py times.

The packed encoding is compared with the oracle's for every row.  Accumulators and outputs are compared with the
oracle's on sampled rows, all N columns: at least one row in every band of 128 rows (every row of workgroup
tiles), the first and the last row.  The oracle's integer product is too slow for all rows, so every other
element is covered by properties that hold at any size: both accumulators of the WHOLE matrix must equal an fp32
library matmul of the oracle's own codes (integer products and partial sums below 2^24 are exact in fp32 in any
summation order), and every output must lie within the rounding bound of the fp64 evaluation of the definition.
The output buffers are pre-filled with a canary.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2512_05409_amd as sq
import workloads
from gpu_util import assert_encoding_equal, assert_outputs_close, dev

pytestmark = pytest.mark.gpu

# the whole-matrix check relies on exact fp32 products and sums of small integers
torch.backends.cuda.matmul.allow_tf32 = False


def _say(msg):
    print(msg, flush=True)


def sample_rows(M, n, seed):
    """One random row in every band of 128 rows, plus the first and the last row (and at least n rows)."""
    if M <= n:
        return np.arange(M)
    rng = np.random.default_rng(seed)
    rows = {0, M - 1}
    for b0 in range(0, M, 128):
        rows.add(int(rng.integers(b0, min(b0 + 128, M))))
    while len(rows) < n:
        rows.add(int(rng.integers(0, M)))
    return np.array(sorted(rows))


CANARY16 = -23131  # 0xA5A5 as int16


def unpack_int4_device(packed, rows, cols):
    """[rows, cols/2] bytes on the device -> [rows, cols] fp32 integers in [-8, 7] (test-side container conversion)."""
    p = packed.view(torch.uint8).view(rows, cols // 2).to(torch.int16)
    lo, hi = p & 0xF, p >> 4
    lo = torch.where(lo >= 8, lo - 16, lo)
    hi = torch.where(hi >= 8, hi - 16, hi)
    return torch.stack((lo, hi), dim=2).view(rows, cols).to(torch.float32)


def whole_matrix_check(enc, wl, alo, ahi, y, out_bf16):
    """Every element: accumulators against an fp32 library matmul of the ORACLE's codes, outputs against the
    fp64 evaluation of the definition within three fp32 roundings (plus half a bf16 step for bf16 output)."""
    M, K, N = wl.M, wl.K, wl.N
    Wf = unpack_int4_device(dev(wl.wq_packed), N, K)
    D = unpack_int4_device(dev(enc.d_lo), M, K)
    want_lo = (D @ Wf.T)
    assert float(want_lo.abs().max()) < 2 ** 24
    assert torch.equal(alo.view(M, N), want_lo.to(torch.int32)), "acc_lo differs somewhere in the whole matrix"
    del D, want_lo
    # dense image of the oracle's high part, built from its mask and compact codes
    G = K // enc.bank
    if enc.mode == 0:
        flags = ((enc.mask[:, :, None] >> np.arange(32, dtype=np.uint32)[None, None, :]) & 1).reshape(M, K).astype(bool)
    else:
        flags = np.broadcast_to(((enc.mask[:, None] >> np.arange(32, dtype=np.uint32)[None, :]) & 1).reshape(1, K).astype(bool), (M, K))
    H = np.zeros((M, K), np.float32)
    H[flags] = enc.hi_val.reshape(-1)
    want_hi = dev(H) @ Wf.T
    assert float(want_hi.abs().max()) < 2 ** 24
    assert torch.equal(ahi.view(M, N), want_hi.to(torch.int32)), "acc_hi differs somewhere in the whole matrix"
    del want_hi, Wf
    slo, shi, sw = dev(enc.s_lo).double(), dev(enc.s_hi).double(), dev(wl.w_scale).double()
    lo = alo.view(M, N).double() * slo[:, None]
    hi = ahi.view(M, N).double() * shi[:, None]
    y64 = (lo + hi) * sw[None, :]
    bound = 4.0 * 2.0 ** -24 * (lo.abs() + hi.abs()) * sw.abs()[None, :]
    del lo, hi
    if out_bf16:
        yv = (y.view(torch.int16).view(M, N).to(torch.int32) << 16).view(torch.float32).double()
        bound = bound + 2.0 ** -8 * y64.abs()
    else:
        yv = y.view(M, N).double()
    assert bool(((yv - y64).abs() <= bound).all()), "an output is off the fp64 value of the definition"


def run_config(wl, n_rows, out_dtype=sq.SQ_OUT_BF16, mask=None):
    M, K, N = wl.M, wl.K, wl.N
    mode = sq.SQ_STATIC if mask is not None else sq.SQ_DYNAMIC
    p = sq.params(M, K, N, wl.bank, wl.topk, mode=mode, out_dtype=out_dtype)
    _say(f"  oracle encode {wl.name} M={M} K={K}")
    enc = oracle.encode(wl.x_bits, wl.bank, wl.topk, static_mask=mask)
    xd, wqd, swd = dev(wl.x_bits), dev(wl.wq_packed), dev(wl.w_scale)
    md = None if mask is None else dev(mask)
    pre = None
    if mask is not None:
        pre = torch.empty(sq.sq_weight_prepack_bytes(p), dtype=torch.uint8, device="cuda")
        sq.sq_weight_prepack(p, wqd, mask, md, pre)
    w = sq.weight(wqd, swd, pre)
    # 1. encode alone: every row
    act = sq.Act(p, static_mask=md)
    sq.sq_encode(p, xd, act, static_mask=md)
    torch.cuda.synchronize()
    assert_encoding_equal(act, enc)
    # 2. gemm on that encoding, with the accumulators dumped
    esz = 4 if out_dtype == sq.SQ_OUT_F32 else 2
    if esz == 4:
        y = torch.full((M * N,), float("nan"), dtype=torch.float32, device="cuda")
    else:
        y = torch.full((M * N,), CANARY16, dtype=torch.int16, device="cuda")
    alo = torch.full((M * N,), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
    ahi = torch.full((M * N,), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
    ws = torch.empty(sq.sq_gemm_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    _say(f"  gpu gemm ({sq.sq_gemm_variant(p)})")
    sq.sq_gemm(p, act, w, y, ws, acc_lo_dbg=alo, acc_hi_dbg=ahi)
    torch.cuda.synchronize()
    _say("  whole-matrix check")
    whole_matrix_check(enc, wl, alo, ahi, y, esz == 2)
    rows = sample_rows(M, n_rows, seed=M + N)
    _say(f"  oracle gemm on {len(rows)} rows")
    prod = oracle.gemm(enc.rows(rows), wl.wq_packed, wl.w_scale)
    rd = torch.from_numpy(rows).cuda()
    assert np.array_equal(alo.view(M, N)[rd].cpu().numpy(), prod.acc_lo), "acc_lo"
    assert np.array_equal(ahi.view(M, N)[rd].cpu().numpy(), prod.acc_hi), "acc_hi"
    yh = y.view(M, N)[rd].cpu().numpy()
    if esz == 4:
        assert_outputs_close(yh, prod, enc.rows(rows), wl.w_scale)
    else:
        assert np.array_equal(yh.view(np.uint16), prod.ybf16), "bf16 outputs"
    del alo, ahi
    # 3. the fused entry point the benchmark times must give the same bytes as encode + gemm
    y2 = torch.full_like(y, 1)
    lws = torch.empty(sq.sq_linear_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    _say("  gpu linear")
    sq.sq_linear(p, xd, w, y2, lws, static_mask=md)
    torch.cuda.synchronize()
    assert torch.equal(y, y2), "sq_linear != sq_encode + sq_gemm"


def test_config1_tiny():
    _say("config 1")
    run_config(workloads.make("c1_tiny"), n_rows=16, out_dtype=sq.SQ_OUT_F32)
    run_config(workloads.make("c1_tiny"), n_rows=16, out_dtype=sq.SQ_OUT_BF16)


def test_config2_qkv7b():
    _say("config 2")
    run_config(workloads.make("c2_qkv7b"), n_rows=12)


@pytest.mark.parametrize("bank,topk", [(64, 8), (32, 2), (32, 4), (32, 8), (64, 4), (64, 16), (128, 8), (128, 16), (128, 32)])
def test_config3_mlp7b(bank, topk):
    _say(f"config 3 bank={bank} topk={topk}")
    # the (b, k) sweep reuses the shape with a reduced N except for the headline setting
    N = None if (bank, topk) == (64, 8) else 2048
    run_config(workloads.make("c3_mlp7b", bank=bank, topk=topk, N=N), n_rows=8)


def test_config4_down7b_static():
    _say("config 4")
    wl = workloads.make("c4_down7b_static")
    mask, _ = oracle.static_mask(wl.calib_bits, wl.wq_packed, wl.w_scale, wl.bank, wl.topk)
    run_config(wl, n_rows=8, mask=mask)


@pytest.mark.parametrize("M", [1, 8, 64, 8192])
def test_config5_up70b(M):
    _say(f"config 5 M={M}")
    run_config(workloads.make("c5_up70b", M=M), n_rows=6)


@pytest.mark.parametrize("name,M", [("c3_mlp7b", None), ("c5_up70b", 8), ("c5_up70b", 64), ("c4_down7b_static", None)])
def test_full_size_runs_are_reproducible(name, M):
    """The kernels use no atomics on the output path: repeated launches at full size, with every compute unit
    busy, must give the same bytes (a hazard between pipeline stages would show up as a difference)."""
    _say(f"reproducibility {name} M={M}")
    wl = workloads.make(name) if M is None else workloads.make(name, M=M)
    static = wl.mode == "static"
    p = sq.params(wl.M, wl.K, wl.N, wl.bank, wl.topk, mode=sq.SQ_STATIC if static else sq.SQ_DYNAMIC,
                  out_dtype=sq.SQ_OUT_BF16)
    xd, wqd, swd = dev(wl.x_bits), dev(wl.wq_packed), dev(wl.w_scale)
    md, pre = None, None
    if static:
        mask, _ = oracle.static_mask(wl.calib_bits, wl.wq_packed, wl.w_scale, wl.bank, wl.topk)
        md = dev(mask)
        pre = torch.empty(sq.sq_weight_prepack_bytes(p), dtype=torch.uint8, device="cuda")
        sq.sq_weight_prepack(p, wqd, mask, md, pre)
    w = sq.weight(wqd, swd, pre)
    ws = torch.empty(sq.sq_linear_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    ys = [torch.empty(wl.M * wl.N, dtype=torch.int16, device="cuda") for _ in range(2)]
    sq.sq_linear(p, xd, w, ys[0], ws, static_mask=md)
    for rep in range(4):
        sq.sq_linear(p, xd, w, ys[1], ws, static_mask=md)
        torch.cuda.synchronize()
        assert torch.equal(ys[0], ys[1]), f"launch {rep + 2} differs from the first"
        ys[1].zero_()

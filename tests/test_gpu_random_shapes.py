"""Seeded sweep over legal shapes and format parameters: sq_linear against the oracle, bit for bit.

The shapes are drawn, not hand-picked, so that tile edges, K tails and every kernel variant (the three GEMM
tiles, the weight-streaming kernel, both encoders) meet combinations nobody thought of; the sizes are small
enough for the oracle to take a fraction of a second each."""
import numpy as np
import pytest
import torch

import oracle
import paper_2512_05409_amd as sq
import workloads
from gpu_util import Guarded, dev

pytestmark = pytest.mark.gpu

FORMATS = [(32, 2), (32, 4), (32, 8), (32, 16), (64, 4), (64, 8), (64, 16), (64, 32), (128, 8), (128, 16), (128, 32)]


def draw_case(rng):
    bank, topk = FORMATS[rng.integers(len(FORMATS))]
    static = bool(rng.integers(2))
    unit = 128 if bank == 128 else 64
    while True:
        K = int(rng.integers(1, 20)) * unit
        if K // bank > 512:
            continue
        if static and ((K // bank) * topk) % 32:
            continue
        break
    M = int(rng.choice([1, 2, 7, 16, 31, 32, 33, 40, 64, 65, 100, 128, 129, 200, 257, 300]))
    N = int(rng.choice([1, 5, 31, 32, 64, 65, 100, 127, 128, 130, 255, 256, 257, 300, 513]))
    return M, K, N, bank, topk, static


@pytest.mark.parametrize("seed", range(24))
def test_random_shape(seed):
    rng = np.random.Generator(np.random.PCG64([seed, 4242]))
    M, K, N, bank, topk, static = draw_case(rng)
    print(f"seed {seed}: M={M} K={K} N={N} bank={bank} topk={topk} {'static' if static else 'dynamic'}", flush=True)
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[:, rng.choice(K, max(1, K // 64), replace=False)] *= 25.0
    if M > 2:
        x[1] = rng.choice(np.array([0.0, 0.5, -0.5, 1.0, 2.0, -2.0], np.float32), size=K)  # heavy ties
        x[2] = 0.0
    bits = workloads.f32_to_bf16_bits(x)
    wq = workloads.pack_int4(rng.integers(-8, 8, size=(N, K), dtype=np.int8))
    sw = rng.uniform(0.005, 0.02, size=N).astype(np.float32)
    mask = None
    if static:
        mask = np.zeros(K // 32, np.uint32)
        for g in range(K // bank):
            for i in rng.choice(bank, topk, replace=False):
                j = g * bank + int(i)
                mask[j // 32] |= np.uint32(1 << (j % 32))
    enc = oracle.encode(bits, bank, topk, static_mask=mask)
    ref = oracle.gemm(enc, wq, sw)

    out_dtype = sq.SQ_OUT_F32 if seed % 2 == 0 else sq.SQ_OUT_BF16
    p = sq.params(M, K, N, bank, topk, mode=sq.SQ_STATIC if static else sq.SQ_DYNAMIC, out_dtype=out_dtype)
    wqd, swd = dev(wq), dev(sw)
    md, pre = None, None
    if static:
        md = dev(mask)
        pre = torch.empty(max(16, sq.sq_weight_prepack_bytes(p)), dtype=torch.uint8, device="cuda")
        sq.sq_weight_prepack(p, wqd, mask, md, pre)
    w = sq.weight(wqd, swd, pre)
    esz = 4 if out_dtype == sq.SQ_OUT_F32 else 2
    y = Guarded(M * N * esz, torch.float32 if esz == 4 else torch.int16)
    ws = Guarded(sq.sq_linear_workspace_bytes(p), torch.uint8)
    sq.sq_linear(p, dev(bits), w, y.t, ws.t, static_mask=md)
    torch.cuda.synchronize()
    y.check(), ws.check()
    if esz == 4:
        assert np.array_equal(y.host(np.uint32).reshape(M, N), ref.y32.view(np.uint32))
    else:
        assert np.array_equal(y.host(np.uint16).reshape(M, N), ref.ybf16)

"""sq_linear_noalloc (the entry point for callers that cannot allocate: its workspace is a fixed device array
inside the library) against sq_linear with a caller-allocated workspace: identical bytes, on two calls in a
row, the second with a smaller input (the array then still holds the first call's encoding), and against the
CPU oracle.  Problems beyond the array's size are refused before anything is launched."""
import numpy as np
import pytest
import torch

import oracle
import paper_2512_05409_amd as sq
from gpu_util import Guarded, dev
from test_gpu_parity import make_static_mask, random_case

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def run_pair(M, K, N, bank, topk, mode, out_dtype, seed):
    bits, wq, sw = random_case(seed, M, K, N, outliers=4)
    static = mode == "static"
    p = sq.params(M, K, N, bank, topk, mode=sq.SQ_STATIC if static else sq.SQ_DYNAMIC, out_dtype=out_dtype)
    assert sq.sq_linear_workspace_bytes(p) <= sq.SQ_NOALLOC_SCRATCH_BYTES
    xd, wqd, swd = dev(bits), dev(wq), dev(sw)
    mask, md, pre = None, None, None
    if static:
        mask = make_static_mask(K, bank, topk, seed=seed + 1)
        md = dev(mask)
        pre = torch.empty(sq.sq_weight_prepack_bytes(p), dtype=torch.uint8, device="cuda")
        sq.sq_weight_prepack(p, wqd, mask, md, pre)
    w = sq.weight(wqd, swd, pre)
    esz = 4 if out_dtype == sq.SQ_OUT_F32 else 2
    tdt = torch.float32 if esz == 4 else torch.int16
    y_ref = Guarded(M * N * esz, tdt)
    ws = torch.empty(sq.sq_linear_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    sq.sq_linear(p, xd, w, y_ref.t, ws, static_mask=md)
    y_new = Guarded(M * N * esz, tdt)
    sq.sq_linear_noalloc(p, xd, w, y_new.t, static_mask=md)
    torch.cuda.synchronize()
    y_ref.check()
    y_new.check()
    assert torch.equal(y_ref.t, y_new.t), "sq_linear_noalloc differs from sq_linear"
    prod = oracle.gemm(oracle.encode(bits, bank, topk, static_mask=mask), wq, sw)
    if esz == 4:
        assert np.array_equal(y_new.host(np.uint32).reshape(M, N), prod.y32.view(np.uint32))
    else:
        assert np.array_equal(y_new.host(np.uint16).reshape(M, N), prod.ybf16)


@pytest.mark.parametrize("mode", ["dynamic", "static"])
def test_two_calls_in_a_row_second_smaller(mode):
    _say(f"noalloc {mode}: first call M=300 K=2048 N=700")
    run_pair(300, 2048, 700, 64, 8, mode, sq.SQ_OUT_F32, seed=91)
    _say(f"noalloc {mode}: second call M=24 K=1024 N=200 (smaller, same scratch)")
    run_pair(24, 1024, 200, 64, 8, mode, sq.SQ_OUT_BF16, seed=92)
    _say(f"noalloc {mode}: third call M=50 K=512 N=130 bank 32")
    run_pair(50, 512, 130, 32, 4, mode, sq.SQ_OUT_F32, seed=93)


def test_problem_beyond_the_scratch_is_refused():
    _say("noalloc: too large")
    p = sq.params(4096, 4096, 512, 64, 8)
    assert sq.sq_linear_workspace_bytes(p) > sq.SQ_NOALLOC_SCRATCH_BYTES
    x = torch.zeros(16, dtype=torch.int16, device="cuda")  # never read: the call must fail before any launch
    wq = torch.zeros(16, dtype=torch.uint8, device="cuda")
    sw = torch.zeros(16, dtype=torch.float32, device="cuda")
    y = torch.full((16,), 7, dtype=torch.int16, device="cuda")
    with pytest.raises(sq.SqError) as e:
        sq.sq_linear_noalloc(p, x, sq.weight(wq, sw), y)
    assert e.value.status == -8 and "SQ_ERR_SCRATCH" in str(e.value)
    torch.cuda.synchronize()
    assert bool((y == 7).all())
    # invalid parameters are still reported as such
    with pytest.raises(sq.SqError) as e:
        sq.sq_linear_noalloc(sq.params(8, 100, 64), x, sq.weight(wq, sw), y)
    assert e.value.status == -2

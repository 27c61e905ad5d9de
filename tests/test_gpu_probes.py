"""The measurement probes for the chip's other matrix paths (the reasons the FP6 and the structured-sparse routes of
the second "next" row are judged on): the FP6 E3M2 path multiplies INT4-range integers exactly while sums stay
below 2^24, and both rate probes run."""
import numpy as np
import pytest
import torch

import paper_2512_05409_amd as sq

pytestmark = pytest.mark.gpu

# E3M2 (1 sign, 3 exponent, 2 mantissa bits, bias 3): code of the integer magnitudes 0 ... 8
E3M2 = [0, 12, 16, 18, 20, 21, 22, 23, 24]


def e3m2(v: int) -> int:
    return (32 if v < 0 else 0) | E3M2[abs(v)]


def pack_operand(mat_rows_by_k: np.ndarray) -> np.ndarray:
    """[32, 64] integers -> the 64 lanes x 8 dwords of one operand (lane l: row l % 32, K slots 32*(l/32) ... +31)."""
    out = np.zeros((64, 8), np.uint64)
    for lane in range(64):
        for t in range(32):
            code = e3m2(int(mat_rows_by_k[lane % 32, 32 * (lane // 32) + t]))
            bit = 6 * t
            w, sh = bit // 32, bit % 32
            out[lane, w] |= (code << sh) & 0xFFFFFFFF
            if sh > 26:
                out[lane, w + 1] |= code >> (32 - sh)
    return out.astype(np.uint32)


def run_tile(A, B, c0=0.0, reps=1):
    a = torch.from_numpy(pack_operand(A).view(np.int32)).cuda()
    b = torch.from_numpy(pack_operand(B.T.copy()).view(np.int32)).cuda()
    c = torch.zeros(64 * 16, dtype=torch.float32, device="cuda")
    sq.sq_probe_fp6_tile(a, b, c, c0, reps)
    torch.cuda.synchronize()
    raw = c.cpu().numpy().reshape(64, 16)
    out = np.zeros((32, 32), np.float64)
    for lane in range(64):
        for r in range(16):
            out[8 * (r // 4) + 4 * (lane // 32) + r % 4, lane % 32] = raw[lane, r]
    return out


@pytest.mark.parametrize("case", ["random int4", "extreme", "chain of 3000", "large start"])
def test_fp6_path_multiplies_int4_codes_exactly(case):
    print("fp6 tile:", case, flush=True)
    rng = np.random.default_rng(11)
    c0, reps = 0.0, 1
    if case == "random int4":
        A, B = rng.integers(-8, 8, (32, 64)), rng.integers(-8, 8, (64, 32))
    elif case == "extreme":
        A = np.where((np.add.outer(np.arange(32), np.arange(64)) & 1) == 1, 8, -8)
        B = np.where((np.arange(64)[:, None] & 1) == 1, -8, 7) * np.ones((1, 32), np.int64)
    elif case == "chain of 3000":
        A, B = np.full((32, 64), -8), np.full((64, 32), 8)
        reps = 3000  # 3000 * 64 * 64 = 12.3 M < 2^24
    else:
        A, B = rng.integers(-1, 2, (32, 64)), rng.integers(-1, 2, (64, 32))
        c0 = 16000000.0
    want = c0 + reps * (A.astype(np.int64) @ B.astype(np.int64))
    assert np.abs(want).max() < 2 ** 24
    got = run_tile(A, B, c0, reps)
    assert np.array_equal(got, want.astype(np.float64))


def test_rate_probes_run():
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    sink = torch.zeros(2 * n_cu * 256, dtype=torch.int32, device="cuda")
    for kind in (0, 1):
        sq.sq_probe_mfma_alt(kind, 2 * n_cu, 64, sink)
    torch.cuda.synchronize()
    with pytest.raises(sq.SqError):
        sq.sq_probe_mfma_alt(2, 8, 64, sink)

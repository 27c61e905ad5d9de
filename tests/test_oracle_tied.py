"""Pins for the tied-scale oracle (oracle/tied.py): one scale step for both parts, s_lo = 16 * s_hi, one INT8
operand, one accumulator.  Hand-built rows, invariants, the two-scale oracle's mask and products on the same
codes, numpy's integer matmul, the k = b reduction to plain per-token INT8, and planted mistakes."""
import os
import subprocess
import sys

import numpy as np
import pytest

import oracle
from workloads import f32_to_bf16_bits, bf16_bits_to_f32, pack_int4, unpack_int4, make

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def row_with(values, K=64, fill=0.0):
    x = np.full((1, K), fill, np.float32)
    x[0, :len(values)] = values
    return f32_to_bf16_bits(x)


def test_scale_one_row_by_hand():
    # one bank of 64, k = 2: the two largest magnitudes are 127 and 100.5 (high; 100.5 is half-way -> 100, the
    # even neighbour); the largest low value is 88
    # -> A = max(127, 56*127/112 = 63.5) = 127, s_hi = 1, s_lo = 16: h = rne(x), d = rne(x / 16).
    vals = [127, 100.5, 56, 8, 24, 40, -24, -8, 7.5, 88, 0.5, 15.9375]
    # x/16:            3.5 0.5 1.5 2.5 -1.5 -0.5 .47 5.5 .03 .996
    enc = oracle.encode_tied(row_with(vals), 64, 2)
    assert enc.s_hi[0] == 1.0 and enc.s_lo[0] == 16.0
    assert int(enc.mask[0, 0]) == 0b11 and int(enc.mask[0, 1]) == 0
    assert list(enc.hi_val[0, 0]) == [127, 100]
    d = unpack_int4(enc.d_lo)[0]
    assert list(d[:12]) == [0, 0, 4, 0, 2, 2, -2, 0, 0, 6, 0, 1]  # half-way cases go to the even code
    assert list(enc.codes[0, :12]) == [127, 100, 64, 0, 32, 32, -32, 0, 0, 96, 0, 16]
    assert not enc.codes[0, 12:].any()


def test_low_part_sets_the_scale_when_it_is_large():
    # high values 100 and 90, largest low value 89.25 (exact in bf16 here: 89.25 = 357/4):
    # 89.25*127/112 = 101.2 > 100 -> A = fl32(89.25 * fl32(127/112)); the low code of 89.25 must be 7, unclipped
    vals = [100, 90, 89.0, -89.0, 44.5]
    bits = row_with(vals)
    enc = oracle.encode_tied(bits, 64, 2)
    A = np.float32(np.float32(89.0) * (np.float32(127.0) / np.float32(112.0)))
    assert A > 100
    assert enc.s_hi[0] == np.float32(A / np.float32(127.0))
    assert enc.s_lo.view(np.uint32)[0] == np.float32(enc.s_hi[0] * np.float32(16)).view(np.uint32)
    d = unpack_int4(enc.d_lo)[0]
    assert list(d[:5]) == [0, 0, 7, -7, 4]          # 44.5 / (16 s_hi) = 3.5 -> 4 (even)
    assert list(enc.hi_val[0, 0]) == [int(np.rint(np.float32(100) * np.float32(np.float32(127) / A))),
                                      int(np.rint(np.float32(90) * np.float32(np.float32(127) / A)))]


def test_zero_row_and_all_equal_row():
    enc = oracle.encode_tied(row_with([], K=128), 64, 8)
    assert enc.s_hi[0] == 1.0 and enc.s_lo[0] == 16.0 and not enc.codes.any() and not enc.d_lo.any()
    assert int(enc.mask[0, 0]) == 0xFF and int(enc.mask[0, 2]) == 0xFF  # first k channels of each bank
    enc = oracle.encode_tied(row_with([], K=64, fill=3.0), 64, 8)
    # all equal: A = 3 * 127/112 rounded; high codes rne(3 * 127 / A) = 112, low codes 7
    assert (enc.hi_val[0, 0] == 112).all()
    assert (unpack_int4(enc.d_lo)[0, 8:] == 7).all()


@pytest.mark.parametrize("bank,topk", [(64, 8), (32, 4), (128, 16), (64, 16)])
def test_invariants_and_mask_equals_two_scale_rule(bank, topk):
    wl = make("c1_tiny", bank=bank, topk=topk)
    enc = oracle.encode_tied(wl.x_bits, bank, topk)
    two = oracle.encode(wl.x_bits, bank, topk)
    assert np.array_equal(enc.mask, two.mask)                      # same selection rule
    assert np.array_equal(enc.s_lo.view(np.uint32), (enc.s_hi * np.float32(16)).astype(np.float32).view(np.uint32))
    flags = ((enc.mask[:, :, None] >> np.arange(32, dtype=np.uint32)[None, None, :]) & 1).reshape(enc.M, enc.K).astype(bool)
    d = unpack_int4(enc.d_lo).astype(np.int32)
    assert np.abs(d).max() <= 7 and not d[flags].any()
    assert np.abs(enc.hi_val.astype(np.int32)).max() <= 127
    H = np.zeros((enc.M, enc.K), np.int32)
    for m in range(enc.M):
        H[m, flags[m]] = enc.hi_val[m].reshape(-1)
    assert np.array_equal(enc.codes.astype(np.int32), np.where(flags, H, 16 * d))
    # reconstruction: half a step of the part's grid (plus fp32 slack)
    x = bf16_bits_to_f32(wl.x_bits).astype(np.float64)
    s = enc.s_hi.astype(np.float64)[:, None]
    err = np.abs(x - s * enc.codes.astype(np.float64))
    assert (err[flags] <= (0.5 * s * np.ones_like(x))[flags] * (1 + 1e-6)).all()
    assert (err[~flags] <= (8.0 * s * np.ones_like(x))[~flags] * (1 + 1e-6)).all()
    # every row reaches its full scale in one of the parts (A is the smallest admissible one)
    top_hi = np.abs(enc.hi_val.reshape(enc.M, -1).astype(np.int32)).max(1)
    top_lo = np.abs(d).max(1)
    assert ((top_hi == 127) | (top_lo == 7)).all()


def test_product_against_numpy_and_the_two_accumulator_oracle():
    wl = make("c1_tiny")
    enc = oracle.encode_tied(wl.x_bits, wl.bank, wl.topk)
    out = oracle.gemm_tied(enc, wl.wq_packed, wl.w_scale)
    W = unpack_int4(wl.wq_packed).astype(np.int64)
    assert np.array_equal(out.acc.astype(np.int64), enc.codes.astype(np.int64) @ W.T)
    # the pinned two-accumulator product on the same codes: acc = 16 * acc_lo + acc_hi, exactly
    as_two = oracle.Encoded(enc.M, enc.K, enc.bank, enc.topk, 0, enc.d_lo, enc.hi_val, enc.mask, enc.s_lo, enc.s_hi)
    two = oracle.gemm(as_two, wl.wq_packed, wl.w_scale)
    assert np.array_equal(out.acc.astype(np.int64), 16 * two.acc_lo.astype(np.int64) + two.acc_hi.astype(np.int64))
    assert np.allclose(out.y64, two.y64, rtol=1e-12, atol=0)
    want = out.acc.astype(np.float64) * enc.s_hi.astype(np.float64)[:, None] * wl.w_scale.astype(np.float64)[None, :]
    assert np.array_equal(out.y64, want)
    assert (np.abs(out.y32.astype(np.float64) - want) <= 2 * 2.0 ** -24 * np.abs(want) + 1e-300).all()
    assert np.array_equal(out.ybf16, f32_to_bf16_bits(out.y32))
    # and it is a layer: it follows the real product, though with x30 outlier channels the tied low grid
    # (16 high-part steps) is coarse: the error is several times that of the two-scale layer (about 0.05)
    X = bf16_bits_to_f32(wl.x_bits).astype(np.float64)
    ref = X @ (W * wl.w_scale.astype(np.float64)[:, None]).T
    rel = np.linalg.norm(out.y64 - ref) / np.linalg.norm(ref)
    rel_two = np.linalg.norm(oracle.gemm(oracle.encode(wl.x_bits, wl.bank, wl.topk), wl.wq_packed, wl.w_scale).y64 - ref) / np.linalg.norm(ref)
    assert rel_two < rel < 0.25


def test_bf16_output_rounding_by_hand():
    """acc = 1, weight scale 1: y32 is the token's s_hi; expected bf16 patterns worked out by hand
    (half-way cases go to the even upper half, the carry may run into the exponent)."""
    cases = [(0x3F808000, 0x3F80), (0x3F818000, 0x3F82), (0x3F808001, 0x3F81), (0x3F807FFF, 0x3F80),
             (0xBF818000, 0xBF82), (0x3FFF8000, 0x4000), (0x40490FDB, 0x4049)]
    M, K = len(cases), 32
    codes = np.zeros((M, K), np.int8)
    codes[:, 3] = 1
    s_hi = np.array([c[0] for c in cases], np.uint32).view(np.float32)
    from oracle.tied import EncodedTied
    enc = EncodedTied(M, K, 32, 1, None, None, None, (s_hi * np.float32(16)).astype(np.float32), s_hi, codes)
    w = np.zeros((1, K), np.int8)
    w[0, 3] = 1
    out = oracle.gemm_tied(enc, pack_int4(w), np.ones(1, np.float32))
    assert [int(v) for v in out.y32.view(np.uint32)[:, 0]] == [c[0] for c in cases]
    assert [hex(int(v)) for v in out.ybf16[:, 0]] == [hex(c[1]) for c in cases]


def test_all_high_reduces_to_plain_per_token_int8():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((7, 128)).astype(np.float32)
    bits = f32_to_bf16_bits(x)
    w = rng.integers(-8, 8, size=(33, 128)).astype(np.int8)
    enc = oracle.encode_tied(bits, 64, 64)
    xv = bf16_bits_to_f32(bits)
    amax = np.abs(xv).max(1).astype(np.float32)
    q = np.rint((xv * (np.float32(127.0) / amax)[:, None]).astype(np.float32)).astype(np.int64)
    assert np.array_equal(enc.codes.astype(np.int64), q) and not enc.d_lo.any()
    out = oracle.gemm_tied(enc, pack_int4(w), np.ones(33, np.float32))
    assert np.array_equal(out.acc.astype(np.int64), q @ w.astype(np.int64).T)


SOURCE = open(os.path.join(ROOT, "oracle", "tied.py")).read()
MUTANTS = [
    ("low grid is 8 steps instead of 16", "F32(sc_hi * F32(16.0)), F32(inv_hi * F32(0.0625))", "F32(sc_hi * F32(8.0)), F32(inv_hi * F32(0.125))"),
    ("combined code uses 8 * d", "np.where(is_hi, h, 16 * d)", "np.where(is_hi, h, 8 * d)"),
    ("scale ignores the low part", "A = max(amax_hi, F32(amax_lo * (F32(127.0) / F32(112.0))))", "A = amax_hi"),
    ("low part allowed 8 levels", "F32(127.0) / F32(112.0)", "F32(127.0) / F32(128.0)"),
    ("high scale divides by 128", "F32(A / F32(127.0)), F32(F32(127.0) / A)", "F32(A / F32(128.0)), F32(F32(128.0) / A)"),
    ("round half up", "h = np.clip(np.rint((x[m] * inv_hi).astype(F32)), -127, 127)", "h = np.clip(np.floor((x[m] * inv_hi).astype(F32) + F32(0.5)), -127, 127)"),
    ("round half up (low)", "d = np.clip(np.rint((x[m] * inv_lo).astype(F32)), -7, 7)", "d = np.clip(np.floor((x[m] * inv_lo).astype(F32) + F32(0.5)), -7, 7)"),
    ("low codes kept at the high channels", "        d[is_hi] = 0\n", ""),
    ("nibbles swapped", "((d[0::2] & 0xF) | ((d[1::2] & 0xF) << 4))", "((d[1::2] & 0xF) | ((d[0::2] & 0xF) << 4))"),
    ("weights read as unsigned", "w[:, 0::2] = np.where(lo >= 8, lo - 16, lo)", "w[:, 0::2] = lo"),
    ("output scaled by s_lo", "t = (acc.astype(F32) * enc.s_hi[:, None]).astype(F32)", "t = (acc.astype(F32) * enc.s_lo[:, None]).astype(F32)"),
    ("bf16 rounds half up", "up = (rest > 0x8000) | ((rest == 0x8000) & ((keep & np.uint32(1)) == 1))", "up = rest >= 0x8000"),
]


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_noticed(tmp_path, name, old, new):
    if os.environ.get("SQ_ORACLE_TIED_SRC"):
        pytest.skip("child process of the mutation test")
    assert SOURCE.count(old) == 1, "the text to mutate must occur exactly once"
    path = str(tmp_path / "tied_mutant.py")
    open(path, "w").write(SOURCE.replace(old, new))
    env = dict(os.environ, SQ_ORACLE_TIED_SRC=path)
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "tests/test_oracle_tied.py"],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode == 1, f"no pin noticed: {name}\n{r.stdout[-1500:]}"
    assert " failed" in r.stdout

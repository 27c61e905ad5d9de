"""Pins for oracle/pairs.py: the precision pairs (8/3), (8/2), (4/2) of Section 4.1 / Table 3 and the bit-packed
storage of the format at its equivalent bit width."""
import os
import subprocess
import sys

import numpy as np
import pytest

import oracle
from workloads import f32_to_bf16_bits, unpack_int4, make

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PAIRS = [(8, 4), (8, 3), (8, 2), (4, 2)]


def row_with(values, K=64, fill=0.0):
    x = np.full((1, K), fill, np.float32)
    x[0, :len(values)] = values
    return f32_to_bf16_bits(x)


def test_pair_8_4_is_the_pinned_two_scale_oracle():
    wl = make("c1_tiny")
    a = oracle.encode_pair(wl.x_bits, wl.bank, wl.topk, 8, 4)
    b = oracle.encode(wl.x_bits, wl.bank, wl.topk)
    for f in ("d_lo", "hi_val", "mask"):
        assert np.array_equal(getattr(a, f), getattr(b, f)), f
    assert np.array_equal(a.s_lo.view(np.uint32), b.s_lo.view(np.uint32))
    assert np.array_equal(a.s_hi.view(np.uint32), b.s_hi.view(np.uint32))
    rng = np.random.default_rng(3)
    mask = np.zeros(wl.K // 32, np.uint32)
    for g in range(wl.K // 64):
        for i in rng.choice(64, 8, replace=False):
            mask[(g * 64 + i) // 32] |= np.uint32(1 << ((g * 64 + i) % 32))
    a = oracle.encode_pair(wl.x_bits, 64, 8, 8, 4, static_mask=mask)
    b = oracle.encode(wl.x_bits, 64, 8, static_mask=mask)
    assert np.array_equal(a.d_lo, b.d_lo) and np.array_equal(a.hi_val, b.hi_val)
    assert np.array_equal(a.s_lo.view(np.uint32), b.s_lo.view(np.uint32))


def test_int3_and_int2_low_codes_by_hand():
    # k = 2: high values 127 and -64; low maximum 3 -> with h_low = 3 (Q = 3) the low scale is 1: d = rne(x)
    vals = [127, -64, 3, 2.5, 1.5, 0.5, -0.5, -1.5, -2.5, 1.25, -3]
    enc = oracle.encode_pair(row_with(vals), 64, 2, 8, 3)
    assert enc.s_lo[0] == 1.0 and enc.s_hi[0] == 1.0
    assert list(unpack_int4(enc.d_lo)[0, :11]) == [0, 0, 3, 2, 2, 0, 0, -2, -2, 1, -3]   # halves go to the even code
    assert list(enc.hi_val[0, 0]) == [127, -64]
    # h_low = 2 (Q = 1, the codes -1, 0, 1 of Section 3.2.1's example): low maximum 1 -> scale 1
    vals = [127, -64, 1, 0.5, 0.75, -0.5, -0.51, -1, 0.25]
    enc = oracle.encode_pair(row_with(vals), 64, 2, 8, 2)
    assert enc.s_lo[0] == 1.0
    assert list(unpack_int4(enc.d_lo)[0, :9]) == [0, 0, 1, 0, 1, 0, -1, -1, 0]
    # (4/2): the high part is INT4, Q = 7: high maximum 7 -> scale 1, codes rne(x), half-way 6.5 -> 6, 5.5 -> 6
    vals = [7, 6.5, 5.5, 1, -1, 0.5]
    enc = oracle.encode_pair(row_with(vals), 64, 4, 4, 2)
    assert enc.s_hi[0] == 1.0 and list(enc.hi_val[0, 0]) == [7, 6, 6, 1]
    assert list(unpack_int4(enc.d_lo)[0, :6]) == [0, 0, 0, 0, -1, 0]


@pytest.mark.parametrize("h_high,h_low", PAIRS)
def test_code_ranges_and_scales(h_high, h_low):
    wl = make("c1_tiny")
    enc = oracle.encode_pair(wl.x_bits, wl.bank, wl.topk, h_high, h_low)
    qh, ql = (1 << (h_high - 1)) - 1, (1 << (h_low - 1)) - 1
    d = unpack_int4(enc.d_lo).astype(np.int32)
    assert np.abs(d).max() == ql and np.abs(enc.hi_val.astype(np.int32)).max() == qh
    assert np.array_equal(enc.mask, oracle.encode(wl.x_bits, wl.bank, wl.topk).mask)   # same selection rule
    x = np.abs((wl.x_bits.astype(np.uint32) << 16).view(np.float32))
    flags = ((enc.mask[:, :, None] >> np.arange(32, dtype=np.uint32)[None, None, :]) & 1).reshape(x.shape).astype(bool)
    assert np.array_equal(enc.s_hi, (np.where(flags, x, 0).max(1) / np.float32(qh)).astype(np.float32))
    assert np.array_equal(enc.s_lo, (np.where(flags, 0, x).max(1) / np.float32(ql)).astype(np.float32))


def table3_rows():
    rows = []
    for line in open(os.path.join(ROOT, "tests", "golden", "equivalent_bits_table3.txt")):
        line = line.split("#")[0].split()
        if len(line) == 4:
            rows.append((int(line[0]), int(line[1]), float(line[2]), float(line[3])))
    return rows


def test_storage_size_is_the_paper_s_equivalent_bit_width():
    """K*y/8 bytes per row with the y printed in the paper's Table 3 (tests/golden, cited there)."""
    rows = table3_rows()
    assert {(r[0], r[1]) for r in rows} >= {(8, 4), (8, 3), (8, 2), (4, 2)}
    K, bank = 4096, 64
    for h_high, h_low, s, y in rows:
        topk = round((1 - s) * bank)
        assert oracle.storage_row_bytes(K, bank, topk, h_high, h_low) * 8 == y * K, (h_high, h_low, s)


def test_pack_by_hand_and_round_trip():
    # two banks of 32, k = 4, (8/3): the row is 8 high bytes, then 56 low codes of 3 bits (21 bytes).
    # bank 0: high codes 127, -64, 100, 90 -> bytes 0x7F, 0xC0, 0x64, 0x5A; bank 1 is zero (its first 4 channels
    # are "high" with code 0).  The low codes start 3, 2, -2, 1, -3, 0 ...: 3-bit two's complement 011, 010, 110,
    # 001, 101, 000 -> bit stream, least significant bit first: 110 010 011 100 101 000 ...
    # byte 0 = bits 1,1,0,0,1,0,0,1 -> 0x93; byte 1 = bits 1,1,0,0,1,0,1,0 -> 0x53
    vals = [127, -64, 100, 90, 3, 2, -2, 1, -3]
    enc = oracle.encode_pair(row_with(vals, K=64), 32, 4, 8, 3)
    assert enc.s_lo[0] == 1.0 and enc.s_hi[0] == 1.0
    assert list(unpack_int4(enc.d_lo)[0, :10]) == [0, 0, 0, 0, 3, 2, -2, 1, -3, 0]
    p = oracle.pack_storage(enc, 8, 3)
    assert p.shape == (1, 8 + 21)
    assert [int(v) for v in p[0, :11]] == [0x7F, 0xC0, 0x64, 0x5A, 0, 0, 0, 0, 0x93, 0x53, 0x00]
    for h_high, h_low in PAIRS:
        wl = make("c1_tiny")
        enc = oracle.encode_pair(wl.x_bits, wl.bank, wl.topk, h_high, h_low)
        packed = oracle.pack_storage(enc, h_high, h_low)
        assert packed.shape == (wl.M, oracle.storage_row_bytes(wl.K, wl.bank, wl.topk, h_high, h_low))
        back = oracle.unpack_storage(packed, enc.mask, wl.K, wl.bank, wl.topk, h_high, h_low, enc.s_lo, enc.s_hi)
        assert np.array_equal(back.d_lo, enc.d_lo) and np.array_equal(back.hi_val, enc.hi_val)


def test_sentinel_form_by_hand_and_round_trip():
    # (8/2), one bank of 32 inside K = 64 (k = 4): low codes are -1, 0, 1; the high channels carry v_mask = -2
    # (bit pattern 10).  Channels 0..3 high; low codes of channels 4.. : 1, -1, 0, 1 -> 2-bit patterns 01, 11, 00, 01.
    # first low byte = channels 0..3 = four sentinels: 10 10 10 10 -> bits (LSB first) 0,1,0,1,0,1,0,1 -> 0xAA
    # second byte = channels 4..7: 01, 11, 00, 01 -> bits 1,0, 1,1, 0,0, 1,0 -> 0x4D
    vals = [127, -64, 100, 90, 1, -1, 0.2, 1]
    enc = oracle.encode_pair(row_with(vals, K=64), 32, 4, 8, 2)
    assert list(unpack_int4(enc.d_lo)[0, :8]) == [0, 0, 0, 0, 1, -1, 0, 1]
    p = oracle.pack_storage_sentinel(enc, 8, 2)
    assert p.shape == (1, 8 + 64 * 2 // 8)
    assert [int(v) for v in p[0, 8:10]] == [0xAA, 0x4D]
    # storage of this form: x = (1-s)*h_high + h_low bits per element (Section 4.1)
    for h_high, h_low in PAIRS:
        for bank, topk in ((64, 8), (32, 16), (128, 16)):
            s = 1 - topk / bank
            assert oracle.sentinel_row_bytes(4096, bank, topk, h_high, h_low) * 8 == 4096 * ((1 - s) * h_high + h_low)
        wl = make("c1_tiny")
        enc = oracle.encode_pair(wl.x_bits, wl.bank, wl.topk, h_high, h_low)
        packed = oracle.pack_storage_sentinel(enc, h_high, h_low)
        back = oracle.unpack_storage_sentinel(packed, wl.K, wl.bank, wl.topk, h_high, h_low, enc.s_lo, enc.s_hi)
        assert np.array_equal(back.mask, enc.mask), "the mask must come back out of the sentinels"
        assert np.array_equal(back.d_lo, enc.d_lo) and np.array_equal(back.hi_val, enc.hi_val)


SOURCE = open(os.path.join(ROOT, "oracle", "pairs.py")).read()
MUTANTS = [
    ("code range 2^(h-1) instead of 2^(h-1)-1", "return (1 << (bits - 1)) - 1", "return 1 << (bits - 1)"),
    ("low scale uses the high range", "F32(amax_lo / q_lo), F32(q_lo / amax_lo)", "F32(amax_lo / q_hi), F32(q_hi / amax_lo)"),
    ("round half up (low)", "d = np.clip(np.rint((x[m] * inv_lo).astype(F32)), -q_lo, q_lo)", "d = np.clip(np.floor((x[m] * inv_lo).astype(F32) + F32(0.5)), -q_lo, q_lo)"),
    ("round half up (high)", "h = np.clip(np.rint((x[m] * inv_hi).astype(F32)), -q_hi, q_hi)", "h = np.clip(np.floor((x[m] * inv_hi).astype(F32) + F32(0.5)), -q_hi, q_hi)"),
    ("low codes kept at high channels", "        d[is_hi] = 0\n", ""),
    ("bit stream is MSB first", 'return np.packbits(bits, bitorder="little")', 'return np.packbits(bits, bitorder="big")'),
    ("storage counts the low part over all channels", "return (k_hi * h_high + (K - k_hi) * h_low) // 8", "return (k_hi * h_high + K * h_low) // 8"),
    ("sentinel is the largest positive code", "v_mask = -(1 << (h_low - 1))\n    out = np.zeros", "v_mask = (1 << (h_low - 1)) - 1\n    out = np.zeros"),
    ("sentinel form keeps the low codes at the high channels", "ls = _pack_section(np.where(flags[m], v_mask, d[m]), h_low)", "ls = _pack_section(d[m], h_low)"),
    ("low section packs the high channels too", "ls = _pack_section(d[m][~flags[m]], h_low)", "ls = _pack_section(d[m], h_low)[: out.shape[1] - len(hs)]"),
]


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_noticed(tmp_path, name, old, new):
    if os.environ.get("SQ_ORACLE_PAIRS_SRC"):
        pytest.skip("child process of the mutation test")
    assert SOURCE.count(old) == 1, "the text to mutate must occur exactly once"
    path = str(tmp_path / "pairs_mutant.py")
    open(path, "w").write(SOURCE.replace(old, new))
    env = dict(os.environ, SQ_ORACLE_PAIRS_SRC=path)
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "tests/test_oracle_pairs.py"],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode == 1, f"no pin noticed: {name}\n{r.stdout[-1500:]}"
    assert " failed" in r.stdout

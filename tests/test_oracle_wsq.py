"""Pins for oracle/wsq.py: SQ-format on weights at run time (Section 3.2.1, Algorithm 1, Figure 1's caption):
per (output channel, bank) groups with their own two scales, the top-k weights of a group by importance in high
precision, v_mask at their places in the low part, plain INT8 activations, bank-by-bank fp32 accumulation."""
import os
import subprocess
import sys
from fractions import Fraction

import numpy as np
import pytest

import oracle
from workloads import f32_to_bf16_bits, bf16_bits_to_f32

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
W = oracle.wsq_module()


def bits_of(rows):
    return f32_to_bf16_bits(np.array(rows, np.float32))


def test_one_group_by_hand():
    # one output channel, one bank of 8, k = 2, (8/4): the two largest |w| are 127 and -64 -> high, scale 1:
    # codes 127, -64.  The low maximum is 7 -> scale 1: codes rne(w); 2.5 -> 2, 3.5 -> 4, -0.5 -> 0 (half to even).
    ws = W.encode_weights(bits_of([[127, 2.5, -64, 3.5, 7, -0.5, 1.25, -6]]), 8, 2)
    assert list(ws.hi_val[0, 0]) == [127, -64]
    assert list(ws.lo[0]) == [-8, 2, -8, 4, 7, 0, 1, -6]          # v_mask = -8 at the high places
    assert ws.s_hi[0, 0] == 1.0 and ws.s_lo[0, 0] == 1.0
    # every group has its own scales: second bank with maxima 254 (high) and 14 (low) -> scales 2 and 2
    ws = W.encode_weights(bits_of([[127, 1, 1, 1, 7, 1, 1, 1, 254, 2, 2, 2, 14, 2, 2, 6]]), 8, 1)
    assert list(ws.s_hi[0]) == [1.0, 2.0] and list(ws.s_lo[0]) == [1.0, 2.0]
    assert list(ws.hi_val[0, :, 0]) == [127, 127] and ws.lo[0, 12] == 7 and ws.lo[0, 15] == 3 and ws.lo[0, 8] == -8


def test_importance_ties_and_the_hessian_diagonal():
    # equal magnitudes: the lower channels win
    ws = W.encode_weights(bits_of([[1, 1, 1, 1, 1, 1, 1, 1]]), 8, 3)
    assert list(ws.is_hi()[0]) == [True, True, True, False, False, False, False, False]
    # I = w^2 / d^2: a large weight on a channel the model is insensitive to (large d) loses to a smaller one
    w = [[8, 1, 1, 1, 4, 1, 1, 1]]
    assert list(np.flatnonzero(W.encode_weights(bits_of(w), 8, 1).is_hi()[0])) == [0]
    d = np.array([4, 1, 1, 1, 1, 1, 1, 1], np.float32)          # I_0 = 64/16 = 4 < I_4 = 16
    assert list(np.flatnonzero(W.encode_weights(bits_of(w), 8, 1, d=d).is_hi()[0])) == [4]


@pytest.mark.parametrize("bank,topk,h_high,h_low", [(64, 8, 8, 4), (128, 16, 8, 4), (64, 16, 8, 2), (64, 8, 4, 2)])
def test_invariants(bank, topk, h_high, h_low):
    rng = np.random.default_rng(bank + topk)
    w = (rng.standard_normal((6, 256)) * 0.05).astype(np.float32)
    wb = f32_to_bf16_bits(w)
    ws = W.encode_weights(wb, bank, topk, h_high, h_low)
    G = 256 // bank
    qh, ql = (1 << (h_high - 1)) - 1, (1 << (h_low - 1)) - 1
    assert (ws.is_hi().reshape(6, G, bank).sum(2) == topk).all()
    assert np.abs(ws.dense_lo()).max() <= ql and np.abs(ws.hi_val.astype(int)).max() <= qh
    assert (ws.dense_lo()[ws.is_hi()] == 0).all()
    wv = bf16_bits_to_f32(wb).astype(np.float64)
    hi = ws.is_hi()
    # in every group the smallest high magnitude is at least the largest low one (d = 1)
    mag = np.abs(wv).reshape(6, G, bank)
    h3 = hi.reshape(6, G, bank)
    assert (np.where(h3, mag, np.inf).min(2) >= np.where(h3, 0, mag).max(2)).all()
    # reconstruction within half a step of the group's scale
    s_hi = np.repeat(ws.s_hi.astype(np.float64), bank, axis=1)
    s_lo = np.repeat(ws.s_lo.astype(np.float64), bank, axis=1)
    rec = ws.dense_hi() * s_hi + ws.dense_lo() * s_lo
    step = np.where(hi, s_hi, s_lo)
    assert (np.abs(wv - rec) <= 0.5 * step * (1 + 1e-4)).all()  # exact half-way cases sit on the bound; the scale itself is rounded
    # each part of each group reaches its full scale
    assert (np.abs(ws.hi_val.astype(int)).max(2) == qh).all()


def test_activation_quantiser_by_hand():
    codes, scale = W.quantize_activations(bits_of([[127, -63.5, 0.5, 1.5, -2.5, 0, 100, -127], [0] * 8]))
    assert list(codes[0]) == [127, -64, 0, 2, -2, 0, 100, -127] and scale[0] == 1.0
    assert not codes[1].any() and scale[1] == 1.0
    codes4, scale4 = W.quantize_activations(bits_of([[14, -7, 1, 3]]), bits=4)
    assert list(codes4[0]) == [7, -4, 0, 2] and scale4[0] == 2.0     # -3.5 -> -4, 0.5 -> 0, 1.5 -> 2


def test_products_and_the_bank_by_bank_sum():
    rng = np.random.default_rng(9)
    wb = f32_to_bf16_bits((rng.standard_normal((11, 256)) * 0.03).astype(np.float32))
    xb = f32_to_bf16_bits(rng.standard_normal((5, 256)).astype(np.float32))
    ws = W.encode_weights(wb, 64, 8)
    a, sa = W.quantize_activations(xb)
    out = W.gemm(a, sa, ws)
    A = a.astype(np.int64)
    for g in range(4):
        sl = slice(64 * g, 64 * g + 64)
        assert np.array_equal(out.acc_lo[:, :, g], A[:, sl] @ ws.dense_lo()[:, sl].astype(np.int64).T)
        assert np.array_equal(out.acc_hi[:, :, g], A[:, sl] @ ws.dense_hi()[:, sl].astype(np.int64).T)
    # the fp32 evaluation, element by element in exact rational arithmetic with the stated roundings
    m, n = 3, 7
    f = np.float32(0)
    for g in range(4):
        t = np.float32(float(Fraction(int(out.acc_lo[m, n, g])) * Fraction(float(ws.s_lo[n, g]))))
        t = np.float32(float(Fraction(int(out.acc_hi[m, n, g])) * Fraction(float(ws.s_hi[n, g])) + Fraction(float(t))))
        f = np.float32(float(Fraction(float(f)) + Fraction(float(t))))
    y = np.float32(float(Fraction(float(f)) * Fraction(float(sa[m]))))
    assert out.y32[m, n] == y
    assert np.allclose(out.y32, out.y64, rtol=1e-5, atol=1e-6)
    # the layer follows the real product
    X = bf16_bits_to_f32(xb).astype(np.float64)
    Wf = bf16_bits_to_f32(wb).astype(np.float64)
    ref = X @ Wf.T
    assert np.linalg.norm(out.y64 - ref) / np.linalg.norm(ref) < 0.08   # INT4 low part of Gaussian weights: about 5 %
    assert np.array_equal(out.ybf16, f32_to_bf16_bits(out.y32))


def test_all_high_is_plain_group_wise_int8():
    rng = np.random.default_rng(4)
    wb = f32_to_bf16_bits((rng.standard_normal((3, 128)) * 0.1).astype(np.float32))
    ws = W.encode_weights(wb, 64, 64)
    wv = bf16_bits_to_f32(wb)
    amax = np.abs(wv).reshape(3, 2, 64).max(2).astype(np.float32)
    q = np.rint((wv.reshape(3, 2, 64) * (np.float32(127) / amax)[:, :, None]).astype(np.float32)).astype(np.int8)
    assert np.array_equal(ws.hi_val, q) and (ws.lo == -8).all()
    assert np.array_equal(ws.s_hi, (amax / np.float32(127)).astype(np.float32))


SOURCE = open(os.path.join(ROOT, "oracle", "wsq.py")).read()
MUTANTS = [
    ("importance ignores d", "imp = ((w * w).astype(F32) / (dd * dd).astype(F32)[None, :]).astype(F32)", "imp = (w * w).astype(F32)"),
    ("ties to the higher channel", "key=lambda i: (-float(imp[n, sl][i]), i)", "key=lambda i: (-float(imp[n, sl][i]), -i)"),
    ("one scale per row instead of per group", "a_lo = F32(np.abs(wg[~hi]).max()) if (~hi).any() else F32(0)", "a_lo = F32(np.abs(w[n]).max())"),
    ("sentinel is zero", "lo[n, sl] = np.where(hi, v_mask, cl)", "lo[n, sl] = np.where(hi, 0, cl)"),
    ("high codes in the low range", "ch = np.clip(np.rint((wg * inv_hi).astype(F32)), -q_hi, q_hi)", "ch = np.clip(np.rint((wg * inv_lo).astype(F32)), -q_lo, q_lo)"),
    ("round half up", "cl = np.clip(np.rint((wg * inv_lo).astype(F32)), -q_lo, q_lo)", "cl = np.clip(np.floor((wg * inv_lo).astype(F32) + F32(0.5)), -q_lo, q_lo)"),
    ("activation scale divides by 128", "q = F32(qmax(bits))", "q = F32(qmax(bits) + 1)"),
    ("bank scales exchanged", "t = (acc_lo[:, :, g].astype(F32) * wsq.s_lo[None, :, g]).astype(F32)", "t = (acc_lo[:, :, g].astype(F32) * wsq.s_hi[None, :, g]).astype(F32)"),
    ("high part dropped", "t = _fma32(acc_hi[:, :, g].astype(F32), np.broadcast_to(wsq.s_hi[None, :, g], t.shape), t)", "t = t"),
    ("token scale of the wrong row", "y32 = (f * a_scale.astype(F32)[:, None]).astype(F32)", "y32 = (f * a_scale.astype(F32)[0]).astype(F32)"),
]


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_noticed(tmp_path, name, old, new):
    if os.environ.get("SQ_ORACLE_WSQ_SRC"):
        pytest.skip("child process of the mutation test")
    assert SOURCE.count(old) == 1, "the text to mutate must occur exactly once"
    path = str(tmp_path / "wsq_mutant.py")
    open(path, "w").write(SOURCE.replace(old, new))
    env = dict(os.environ, SQ_ORACLE_WSQ_SRC=path)
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "tests/test_oracle_wsq.py"],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode == 1, f"no pin noticed: {name}\n{r.stdout[-1500:]}"
    assert " failed" in r.stdout

"""Do the pins pin?  Each case plants one plausible mistake in a copy of the oracle's source (a wrong tie-break,
a sign, a dropped term, a swapped nibble, a wrong denominator, ...), compiles it, and runs the pin tests of
test_oracle_select / _encode / _gemm against that library in a child process: at least one pin must fail.
A mistake that no pin notices would mean the oracle could carry it unseen."""
import os
import subprocess
import sys

import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SOURCE = open(os.path.join(ROOT, "oracle", "sq_oracle.c")).read()
PIN_FILES = ["tests/test_oracle_select.py", "tests/test_oracle_encode.py", "tests/test_oracle_gemm.py"]

# (name, text in the oracle, what the mistake turns it into)
MUTANTS = [
    ("ties go to the higher channel",
     "magnitude_key(xb[order[p - 1]]) < key", "magnitude_key(xb[order[p - 1]]) <= key"),
    ("selection by signed value instead of magnitude",
     "static int magnitude_key(uint16_t bits) { return bits & 0x7FFF; }", "static int magnitude_key(uint16_t bits) { return (int16_t)bits; }"),
    ("high scale divides by 128",
     "sc_hi = amax_hi / 127.0f; inv_hi = 127.0f / amax_hi;", "sc_hi = amax_hi / 128.0f; inv_hi = 128.0f / amax_hi;"),
    ("low scale uses 8 levels",
     "sc_lo = amax_lo / 7.0f;   inv_lo = 7.0f / amax_lo;", "sc_lo = amax_lo / 8.0f;   inv_lo = 8.0f / amax_lo;"),
    ("low scale from the whole row",
     "        else          { if (a > amax_lo) amax_lo = a; }", "        if (a > amax_lo) amax_lo = a;"),
    ("round half up instead of half even (low part)",
     "volatile float p = v * inv_lo;\n          float r = nearbyintf(p);", "volatile float p = v * inv_lo;\n          float r = floorf(p + 0.5f);"),
    ("round half up instead of half even (high part)",
     "volatile float p = v * inv_hi; /* one fp32 multiply, rounded to fp32 before rounding to integer */\n          float r = nearbyintf(p);",
     "volatile float p = v * inv_hi;\n          float r = floorf(p + 0.5f);"),
    ("nibbles swapped in the packed low part",
     "dl[i] = (uint8_t)((code_lo[2 * i] & 0xF) | ((code_lo[2 * i + 1] & 0xF) << 4));",
     "dl[i] = (uint8_t)((code_lo[2 * i + 1] & 0xF) | ((code_lo[2 * i] & 0xF) << 4));"),
    ("low code kept at the high positions",
     "          code_lo[j] = 0;\n", "          { volatile float q = v * inv_lo; float rq = nearbyintf(q); if (rq > 7.0f) rq = 7.0f; if (rq < -7.0f) rq = -7.0f; code_lo[j] = (int)rq; }\n"),
    ("mask bits in reverse order inside a word",
     "bits |= (uint32_t)is_hi[wd * 32 + t] << t;", "bits |= (uint32_t)is_hi[wd * 32 + t] << (31 - t);"),
    ("high product reads the wrong weight column",
     "a_hi += (int64_t)h[t] * (int64_t)wr[pos[t]];", "a_hi += (int64_t)h[t] * (int64_t)wr[t];"),
    ("high part dropped from the epilogue",
     "float t1 = fmaf((float)(int32_t)a_hi, s_hi[m], t0);", "float t1 = t0;"),
    ("scales of the two parts exchanged in the epilogue",
     "volatile float t0 = (float)(int32_t)a_lo * s_lo[m];\n        float t1 = fmaf((float)(int32_t)a_hi, s_hi[m], t0);",
     "volatile float t0 = (float)(int32_t)a_lo * s_hi[m];\n        float t1 = fmaf((float)(int32_t)a_hi, s_lo[m], t0);"),
    ("weight codes read as unsigned",
     "  return v >= 8 ? v - 16 : v;", "  return v;"),
    ("weight scale of the wrong output channel",
     "volatile float y = t1 * s_w[n];", "volatile float y = t1 * s_w[0];"),
    ("importance keeps the sign",
     "imp[j] = fabs(a * cs);", "imp[j] = a * cs;"),
    ("calibration averages x instead of |x|",
     "a += fabs((double)bf16_value(calib[t * K + j]));", "a += (double)bf16_value(calib[t * K + j]);"),
    ("importance ignores the weights",
     "imp[j] = fabs(a * cs);", "imp[j] = fabs(a);"),
    ("bf16 output rounds half-way cases up instead of to even",
     "u += 0x7FFFu + ((u >> 16) & 1u);", "u += 0x8000u;"),
    ("bf16 output truncates",
     "u += 0x7FFFu + ((u >> 16) & 1u);", "u += 0u;"),
]


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_noticed(tmp_path, name, old, new):
    assert SOURCE.count(old) == 1, "the text to mutate must occur exactly once in the oracle"
    lib = oracle.build_from_source(SOURCE.replace(old, new), str(tmp_path / "libsq_oracle_mutant.so"))
    env = dict(os.environ, SQ_ORACLE_LIB=lib)
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu"] + PIN_FILES,
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode == 1, f"no pin noticed: {name}\n{r.stdout[-2000:]}"
    assert " failed" in r.stdout


def test_unmodified_source_passes_in_a_child_process(tmp_path):
    lib = oracle.build_from_source(SOURCE, str(tmp_path / "libsq_oracle_same.so"))
    env = dict(os.environ, SQ_ORACLE_LIB=lib)
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu"] + PIN_FILES,
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-2000:]

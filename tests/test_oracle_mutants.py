"""The pins must reject a broken oracle.

Each case plants one plausible mistake (a wrong comparison, sign, index, weight, a dropped term, a
transposed operand) in a copy of the oracle's C source, builds it, and runs the pin tests against that
build in a child process; the pins pass only if no test notices, which fails the case.  The mistakes are
planted on the CPU, in the oracle only; nothing here touches the GPU path.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "bnn_oracle.c")

# (name, text in bnn_oracle.c, replacement).  Every `old` occurs exactly once in the source.
MUTANTS = [
    ("sign_excludes_zero", "return (x >= 0.0f) ? (int8_t)1 : (int8_t)-1;", "return (x > 0.0f) ? (int8_t)1 : (int8_t)-1;"),
    ("matmul_transposed_operand", "c[n] += a * (int32_t)b[n];", "c[n] += a * (int32_t)Bm[n * K + k];"),
    ("matmul_wrong_sign", "c[n] += a * (int32_t)b[n];", "c[n] -= a * (int32_t)b[n];"),
    ("matmul_drops_last_term", "for (int64_t k = 0; k < K; ++k) {\n            const int32_t a = A[m * K + k];",
     "for (int64_t k = 0; k < K - 1; ++k) {\n            const int32_t a = A[m * K + k];"),
    ("bn_drops_beta", "volatile float y = scaled + beta;", "volatile float y = scaled;"),
    ("bn_drops_eps", "volatile float denom = sqrtf(var + eps);", "volatile float denom = sqrtf(var);"),
    ("bn_adds_mean", "volatile float centred = s - mean;", "volatile float centred = s + mean;"),
    ("bn_variance_not_rooted", "volatile float denom = sqrtf(var + eps);", "volatile float denom = var + eps;"),
    ("pack_msb_first", "words[r * kw + k / 32] |= (uint32_t)1 << (k % 32);",
     "words[r * kw + k / 32] |= (uint32_t)1 << (31 - k % 32);"),
    ("pack_and_unpack_msb_first",
     "words[r * kw + k / 32] |= (uint32_t)1 << (k % 32);",
     "words[r * kw + k / 32] |= (uint32_t)1 << (31 - k % 32);",
     "((words[r * kw + k / 32] >> (k % 32)) & 1u)", "((words[r * kw + k / 32] >> (31 - k % 32)) & 1u)"),
    ("unpack_polarity", "? (int8_t)1\n                                                            : (int8_t)-1;",
     "? (int8_t)-1\n                                                            : (int8_t)1;"),
    ("padding_reads_minus_one", "if (y < 0 || y >= H || x < 0 || x >= W)\n        return 1;",
     "if (y < 0 || y >= H || x < 0 || x >= W)\n        return -1;"),
    ("conv_taps_swapped", "acc += in_at(in, H, W, Cin, b,\n                                             oy * stride + ky - pad,\n                                             ox * stride + kx - pad, ci) *",
     "acc += in_at(in, H, W, Cin, b,\n                                             oy * stride + kx - pad,\n                                             ox * stride + ky - pad, ci) *"),
    ("conv_drops_first_tap_row", "for (int64_t ky = 0; ky < kh; ++ky)\n                        for (int64_t kx = 0; kx < kw; ++kx)\n                            for (int64_t ci = 0; ci < Cin; ++ci)\n                                acc +=",
     "for (int64_t ky = 1; ky < kh; ++ky)\n                        for (int64_t kx = 0; kx < kw; ++kx)\n                            for (int64_t ci = 0; ci < Cin; ++ci)\n                                acc +="),
    ("im2col_channel_major", "row[(ky * kw + kx) * Cin + ci] = (int8_t)in_at(", "row[(ci * kh + ky) * kw + kx] = (int8_t)in_at("),
    ("maxpool_takes_minimum", "if (v > best)", "if (v < best)"),
    ("bitplane_weight_off_by_one", "const int32_t weight = (int32_t)1 << (p - 1);", "const int32_t weight = (int32_t)1 << p;"),
    ("bitplane_msb_first", "const int32_t xbit = (X[m * K + k] >> (p - 1)) & 1;", "const int32_t xbit = (X[m * K + k] >> (8 - p)) & 1;"),
]


def _build_mutant(case, tmp_dir):
    name, subs = case[0], case[1:]
    text = open(SRC).read()
    for old, new in zip(subs[0::2], subs[1::2]):
        assert text.count(old) == 1, f"{name}: the text to replace must occur exactly once in bnn_oracle.c"
        text = text.replace(old, new)
    c_path = os.path.join(tmp_dir, name + ".c")
    so_path = os.path.join(tmp_dir, name + ".so")
    with open(c_path, "w") as f:
        f.write(text)
    subprocess.run(["gcc", "-O1", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-std=c99", "-shared", "-fPIC",
                    c_path, "-o", so_path, "-lm"], check=True)
    return so_path


def _pins_pass(so_path):
    env = dict(os.environ, BNN_ORACLE_LIB=so_path, OMP_NUM_THREADS="2")
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], env=env, cwd=ROOT, stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                       text=True)
    return r.returncode == 0, r.stdout[-800:]


def test_every_planted_mistake_is_caught(tmp_path):
    libs = [(case[0], _build_mutant(case, str(tmp_path))) for case in MUTANTS]
    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(lambda nl: (nl[0],) + _pins_pass(nl[1]), libs))
    survivors = [name for name, passed, _ in results if passed]
    assert not survivors, f"the pins did not notice these planted mistakes: {survivors}"


def test_unmodified_oracle_passes_the_same_run(tmp_path):
    # Control: the same child-process run on an unmodified copy passes, so a failure above is the mutant's.
    so = _build_mutant(("control",), str(tmp_path))
    passed, tail = _pins_pass(so)
    assert passed, tail

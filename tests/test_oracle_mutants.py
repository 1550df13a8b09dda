"""Mutation check of the oracle's pins (CPU only).

Every plausible mistake planted in a copy of oracle/gptq_oracle.c - a wrong nibble order, an off-by-one row, reversed
zero-point nibbles, a sign, a wrong scale index, a second rounding, a g_idx stride, a transposed operand, a rounding
mode - must make tests/test_oracle_pins.py fail.  The mutants are compiled into a temporary directory and the pin
tests run against them in a child process; the oracle in the tree is never touched.  One mutant is listed as
equivalent: rounding the exact product of two fp16 values to fp32 before adding it in fp64 changes nothing, because
the product of two 11-bit significands has 22 bits and fits fp32 exactly.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "gptq_oracle.c")

# (text in the oracle, planted replacement, killed?)
MUTANTS = [
    ("(4 * idx)", "(4 * (7 - idx))", True),                                          # nibble order in a word
    ("qweight[(size_t)(k / 8) * N + n], k % 8);", "qweight[(size_t)(k / 8) * N + n], (k + 1) % 8);", True),
    ("qzeros[(size_t)r * (N / 8) + n / 8], n % 8);", "qzeros[(size_t)r * (N / 8) + n / 8], 7 - n % 8);", True),
    ("int d = q - z;", "int d = z - q;", True),                                      # sign
    ("int d = q - z;", "int d = q - z - 1;", True),                                  # zero-point offset
    ("double s = half_bits_to_double(scales[(size_t)r * N + n]);",
     "double s = half_bits_to_double(scales[(size_t)n + 0 * r]);", True),            # scale row ignored
    ("return double_to_half_bits_rne(s * (double)d);",
     "return double_to_half_bits_rne((double)(float)(s * (double)d * 1.0000001));", True),  # perturbed product
    ("return g_idx ? g_idx[k] : k / group_size;", "return g_idx ? g_idx[k / 8 * 8] : k / group_size;", True),
    ("return g_idx ? g_idx[k] : k / group_size;", "return k / group_size;", True),   # g_idx ignored
    ("o[n] += xv * wrow[n];", "o[n] += (double)(float)(xv * wrow[n]);", False),      # equivalent program (see above)
    ("double xv = half_bits_to_double(x[(size_t)m * K + k]);",
     "double xv = half_bits_to_double(x[(size_t)k * M + m]);", True),                # transposed activations
    ("double r = rint(a / quantum);", "double r = floor(a / quantum + 0.5);", True),  # rounding mode of the fp16 grid
    ("double code = rint(w / s) + (double)z[(size_t)r * N + n];",
     "double code = floor(w / s) + (double)z[(size_t)r * N + n];", True),            # quantiser rounding
    ("acc += half_bits_to_double(x[(size_t)m * K + k]) * w;",
     "acc += half_bits_to_double(x[(size_t)m * K + k]) * w; if (k == 3) acc += 1e-9;", True),  # stray term
]


def run_pins_against(src_text, workdir, tag):
    c_path = os.path.join(workdir, f"mutant_{tag}.c")
    so_path = os.path.join(workdir, f"mutant_{tag}.so")
    with open(c_path, "w") as f:
        f.write(src_text)
    subprocess.run(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off", "-o", so_path, c_path,
                    "-lm"], check=True, capture_output=True)
    env = dict(os.environ, GPTQ_ORACLE_LIB_OVERRIDE=so_path, OMP_NUM_THREADS="2")
    proc = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                           "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True)
    return proc.returncode


def test_every_planted_mistake_fails_a_pin(tmp_path):
    text = open(SRC).read()
    jobs = [("original", text)]
    for i, (old, new, _) in enumerate(MUTANTS):
        assert text.count(old) >= 1, f"mutant {i}: the text to replace is gone from the oracle: {old!r}"
        jobs.append((str(i), text.replace(old, new, 1)))
    with ThreadPoolExecutor(max_workers=4) as pool:
        codes = list(pool.map(lambda j: run_pins_against(j[1], str(tmp_path), j[0]), jobs))
    assert codes[0] == 0, "the pins must pass on the unmodified oracle built the same way"
    for i, (old, new, killed) in enumerate(MUTANTS):
        if killed:
            assert codes[i + 1] != 0, f"mutant {i} survived the pins: {old!r} -> {new!r}"
        else:
            assert codes[i + 1] == 0, f"mutant {i} was believed equivalent but a pin now tells it apart"

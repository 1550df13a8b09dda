"""The stored oracle values under tests/golden/ still come out of the oracle (CPU only)."""
import os

import numpy as np

import oracle
from paper_2511_19438_amd import workloads

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def read_rows(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            if not line.startswith("#"):
                rows.append(line.split())
    return rows


def test_config0_gemm_samples_reproduce():
    rows = read_rows("config0_gemm_samples.txt")
    m_idx = np.array([int(r[0]) for r in rows], np.int32)
    n_idx = np.array([int(r[1]) for r in rows], np.int32)
    stored = np.array([float.fromhex(r[2]) for r in rows])
    case = workloads.make_case(1, 4096, 4096, 128, seed=workloads.case_seed(0))
    ref = oracle.gemm_ref_sampled(case["x"], case["qweight"], case["qzeros"], case["scales"], None, 128, m_idx, n_idx)
    assert len(rows) == 96 and np.array_equal(ref, stored)


def test_config0_dequant_samples_reproduce():
    rows = read_rows("config0_dequant_samples.txt")
    case = workloads.make_weights(4096, 4096, 128, seed=workloads.case_seed(0))
    w = oracle.dequant(case["qweight"], case["qzeros"], case["scales"], None, 128).view(np.uint16)
    assert len(rows) == 96
    for k, n, bits in rows:
        assert int(w[int(k), int(n)]) == int(bits, 16)

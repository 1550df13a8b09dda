"""Writes the stored expected values under tests/golden/ from the CPU oracle alone.

Run from the repo root:  python tests/golden/make_golden.py
It imports only ``oracle`` and the seeded input generators; nothing from the HIP path.
The paper (Opt4GPTQ) prints no numeric example for the 4-bit GEMM, so these files hold the
oracle's values for the first benchmark configuration (M=1, K=N=4096, group 128, seed 0) at
sampled positions.  They guard the oracle against silent change and give the GPU tests a
fixed target that does not depend on the machine they run on.
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2511_19438_amd import workloads  # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))


def main():
    M, K, N, G = 1, 4096, 4096, 128
    case = workloads.make_case(M, K, N, G, seed=workloads.case_seed(0))
    m_idx, n_idx = workloads.sample_positions(M, N, 96, seed=100)
    ref = oracle.gemm_ref_sampled(case["x"], case["qweight"], case["qzeros"], case["scales"], None, G, m_idx, n_idx)
    w = oracle.dequant(case["qweight"], case["qzeros"], case["scales"], None, G)
    k_idx, c_idx = workloads.sample_positions(K, N, 96, seed=101)
    with open(os.path.join(HERE, "config0_gemm_samples.txt"), "w") as f:
        f.write("# oracle fp64 reference ref[m, n] of benchmark configuration 0 (M=1, K=4096, N=4096, group 128, seed 0)\n")
        f.write("# written by tests/golden/make_golden.py from oracle/ only; columns: m n ref(hex float64)\n")
        for m, n, v in zip(m_idx, n_idx, ref):
            f.write(f"{m} {n} {float(v).hex()}\n")
    with open(os.path.join(HERE, "config0_dequant_samples.txt"), "w") as f:
        f.write("# oracle fp16 weight bits w16[k, n] of benchmark configuration 0 (K=4096, N=4096, group 128, seed 0)\n")
        f.write("# written by tests/golden/make_golden.py from oracle/ only; columns: k n bits(hex uint16)\n")
        for k, n in zip(k_idx, c_idx):
            f.write(f"{k} {n} {int(w.view(np.uint16)[k, n]):04x}\n")


if __name__ == "__main__":
    main()

"""GPU parity on seeded random problem shapes under the automatic plan: batch sizes on both sides of every
dispatch threshold, K of few and many stages, ragged N, all supported group sizes, with and without g_idx."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
from paper_2511_19438_amd import workloads  # noqa: E402
from test_gpu_parity import B, assert_within_band, run_gemm  # noqa: E402,F401


def _cases(n=64, seed=20251127):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        group = int(rng.choice([32, 64, 128, 128, 128]))
        K = group * int(rng.integers(1, 2048 // group + 1))
        N = 8 * int(rng.integers(1, 80))
        M = int(rng.choice([1, 2, 3, 5, 8, 15, 16, 17, 31, 32, 33, 40, 47, 48, 49, 63, 64, 65, 100, 128, 129, 200, 257, 300]))
        act = bool(rng.integers(0, 4) == 0)
        out.append((i, M, K, N, group, act))
    return out


@pytest.mark.parametrize("i,M,K,N,group,act", _cases())
def test_random_shape_matches_oracle(B, i, M, K, N, group, act):
    case = workloads.make_case(M, K, N, group, seed=1000 + i, act_order=act)
    ref = oracle.gemm_ref(case["x"], case["qweight"], case["qzeros"], case["scales"], case["g_idx"], group)
    out = run_gemm(B, case, group)
    assert_within_band(out, ref, f"case {i}: M={M} K={K} N={N} g={group} act={act}")
    again = run_gemm(B, case, group)
    assert np.array_equal(out.view(np.uint16), again.view(np.uint16)), "two calls differ"

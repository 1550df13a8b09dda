"""The allocation-free entry point gptq_w4a16_gemm_static against gptq_w4a16_gemm (GPU, through the C ABI).

Both run the same kernels under the same automatic plan, so the outputs must be bit-identical (a stronger
statement than the GEMM tolerance band, which is checked against the oracle as well).  Every pair of calls is
made back to back on the shared static block, the second with a smaller input: stale partial sums or arrival
counters from the first would show in the second.
"""
import ctypes

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
from paper_2511_19438_amd import workloads  # noqa: E402

TOL = 2e-2


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2511_19438_amd import binding

    binding.load()
    return binding


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


def both(B, M, K, N, group, act, seed):
    case = workloads.make_case(M, K, N, group, seed=seed, act_order=act)
    x, qw, qz, sc, gi = (dev(case[k]) for k in ("x", "qweight", "qzeros", "scales", "g_idx"))
    got = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
    B.gptq_w4a16_gemm_static(x, qw, qz, sc, gi, got, group)
    torch.cuda.synchronize()
    want = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
    B.gptq_w4a16_gemm(x, qw, qz, sc, gi, want, group)
    torch.cuda.synchronize()
    got, want = got.cpu().numpy(), want.cpu().numpy()
    assert np.array_equal(got.view(np.uint16), want.view(np.uint16)), f"static != regular entry point at {(M, K, N, act)}"
    ref = oracle.gemm_ref(case["x"], case["qweight"], case["qzeros"], case["scales"], case["g_idx"], group)
    ratio = np.abs(got.astype(np.float64) - ref) / (TOL * np.maximum(1.0, np.abs(ref)))
    assert float(ratio.max()) <= 0.25, f"static entry point outside the band at {(M, K, N, act)}: {ratio.max()}"


# (first call, second smaller call); every first call needs split-K scratch under the automatic plan:
# vector kernel, small-batch MFMA kernel, mid-batch MFMA kernel, big-tile MFMA kernel with K slices, act-order
# lookup kernel
PAIRS = [
    ((1, 11008, 4096, 128, False), (1, 4096, 520, 128, False)),
    ((8, 4096, 1024, 128, False), (3, 2048, 264, 128, False)),
    ((64, 4096, 1024, 128, False), (40, 2048, 520, 128, False)),
    ((200, 4096, 1024, 128, False), (130, 2048, 520, 128, False)),
    ((4, 4096, 1032, 128, True), (1, 1024, 264, 128, True)),
]


@pytest.mark.parametrize("first,second", PAIRS)
def test_static_matches_regular_twice_in_a_row(B, first, second):
    for i, (M, K, N, group, act) in enumerate((first, second)):
        plan = B.gptq_w4a16_plan_query(M, K, N, group, act)
        if i == 0:
            assert plan.split_k > 1, "the first call of a pair is meant to use the scratch"
        both(B, M, K, N, group, act, seed=7 * M + i)


def test_static_rejects_a_problem_beyond_its_block(B):
    # automatic plan: small-batch kernel with 8 K slices of 16 x 131072 fp32 partial sums = 64 MiB > 48 MiB.
    # The call returns before anything is enqueued, so the pointers only have to be non-null and aligned.
    M, K, N, group = 16, 8192, 131072, 128
    plan = B.gptq_w4a16_plan_query(M, K, N, group, False)
    assert plan.split_k * M * N * 4 > 48 << 20
    buf = torch.zeros(1024, dtype=torch.int32, device="cuda")
    p = ctypes.c_void_p(buf.data_ptr())
    rc = B.load().gptq_w4a16_gemm_static(p, p, p, p, None, p, M, K, N, group, None)
    assert rc == -6
    assert "static" in B.strerror(rc)
    torch.cuda.synchronize()

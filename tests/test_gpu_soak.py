"""Bounded soak of the K-slice exchange (GPU): a few thousand launches that cycle through the K-split paths of all
four GEMM kernels over changing shapes, every result compared bit for bit with the first result of its case.

The exchange of partial sums between workgroups rests on write-through stores, an acknowledged-store wait and an
arrival counter (see csrc/exchange.h); a lost or stale partial sum would show as a changed output bit.  The run
stops at the first mismatch and takes well under half a minute.
"""
import time

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2511_19438_amd import workloads  # noqa: E402

# (M, K, N, act_order, plan fields): every plan has K slices
CASES = [
    (1, 4096, 1024, False, dict(kernel=1, tile=64, split_k=4)),
    (4, 2048, 520, False, dict(kernel=1, tile=32, split_k=7)),
    (1, 11008, 4096, False, dict()),                              # the benchmark's down projection, automatic plan
    (2, 1024, 264, True, dict(kernel=1, split_k=2)),
    (8, 4096, 1024, False, dict(kernel=3, tile=64, split_k=4)),
    (24, 2048, 520, False, dict(kernel=3, tile=64, split_k=3)),
    (16, 4096, 4096, False, dict()),                              # small-batch kernel, automatic plan (4 slices)
    (48, 4096, 1024, False, dict(kernel=3, tile=64, split_k=2)),
    (64, 4096, 1024, False, dict(kernel=2, tile=5, split_k=8)),
    (56, 4096, 1024, False, dict(kernel=4, tile=64, split_k=4)),
    (120, 2048, 544, False, dict(kernel=4, split_k=3)),
    (100, 2048, 544, False, dict(kernel=2, tile=3, split_k=2)),
    (64, 4096, 4096, False, dict()),                              # mid-batch kernel, automatic plan with K slices
]
ROUNDS = 1500
BUDGET_S = 25.0


def test_k_split_exchange_soak():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2511_19438_amd import binding as B

    B.load()
    group = 128
    prepared = []
    for i, (M, K, N, act, plan_args) in enumerate(CASES):
        plan = B.Plan(**plan_args) if plan_args else None
        resolved = B.gptq_w4a16_plan_query(M, K, N, group, act, plan)
        assert resolved.split_k > 1, f"case {i} is meant to exchange partial sums"
        case = workloads.make_case(M, K, N, group, seed=900 + i, act_order=act)
        dev = {k: (None if v is None else torch.from_numpy(np.ascontiguousarray(v)).cuda()) for k, v in case.items()}
        out = torch.zeros((M, N), dtype=torch.float16, device="cuda")
        B.gptq_w4a16_gemm(dev["x"], dev["qweight"], dev["qzeros"], dev["scales"], dev["g_idx"], out, group, plan)
        torch.cuda.synchronize()
        prepared.append((dev, plan, out, out.clone().view(torch.int16)))
    bad = torch.zeros(len(CASES), dtype=torch.int32, device="cuda")
    t0 = time.perf_counter()
    launches = 0
    for rnd in range(ROUNDS):
        for i, (dev, plan, out, first) in enumerate(prepared):
            out.fill_(float("nan"))
            B.gptq_w4a16_gemm(dev["x"], dev["qweight"], dev["qzeros"], dev["scales"], dev["g_idx"], out, group, plan)
            bad[i] += (out.view(torch.int16) != first).any().to(torch.int32)
            launches += 1
        if rnd % 20 == 19 or rnd == ROUNDS - 1:
            counts = bad.cpu().numpy()  # synchronises
            assert not counts.any(), f"round {rnd}: outputs changed between launches, per case {counts.tolist()}"
            if time.perf_counter() - t0 > BUDGET_S:
                break
    assert launches >= 20 * len(CASES)

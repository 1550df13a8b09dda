"""GPU parity at the full benchmark sizes, in the launch configuration the bench times (automatic plan).

The oracle cannot finish the large products in seconds, so outputs are compared at sampled positions that the
oracle computes one by one (fp64, ascending k); the smallest configuration is compared in full.  All five
benchmark configurations are covered: single GEMV, decode batch sweep on the Llama-7B-shaped layers, act-order,
prefill, and the Llama-70B-shaped layers.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
from paper_2511_19438_amd import workloads  # noqa: E402

TOL = 2e-2
GROUP = workloads.GROUP_SIZE
SAMPLES = 1536


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2511_19438_amd import binding

    binding.load()
    return binding


_weights_cache = {}


def device_weights(K, N, seed, act_order=False):
    """Weights of one layer on host and device (cached: several batch sizes reuse them)."""
    key = (K, N, seed, act_order)
    if key not in _weights_cache:
        _weights_cache.clear()  # one layer at a time: the largest is 235 MB packed
        w = workloads.make_weights(K, N, GROUP, seed=seed, act_order=act_order)
        d = {k: (None if v is None else torch.from_numpy(v).cuda()) for k, v in w.items()}
        _weights_cache[key] = (w, d)
    return _weights_cache[key]


def check_sampled(B, M, K, N, seed, act_order=False, tight=0.25, plan=None):
    w, d = device_weights(K, N, seed, act_order)
    x = workloads.make_activations(M, K, seed=seed)
    out = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
    B.gptq_w4a16_gemm(torch.from_numpy(x).cuda(), d["qweight"], d["qzeros"], d["scales"], d["g_idx"], out, GROUP, plan)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.all(np.isfinite(got)), "non-finite output"
    m_idx, n_idx = workloads.sample_positions(M, N, SAMPLES, seed=seed + 7)
    # always include the corners and the last row / column (ragged tails of tiles and slices)
    m_idx[:4] = [0, 0, M - 1, M - 1]
    n_idx[:4] = [0, N - 1, 0, N - 1]
    ref = oracle.gemm_ref_sampled(x, w["qweight"], w["qzeros"], w["scales"], w["g_idx"], GROUP, m_idx, n_idx)
    ratio = np.abs(got[m_idx, n_idx].astype(np.float64) - ref) / (TOL * np.maximum(1.0, np.abs(ref)))
    worst = float(ratio.max())
    assert worst <= 1.0, f"M={M} K={K} N={N}: max err/tol = {worst:.3f}"
    assert worst <= tight, f"M={M} K={K} N={N}: err/tol = {worst:.3f} is suspiciously large for fp32 accumulation"


def test_config0_single_gemv_in_full(B):
    case = workloads.make_case(1, 4096, 4096, GROUP, seed=workloads.case_seed(0))
    ref = oracle.gemm_ref(case["x"], case["qweight"], case["qzeros"], case["scales"], None, GROUP)
    dev = {k: (None if v is None else torch.from_numpy(v).cuda()) for k, v in case.items()}
    out = torch.empty((1, 4096), dtype=torch.float16, device="cuda")
    B.gptq_w4a16_gemm(dev["x"], dev["qweight"], dev["qzeros"], dev["scales"], None, out, GROUP)
    ratio = np.abs(out.cpu().numpy().astype(np.float64) - ref) / (TOL * np.maximum(1.0, np.abs(ref)))
    assert float(ratio.max()) <= 0.25
    # dequantised weights of the same configuration, every element, bit for bit
    w_out = torch.empty((4096, 4096), dtype=torch.float16, device="cuda")
    B.gptq_w4a16_dequant(dev["qweight"], dev["qzeros"], dev["scales"], None, w_out, GROUP)
    expect = oracle.dequant(case["qweight"], case["qzeros"], case["scales"], None, GROUP)
    assert np.array_equal(w_out.cpu().numpy().view(np.uint16), expect.view(np.uint16))


@pytest.mark.parametrize("shape_index", [0, 1, 2, 3])
@pytest.mark.parametrize("M", workloads.DECODE_BATCHES)
def test_config1_decode_sweep_llama7b(B, shape_index, M):
    sh = workloads.LLAMA_7B[shape_index]
    check_sampled(B, M, sh.K, sh.N, workloads.case_seed(1, shape_index))


@pytest.mark.parametrize("M", [1, 8])
def test_config2_act_order(B, M):
    sh = workloads.ACT_ORDER_SHAPE
    check_sampled(B, M, sh.K, sh.N, workloads.case_seed(2), act_order=True)


@pytest.mark.parametrize("M", [1, 8, 16, 40])
def test_config2_act_order_through_the_one_time_repack(B, M):
    """The act-order configuration at full size through gptq_w4a16_act_order_prepare + gptq_w4a16_gemm_prepared,
    against the ORACLE's act-order result (raw qweight and g_idx)."""
    sh = workloads.ACT_ORDER_SHAPE
    seed = workloads.case_seed(2)
    w, d = device_weights(sh.K, sh.N, seed, act_order=True)
    qs = torch.empty_like(d["qweight"])
    perm = torch.empty(sh.K, dtype=torch.int32, device="cuda")
    B.gptq_w4a16_act_order_prepare(d["qweight"], d["g_idx"], qs, perm, GROUP)
    order = np.argsort(w["g_idx"], kind="stable").astype(np.int32)
    assert np.array_equal(perm.cpu().numpy(), order)
    x = workloads.make_activations(M, sh.K, seed=seed + M)
    out = torch.full((M, sh.N), float("nan"), dtype=torch.float16, device="cuda")
    B.gptq_w4a16_gemm_prepared(torch.from_numpy(x).cuda(), qs, d["qzeros"], d["scales"], perm, out, GROUP)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    m_idx, n_idx = workloads.sample_positions(M, sh.N, SAMPLES, seed=seed + 11)
    m_idx[:4] = [0, 0, M - 1, M - 1]
    n_idx[:4] = [0, sh.N - 1, 0, sh.N - 1]
    ref = oracle.gemm_ref_sampled(x, w["qweight"], w["qzeros"], w["scales"], w["g_idx"], GROUP, m_idx, n_idx)
    ratio = np.abs(got[m_idx, n_idx].astype(np.float64) - ref) / (TOL * np.maximum(1.0, np.abs(ref)))
    assert float(ratio.max()) <= 0.25, f"repacked act-order M={M}: err/tol = {ratio.max():.3f}"


@pytest.mark.parametrize("shape_index", [0, 2, 3])
@pytest.mark.parametrize("M", workloads.PREFILL_BATCHES)
def test_config3_prefill_llama7b(B, shape_index, M):
    sh = workloads.LLAMA_7B[shape_index]
    check_sampled(B, M, sh.K, sh.N, workloads.case_seed(3, shape_index))


@pytest.mark.parametrize("shape_index", [0, 1, 2, 3])
@pytest.mark.parametrize("M", [1, 16, 2048])
def test_config4_llama70b(B, shape_index, M):
    sh = workloads.LLAMA_70B[shape_index]
    check_sampled(B, M, sh.K, sh.N, workloads.case_seed(4, shape_index))


@pytest.mark.parametrize("family,shape_index", [(7, 0), (7, 1), (7, 2), (7, 3), (70, 0), (70, 2), (70, 3)])
@pytest.mark.parametrize("M", [24, 64, 128])
def test_mid_batch_sweep_at_full_size(B, family, shape_index, M):
    """Mid batch (17-128 rows) on the Llama shapes, automatic plan: the mid-batch streaming kernel where the
    dispatch picks it (many workgroups, two rounds of them on the widest layer), the others elsewhere."""
    sh = (workloads.LLAMA_7B if family == 7 else workloads.LLAMA_70B)[shape_index]
    check_sampled(B, M, sh.K, sh.N, 7000 + 10 * shape_index + M)


def test_dequant_full_size_70b_down_projection_is_bit_exact_on_samples(B):
    sh = workloads.LLAMA_70B[3]
    w, d = device_weights(sh.K, sh.N, workloads.case_seed(4, 3))
    w_out = torch.empty((sh.K, sh.N), dtype=torch.float16, device="cuda")
    B.gptq_w4a16_dequant(d["qweight"], d["qzeros"], d["scales"], None, w_out, GROUP)
    torch.cuda.synchronize()
    # the oracle dequantises a row block in full; compare three blocks (first, middle, last groups)
    got = w_out.cpu().numpy().view(np.uint16)
    for k0 in (0, sh.K // 2, sh.K - GROUP):
        rows = slice(k0 // 8, (k0 + GROUP) // 8)
        g = k0 // GROUP
        expect = oracle.dequant(w["qweight"][rows], w["qzeros"][g:g + 1], w["scales"][g:g + 1], None, GROUP)
        assert np.array_equal(got[k0:k0 + GROUP], expect.view(np.uint16))


@pytest.mark.parametrize("tile,split_k", [(5, 1), (5, 4), (3, 1), (3, 2), (8, 1), (1, 1)])
def test_big_tile_kernel_with_several_workgroups_per_compute_unit(B, tile, split_k):
    """Enough workgroups of every tile shape that several share a compute unit (small tiles: up to 1024 of them):
    LDS latencies are then longer than when a workgroup runs alone, which is what the hand-placed waits of the
    pipelined kernel must cover."""
    check_sampled(B, 512, 2048, 4096, seed=4242, plan=B.Plan(kernel=2, tile=tile, split_k=split_k))

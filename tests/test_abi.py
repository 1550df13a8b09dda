"""CPU-only checks of the C-ABI boundary: the library loads, exports what the header declares,
and rejects bad arguments before it touches the GPU (no compute call is made here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "gptq_w4a16.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2511_19438_amd import binding, build

    if not os.path.exists(binding.LIB_PATH):
        build.build()
    return binding.load()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return re.findall(r"GPTQ_API\s+[\w\s\*]+?\b(gptq_w4a16_\w+)\s*\(", text)


def test_header_declares_the_expected_entry_points():
    names = declared_functions()
    assert len(names) == len(set(names)) == 16
    for required in ("gptq_w4a16_gemm", "gptq_w4a16_dequant", "gptq_w4a16_unpack", "gptq_w4a16_workspace_bytes",
                     "gptq_w4a16_set_workspace", "gptq_w4a16_strerror", "gptq_w4a16_version",
                     "gptq_w4a16_gemm_plan", "gptq_w4a16_plan_query", "gptq_w4a16_act_order_prepare",
                     "gptq_w4a16_gemm_prepared", "gptq_w4a16_shift_zeros", "gptq_w4a16_gemm_static"):
        assert required in names


def test_library_exports_every_declared_symbol(lib):
    from paper_2511_19438_amd import binding

    for name in declared_functions():
        assert hasattr(lib, name), name
    assert sorted(binding.EXPORTS) == sorted(declared_functions())
    assert lib.gptq_w4a16_version() >= 100


def test_status_strings(lib):
    from paper_2511_19438_amd import binding

    texts = {binding.strerror(c) for c in (0, -1, -2, -3, -4, -5, -6)}
    assert len(texts) == 7
    assert "unknown" in binding.strerror(-99)


def test_argument_validation_happens_before_any_gpu_work(lib):
    p = ctypes.c_void_p(0x1000)       # never dereferenced: every call below must fail validation first
    odd = ctypes.c_void_p(0x1008)
    gemm = lib.gptq_w4a16_gemm
    assert gemm(None, p, p, p, None, p, 1, 128, 8, 128, None) == -1
    assert gemm(p, p, p, p, None, None, 1, 128, 8, 128, None) == -1
    assert gemm(p, p, p, p, None, p, 0, 128, 8, 128, None) == -1
    assert gemm(p, p, p, p, None, p, 1, -8, 8, 128, None) == -1
    assert gemm(p, p, p, p, None, p, 1, 128, 8, 0, None) == -1
    assert gemm(p, p, p, p, None, p, 1, 132, 8, 132, None) == -2   # K not a multiple of 8
    assert gemm(p, p, p, p, None, p, 1, 128, 12, 128, None) == -2  # N not a multiple of 8
    assert gemm(p, p, p, p, None, p, 1, 192, 8, 128, None) == -2   # group does not divide K
    assert gemm(p, p, p, p, None, p, 1, 128, 8, 4, None) == -2     # group not a multiple of 8
    assert gemm(odd, p, p, p, None, p, 1, 128, 8, 128, None) == -3
    assert gemm(p, p, p, p, odd, p, 1, 128, 8, 128, None) == -3
    assert lib.gptq_w4a16_dequant(None, p, p, None, p, 128, 8, 128, None) == -1
    assert lib.gptq_w4a16_dequant(p, p, p, None, odd, 128, 8, 128, None) == -3
    assert lib.gptq_w4a16_unpack(p, None, p, None, 128, 8, 128, None) == -1
    assert lib.gptq_w4a16_unpack(p, p, None, p, 128, 8, 128, None) == -1
    assert lib.gptq_w4a16_unpack(p, p, p, None, 128, 9, 128, None) == -2


def test_plan_validation(lib):
    from paper_2511_19438_amd import binding

    p = ctypes.c_void_p(0x1000)
    bad = binding.Plan(kernel=5)
    assert lib.gptq_w4a16_gemm_plan(p, p, p, p, None, p, 1, 128, 8, 128, None, ctypes.byref(bad)) == -1
    # the ablation switches belong to the vector kernel, have three bits and exist for small plain problems
    for bad in (binding.Plan(flags=1), binding.Plan(kernel=2, flags=1), binding.Plan(kernel=1, flags=16),
                binding.Plan(kernel=1, flags=-1)):
        assert lib.gptq_w4a16_gemm_plan(p, p, p, p, None, p, 1, 128, 8, 128, None, ctypes.byref(bad)) == -1
    ok = binding.Plan(kernel=1, flags=5)
    assert lib.gptq_w4a16_gemm_plan(p, p, p, p, None, p, 5, 128, 8, 128, None, ctypes.byref(ok)) == -2   # M > 4
    assert lib.gptq_w4a16_gemm_plan(p, p, p, p, p, p, 1, 128, 8, 128, None, ctypes.byref(ok)) == -2      # g_idx
    res = binding.gptq_w4a16_plan_query(1, 4096, 12288, 128, plan=ok)
    assert (res.kernel, res.tile, res.flags) == (1, 64, 5)
    bad = binding.Plan()
    bad.reserved[2] = 7
    assert lib.gptq_w4a16_gemm_plan(p, p, p, p, None, p, 1, 128, 8, 128, None, ctypes.byref(bad)) == -1
    # the big-tile kernel has four tile shapes; other ids are refused
    for tile in (2, 4, 6, 7, 9, 10, 11):
        bad = binding.Plan(kernel=2, tile=tile)
        assert lib.gptq_w4a16_gemm_plan(p, p, p, p, None, p, 64, 128, 32, 128, None, ctypes.byref(bad)) == -1
    for tile in (1, 3, 5, 8):
        assert binding.gptq_w4a16_plan_query(512, 4096, 4096, 128, plan=binding.Plan(kernel=2, tile=tile)).tile == tile


def test_workspace_bytes_is_host_only_and_monotone_in_batch(lib):
    f = lib.gptq_w4a16_workspace_bytes
    assert f(1, 4096, 4096, 128) > 0
    assert f(16, 4096, 4096, 128) >= f(1, 4096, 4096, 128)
    assert f(1, 4100, 4096, 128) == 0
    assert f(0, 4096, 4096, 128) == 0
    # partial sums of the K slices in fp32 stay a small fraction of the packed weights
    assert f(1, 4096, 4096, 128) < 4096 * 4096 // 2 // 4


# ---- host logic of the launch plans (no device is touched) ----

def test_default_dispatch_by_batch_size(lib):
    from paper_2511_19438_amd import binding

    q = binding.gptq_w4a16_plan_query
    assert [q(M, 4096, 4096, 128).kernel for M in (1, 2, 3, 16, 32, 33, 64, 65, 128, 129, 2048)] == \
        [1, 3, 3, 3, 3, 4, 4, 2, 2, 2, 2]
    # the mid-batch streaming kernel: 33-64 rows everywhere, 17-32 rows on wide or very deep layers, 65-128 rows
    # where its 64-column tiles give half to all of the compute units a workgroup or K is deep
    assert [q(M, 4096, 22016, 128).kernel for M in (16, 17, 32, 33, 64, 65, 128)] == [3, 4, 4, 4, 4, 2, 2]
    assert [q(M, 4096, 12288, 128).kernel for M in (16, 17, 64, 65, 128, 129)] == [3, 4, 4, 4, 4, 2]
    assert [q(M, 28672, 8192, 128).kernel for M in (16, 24, 100)] == [3, 4, 4]
    assert [q(M, 11008, 4096, 128).kernel for M in (24, 48, 100)] == [3, 4, 4]
    # act-order and group sizes the small-batch MFMA kernel does not take fall back
    assert q(8, 4096, 4096, 128, act_order=True).kernel == 1
    assert q(24, 4096, 4096, 128, act_order=True).kernel == 2
    assert q(8, 4096, 4096, 64).kernel == 3 and q(8, 4096, 4096, 32).kernel == 3  # small groups: own variants
    assert q(8, 4096, 4096, 16).kernel == 1 and q(8, 4096, 4096, 256).kernel == 3
    assert q(40, 4096, 4096, 64).kernel == 4 and q(40, 4096, 4096, 32).kernel == 2  # groups of 64 k: one stage each
    assert q(40, 4096, 4096, 128, act_order=True).kernel == 2
    assert q(40, 4096 + 32, 4096, 4096 + 32).kernel == 2   # K must be a multiple of 64
    # an explicit request is honoured where the kernel supports the problem
    assert q(1, 4096, 4096, 128, plan=binding.Plan(kernel=2)).kernel == 2
    assert q(64, 4096, 4096, 128, plan=binding.Plan(kernel=3)).kernel == 3
    assert q(8, 4096, 4096, 128, plan=binding.Plan(kernel=4)).kernel == 4
    assert q(200, 4096, 4096, 128, plan=binding.Plan(kernel=4)).kernel == 2
    assert q(8, 4096, 4096, 128, act_order=True, plan=binding.Plan(kernel=4)).kernel == 1
    assert q(8, 4096, 4096, 128, act_order=True, plan=binding.Plan(kernel=3)).kernel == 1


def test_vector_plan_is_well_formed_for_every_shape(lib):
    """Tile widths come from the supported set, slices are whole pipeline steps and never exceed the LDS budget."""
    from paper_2511_19438_amd import binding, workloads

    shapes = [(s.K, s.N) for s in workloads.LLAMA_7B + workloads.LLAMA_70B] + [(128, 8), (256, 24), (4096, 11008), (65536, 512)]
    for (K, N) in shapes:
        for M in (1, 2, 4, 8, 16):
            for act in (False, True):
                pl = binding.gptq_w4a16_plan_query(M, K, N, 128, act_order=act, plan=binding.Plan(kernel=1))
                if act and M >= 8 and K // 128 >= 512:
                    # the act-order table of all groups plus the staged rows exceed the LDS: big-tile kernel instead
                    assert pl.kernel == 2
                    continue
                assert pl.kernel == 1
                assert pl.tile in (32, 64, 128, 256) and (not act or pl.tile == 64)
                chunks = K // 32
                assert 1 <= pl.split_k <= chunks
                per_slice = -(-chunks // pl.split_k) * 32  # activations per row and slice (upper bound)
                assert per_slice * 2 * M <= 2 * 32 * 1024 + 4096 or pl.split_k == chunks
    # explicit requests are kept
    pl = binding.gptq_w4a16_plan_query(1, 4096, 4096, 128, plan=binding.Plan(kernel=1, tile=16, split_k=2))
    assert (pl.tile, pl.split_k) == (16, 2)
    pl = binding.gptq_w4a16_plan_query(1, 4096, 4096, 128, plan=binding.Plan(kernel=1, tile=256))
    assert pl.tile == 256


def test_vector_plan_prefers_one_slice_per_compute_unit_on_wide_layers(lib):
    """Wide layers at M = 1 get at most one workgroup per compute unit and no K split (no combine step)."""
    from paper_2511_19438_amd import binding

    for (K, N) in ((4096, 12288), (4096, 22016), (8192, 57344)):
        pl = binding.gptq_w4a16_plan_query(1, K, N, 128)
        assert pl.split_k == 1 and -(-N // pl.tile) <= 256, (K, N, pl.tile, pl.split_k)
    # a narrow, deep layer needs the K split to fill the chip
    pl = binding.gptq_w4a16_plan_query(1, 11008, 4096, 128)
    assert pl.split_k > 1 and 128 <= -(-4096 // pl.tile) * pl.split_k <= 512


def test_plan_query_validates_like_the_gemm(lib):
    from paper_2511_19438_amd import binding

    with pytest.raises(binding.GptqError):
        binding.gptq_w4a16_plan_query(0, 4096, 4096, 128)
    with pytest.raises(binding.GptqError):
        binding.gptq_w4a16_plan_query(1, 4100, 4096, 128)
    with pytest.raises(binding.GptqError):
        binding.gptq_w4a16_plan_query(1, 4096, 4096, 128, plan=binding.Plan(kernel=7))


def test_repack_entry_points_validate_before_any_gpu_work(lib):
    """NULL pointers, bad shapes and misaligned pointers are refused on the host."""
    buf = (ctypes.c_char * 4096)()
    base = ctypes.addressof(buf)
    base += (-base) % 256
    p = ctypes.c_void_p(base)
    odd = ctypes.c_void_p(base + 4)
    assert lib.gptq_w4a16_act_order_prepare(None, p, p, p, 128, 8, 128, None) == -1
    assert lib.gptq_w4a16_act_order_prepare(p, p, p, p, 128, 8, 128, None) == -1   # in place
    assert lib.gptq_w4a16_act_order_prepare(p, p, odd, p, 128, 8, 128, None) == -3
    assert lib.gptq_w4a16_act_order_prepare(p, p, ctypes.c_void_p(base + 1024), p, 100, 8, 128, None) == -2
    assert lib.gptq_w4a16_gemm_prepared(p, p, p, p, None, p, 1, 128, 8, 128, None) == -1
    assert lib.gptq_w4a16_gemm_prepared(p, p, p, p, p, p, 0, 128, 8, 128, None) == -1
    assert lib.gptq_w4a16_gemm_prepared(p, p, p, p, p, p, 1, 128, 12, 128, None) == -2
    assert lib.gptq_w4a16_gemm_prepared(p, p, odd, p, p, p, 1, 128, 8, 128, None) == -3
    assert lib.gptq_w4a16_shift_zeros(None, p, 1, 128, 8, 128, None) == -1
    assert lib.gptq_w4a16_shift_zeros(p, odd, 1, 128, 8, 128, None) == -3
    assert lib.gptq_w4a16_shift_zeros(p, p, 1, 128, 8, 100, None) == -2


def test_shape_limits_of_the_32_bit_offsets(lib):
    """Matrices whose packed weights would pass 4 GiB (or rows / columns 2^23 / 2^24) are refused, not mis-addressed."""
    from paper_2511_19438_amd import binding

    for (K, N) in ((1 << 23, 1024), (1024, 1 << 24), (1 << 20, 1 << 13)):
        with pytest.raises(binding.GptqError) as e:
            binding.gptq_w4a16_plan_query(1, K, N, 128)
        assert e.value.code == -2
        assert lib.gptq_w4a16_workspace_bytes(1, K, N, 128) == 0
    assert binding.gptq_w4a16_plan_query(1, 1 << 19, 1 << 13, 128).kernel == 1


def test_big_tile_plan_is_well_formed_for_every_shape(lib):
    """The big-tile kernel's automatic plan names an existing tile, splits K on every tile but 256x256, never
    into more slices than 64-k stages, and its scratch is covered by the workspace bound wherever the default
    dispatch would run it."""
    from paper_2511_19438_amd import binding, workloads

    tile_dims = {1: (256, 256), 3: (128, 128), 5: (64, 128), 8: (128, 256)}
    shapes = [(s.K, s.N) for s in workloads.LLAMA_7B + workloads.LLAMA_70B] + [(128, 32), (512, 264), (4096, 11008)]
    for (K, N) in shapes:
        for M in (33, 48, 64, 100, 128, 256, 512, 2048, 5000):
            pl = binding.gptq_w4a16_plan_query(M, K, N, 128, plan=binding.Plan(kernel=2))
            assert pl.kernel == 2 and pl.tile in tile_dims, (M, K, N, pl.tile)
            assert 1 <= pl.split_k <= max(1, K // 64)
            assert pl.split_k == 1 or pl.tile in (3, 5, 8), (M, K, N, pl.tile, pl.split_k)
            if pl.tile == 8 and pl.split_k > 1:  # 128x256 tile: K slices only with one workgroup per compute unit
                assert -(-M // 128) * -(-N // 256) * pl.split_k <= 256, (M, K, N, pl.split_k)
            if pl.split_k > 1 and binding.gptq_w4a16_plan_query(M, K, N, 128).kernel == 2:
                bm, bn = tile_dims[pl.tile]
                partial = pl.split_k * (-(-M // bm)) * (-(-N // bn)) * bm * bn * 4
                assert lib.gptq_w4a16_workspace_bytes(M, K, N, 128) >= partial
    # few output tiles and a deep K: slices; many tiles: none
    assert binding.gptq_w4a16_plan_query(64, 11008, 4096, 128).split_k > 1
    assert binding.gptq_w4a16_plan_query(2048, 4096, 22016, 128).split_k == 1


def test_mid_batch_plan_is_well_formed_for_every_shape(lib):
    """The mid-batch kernel's automatic plan: 64- or 128-column tiles (64 with more than 64 rows), one workgroup per
    compute unit at most once K is split, every wavefront keeps at least 128 k, slices cover K, and the scratch of
    the slices is covered by the workspace bound wherever the default dispatch runs the kernel."""
    from paper_2511_19438_amd import binding, workloads

    shapes = [(s.K, s.N) for s in workloads.LLAMA_7B + workloads.LLAMA_70B] + [(64, 8), (512, 264), (4096, 11008)]
    for (K, N) in shapes:
        for M in (1, 17, 32, 33, 64, 65, 128):
            pl = binding.gptq_w4a16_plan_query(M, K, N, 64, plan=binding.Plan(kernel=4))
            assert pl.kernel == 4 and pl.tile in (64, 128), (M, K, N, pl.tile)
            assert pl.tile == 64 or M <= 64
            tiles = -(-N // pl.tile)
            assert 1 <= pl.split_k <= max(1, K // 64)
            if pl.split_k > 1:
                assert tiles * pl.split_k <= 256, (M, K, N, pl.split_k)
                assert K // pl.split_k >= 8 * 128 or pl.split_k == 1, (M, K, N, pl.split_k)
            auto = binding.gptq_w4a16_plan_query(M, K, N, 64)
            if auto.kernel == 4 and auto.split_k > 1:
                assert lib.gptq_w4a16_workspace_bytes(M, K, N, 64) >= auto.split_k * M * N * 4
            # an explicit slice count is honoured (up to one slice per 64-k stage)
            asked = binding.gptq_w4a16_plan_query(M, K, N, 64, plan=binding.Plan(kernel=4, split_k=3))
            assert asked.split_k == min(3, K // 64) or (K // 64) % 3 != 0 and asked.split_k <= 3
    # wide layers: no split; narrow and deep ones: slices
    assert binding.gptq_w4a16_plan_query(64, 4096, 22016, 128).split_k == 1
    assert binding.gptq_w4a16_plan_query(64, 11008, 4096, 128).split_k > 1

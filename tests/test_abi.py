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
    assert len(names) == len(set(names)) == 8
    for required in ("gptq_w4a16_gemm", "gptq_w4a16_dequant", "gptq_w4a16_unpack", "gptq_w4a16_workspace_bytes",
                     "gptq_w4a16_set_workspace", "gptq_w4a16_strerror", "gptq_w4a16_version"):
        assert required in names


def test_library_exports_every_declared_symbol(lib):
    from paper_2511_19438_amd import binding

    for name in declared_functions():
        assert hasattr(lib, name), name
    assert sorted(binding.EXPORTS) == sorted(declared_functions())
    assert lib.gptq_w4a16_version() >= 100


def test_status_strings(lib):
    from paper_2511_19438_amd import binding

    texts = {binding.strerror(c) for c in (0, -1, -2, -3, -4, -5)}
    assert len(texts) == 6
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
    bad = binding.Plan(kernel=4)
    assert lib.gptq_w4a16_gemm_plan(p, p, p, p, None, p, 1, 128, 8, 128, None, ctypes.byref(bad)) == -1
    bad = binding.Plan(flags=1)
    assert lib.gptq_w4a16_gemm_plan(p, p, p, p, None, p, 1, 128, 8, 128, None, ctypes.byref(bad)) == -1
    bad = binding.Plan()
    bad.reserved[2] = 7
    assert lib.gptq_w4a16_gemm_plan(p, p, p, p, None, p, 1, 128, 8, 128, None, ctypes.byref(bad)) == -1


def test_workspace_bytes_is_host_only_and_monotone_in_batch(lib):
    f = lib.gptq_w4a16_workspace_bytes
    assert f(1, 4096, 4096, 128) > 0
    assert f(16, 4096, 4096, 128) >= f(1, 4096, 4096, 128)
    assert f(1, 4100, 4096, 128) == 0
    assert f(0, 4096, 4096, 128) == 0
    # partial sums of the K slices in fp32 stay a small fraction of the packed weights
    assert f(1, 4096, 4096, 128) < 4096 * 4096 // 2 // 4

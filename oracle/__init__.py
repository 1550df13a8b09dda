"""CPU oracle for the W4A16 GPTQ matrix multiply: test infrastructure only.

Only the tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py``
may import this package.  The product (``paper_2511_19438_amd``) never does.
"""
from .oracle import (  # noqa: F401
    build,
    dequant,
    double_to_half_bits,
    gemm_ref,
    gemm_ref_sampled,
    half_bits_to_double,
    num_threads,
    pack_qweight,
    pack_qzeros,
    quantize,
    unpack_qweight,
    unpack_qzeros,
)

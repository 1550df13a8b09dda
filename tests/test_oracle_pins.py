"""Pins for the CPU oracle: each check ties one step of it to something other than itself.

The paper (Opt4GPTQ) prints no worked example, tensor value or closed form for the 4-bit
GEMM; what it fixes is that the optimised kernels equal the plain GPTQ computation up to
the order of floating point additions (Section 4.4) and that multiply/add are the IEEE
operations of Eq. 14-15.  The pins are therefore: words packed by hand and written as hex
literals with hand-derived expected values, closed forms, invariants, special cases that
reduce to a library routine (numpy's IEEE fp16 multiply, numpy's fp64 matmul), and a
brute force in exact rational arithmetic on tiny inputs.
"""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2511_19438_amd import workloads

F16 = np.float16


def u32(words):
    """Hex literals -> the int32 storage type of the format."""
    return np.array(words, dtype=np.uint32).view(np.int32)


# --------------------------------------------------------------------------------------
# O1 / O2: bit layout, from words packed by hand
# --------------------------------------------------------------------------------------

def test_unpack_qweight_hand_packed_words():
    # 0x76543210: nibble j (counted from the low end) holds the value j  =>  q[k, n] = k.
    qweight = u32([[0x76543210] * 8])
    q = oracle.unpack_qweight(qweight)
    assert q.shape == (8, 8)
    assert np.array_equal(q, np.arange(8, dtype=np.uint8)[:, None].repeat(8, axis=1))
    # top nibble 0xF must not sign-extend; low nibble is k = 0
    q = oracle.unpack_qweight(u32([[0xF0000001, 0x8000000F]]))
    assert q[:, 0].tolist() == [1, 0, 0, 0, 0, 0, 0, 15]
    assert q[:, 1].tolist() == [15, 0, 0, 0, 0, 0, 0, 8]


def test_unpack_qweight_row_and_column_index():
    # word [r][n] = 0x11111111 * ((3r + n) % 16): every k in word-row r has the same code.
    R, N = 5, 16
    words = [[0x11111111 * ((3 * r + n) % 16) for n in range(N)] for r in range(R)]
    q = oracle.unpack_qweight(u32(words))
    assert q.shape == (8 * R, N)
    for k in range(8 * R):
        for n in range(N):
            assert q[k, n] == (3 * (k // 8) + n) % 16


def test_unpack_qzeros_hand_packed_words():
    # 0xFEDCBA98: nibble j holds 8 + j  =>  z[0, n] = 8 + n ; second word 0x01234567 => z[0, 8+j] = 7 - j
    qzeros = u32([[0xFEDCBA98, 0x01234567], [0x00000000, 0xA0000005]])
    z = oracle.unpack_qzeros(qzeros)
    assert z.shape == (2, 16)
    assert z[0].tolist() == [8, 9, 10, 11, 12, 13, 14, 15, 7, 6, 5, 4, 3, 2, 1, 0]
    assert z[1].tolist() == [0] * 8 + [5, 0, 0, 0, 0, 0, 0, 10]


def test_pack_unpack_are_inverse_bijections():
    rng = np.random.default_rng(7)
    q = rng.integers(0, 16, size=(64, 24), dtype=np.uint8)
    assert np.array_equal(oracle.unpack_qweight(oracle.pack_qweight(q)), q)
    words = rng.integers(0, 2 ** 32, size=(9, 40), dtype=np.uint32).view(np.int32)
    assert np.array_equal(oracle.pack_qweight(oracle.unpack_qweight(words)), words)
    z = rng.integers(0, 16, size=(3, 32), dtype=np.uint8)
    assert np.array_equal(oracle.unpack_qzeros(oracle.pack_qzeros(z)), z)
    zw = rng.integers(0, 2 ** 32, size=(5, 7), dtype=np.uint32).view(np.int32)
    assert np.array_equal(oracle.pack_qzeros(oracle.unpack_qzeros(zw)), zw)
    # packing the hand-written table reproduces the hand-written literal
    assert oracle.pack_qweight(np.arange(8, dtype=np.uint8)[:, None].repeat(8, 1))[0, 0] == 0x76543210
    assert oracle.pack_qzeros(np.array([[8, 9, 10, 11, 12, 13, 14, 15]], np.uint8)).view(np.uint32)[0, 0] == 0xFEDCBA98


# --------------------------------------------------------------------------------------
# O4 / O5: dequantisation
# --------------------------------------------------------------------------------------

def test_dequant_hand_case_closed_form():
    # q[k, n] = k, z[0, n] = 8 + n, scale 0.5  =>  w[k, n] = (k - 8 - n) / 2, all exact in fp16.
    qweight = u32([[0x76543210] * 8])
    qzeros = u32([[0xFEDCBA98]])
    scales = np.full((1, 8), 0.5, F16)
    w = oracle.dequant(qweight, qzeros, scales, None, 8)
    expected_row0 = [-4.0, -4.5, -5.0, -5.5, -6.0, -6.5, -7.0, -7.5]
    expected_row7 = [-0.5, -1.0, -1.5, -2.0, -2.5, -3.0, -3.5, -4.0]
    assert w[0].astype(float).tolist() == expected_row0
    assert w[7].astype(float).tolist() == expected_row7
    k, n = np.meshgrid(np.arange(8), np.arange(8), indexing="ij")
    assert np.array_equal(w.astype(np.float64), (k - 8 - n) / 2.0)


def test_dequant_group_row_and_scale_indexing():
    # group_size 8: word-row r is group r.  z[r, n] = (r + n//8) % 16 (constant words), q = 15 everywhere,
    # scales[r, n] = 2^-(r % 4) * (1 + n % 4): distinct per (group, column), all products exact.
    G, N = 6, 32
    qweight = u32([[0xFFFFFFFF] * N for _ in range(G)])
    qzeros = u32([[0x11111111 * ((r + nw) % 16) for nw in range(N // 8)] for r in range(G)])
    scales = np.array([[2.0 ** -(r % 4) * (1 + n % 4) for n in range(N)] for r in range(G)], F16)
    w = oracle.dequant(qweight, qzeros, scales, None, 8).astype(np.float64)
    for k in range(8 * G):
        r = k // 8
        for n in range(N):
            assert w[k, n] == 2.0 ** -(r % 4) * (1 + n % 4) * (15 - (r + n // 8) % 16)


def test_dequant_exhaustive_against_library_fp16_multiply():
    # every (q, z) pair x every fp16 scale between 0.001 and 0.01, against numpy's IEEE
    # binary16 multiply of the scale by the (exactly representable) integer difference.
    lo, hi = F16(0.001).view(np.uint16), F16(0.01).view(np.uint16)
    scale_bits = np.arange(int(lo), int(hi) + 1, dtype=np.uint16)
    pad = (-len(scale_bits)) % 8
    scale_bits = np.concatenate([scale_bits, np.full(pad, scale_bits[-1], np.uint16)])
    s_row = scale_bits.view(F16)
    N = len(s_row)
    assert N > 3000
    # group g has zero point g; inside a group of 16 rows the code runs through 0..15
    G, group = 16, 16
    q = np.tile(np.arange(16, dtype=np.uint8)[:, None], (G, N))
    z = np.arange(16, dtype=np.uint8)[:, None].repeat(N, axis=1)
    scales = np.tile(s_row[None, :], (G, 1))
    w = oracle.dequant(oracle.pack_qweight(q), oracle.pack_qzeros(z), scales, None, group)
    d = (q.astype(np.int32) - np.repeat(z, group, axis=0).astype(np.int32)).astype(F16)
    expected = np.repeat(scales, group, axis=0) * d  # float16 * float16 -> IEEE binary16 product
    assert expected.dtype == F16
    assert w.size == 256 * N
    assert np.array_equal(w.view(np.uint16), expected.view(np.uint16))


def test_dequant_zero_difference_subnormals_and_overflow():
    q = np.array([[3] * 8] * 8, np.uint8)
    z = np.array([[3, 3, 3, 3, 0, 0, 0, 0]], np.uint8)
    scales = np.array([[0.007, -0.007, 2.0 ** -20, 2.0 ** -24, 2.0 ** -20, 2.0 ** -24, 30000.0, -30000.0]], F16)
    w = oracle.dequant(oracle.pack_qweight(q), oracle.pack_qzeros(z), scales, None, 8)
    bits = w.view(np.uint16)[0]
    # q == z: +0 for a positive scale, -0 for a negative one (IEEE sign rule of a product)
    assert bits[0] == 0x0000 and bits[1] == 0x8000
    assert bits[2] == 0x0000 and bits[3] == 0x0000
    # subnormal results are kept, not flushed: 3 * 2^-20 = 48 * 2^-24 ; 3 * 2^-24
    assert bits[4] == 48 and bits[5] == 3
    # 3 * 30000 overflows binary16
    assert bits[6] == 0x7C00 and bits[7] == 0xFC00


def test_quantize_round_trip_on_workload_ranges():
    case = workloads.make_weights(256, 64, 128, seed=11)
    q = oracle.unpack_qweight(case["qweight"])
    z = oracle.unpack_qzeros(case["qzeros"])
    w = oracle.dequant(case["qweight"], case["qzeros"], case["scales"], None, 128)
    assert np.array_equal(oracle.quantize(w, case["scales"], z, None, 128), q)
    # and through an act-order group map
    case = workloads.make_weights(256, 64, 32, seed=12, act_order=True)
    q = oracle.unpack_qweight(case["qweight"])
    z = oracle.unpack_qzeros(case["qzeros"])
    w = oracle.dequant(case["qweight"], case["qzeros"], case["scales"], case["g_idx"], 32)
    assert np.array_equal(oracle.quantize(w, case["scales"], z, case["g_idx"], 32), q)


def test_quantize_round_trip_all_codes_all_scales():
    lo, hi = F16(0.001).view(np.uint16), F16(0.01).view(np.uint16)
    s_row = np.arange(int(lo), int(hi) + 1 - (int(hi) + 1 - int(lo)) % 8, dtype=np.uint16).view(F16)
    N = len(s_row)
    q = np.tile(np.arange(16, dtype=np.uint8)[:, None], (16, N))
    z = np.arange(16, dtype=np.uint8)[:, None].repeat(N, axis=1)
    scales = np.tile(s_row[None, :], (16, 1))
    w = oracle.dequant(oracle.pack_qweight(q), oracle.pack_qzeros(z), scales, None, 16)
    assert np.array_equal(oracle.quantize(w, scales, z, None, 16), q)


# --------------------------------------------------------------------------------------
# O3: group lookup
# --------------------------------------------------------------------------------------

def test_explicit_trivial_g_idx_equals_none():
    case = workloads.make_case(3, 256, 64, 32, seed=5)
    g_idx = (np.arange(256) // 32).astype(np.int32)
    a = oracle.dequant(case["qweight"], case["qzeros"], case["scales"], None, 32)
    b = oracle.dequant(case["qweight"], case["qzeros"], case["scales"], g_idx, 32)
    assert np.array_equal(a.view(np.uint16), b.view(np.uint16))
    ra = oracle.gemm_ref(case["x"], case["qweight"], case["qzeros"], case["scales"], None, 32)
    rb = oracle.gemm_ref(case["x"], case["qweight"], case["qzeros"], case["scales"], g_idx, 32)
    assert np.array_equal(ra, rb)


def test_reversed_groups_equal_flipped_tables():
    # g_idx[k] = G-1 - k//g reads the tables bottom-up: same as flipping the tables and using no g_idx
    case = workloads.make_weights(128, 32, 16, seed=6)
    G = 8
    g_idx = (G - 1 - np.arange(128) // 16).astype(np.int32)
    a = oracle.dequant(case["qweight"], case["qzeros"], case["scales"], g_idx, 16)
    b = oracle.dequant(case["qweight"], case["qzeros"][::-1].copy(), case["scales"][::-1].copy(), None, 16)
    assert np.array_equal(a.view(np.uint16), b.view(np.uint16))


def test_g_idx_out_of_range_is_rejected():
    case = workloads.make_case(1, 64, 8, 32, seed=1)
    bad = np.zeros(64, np.int32)
    bad[17] = 2
    with pytest.raises(ValueError):
        oracle.dequant(case["qweight"], case["qzeros"], case["scales"], bad, 32)
    bad[17] = -1
    with pytest.raises(ValueError):
        oracle.gemm_ref(case["x"], case["qweight"], case["qzeros"], case["scales"], bad, 32)


def test_joint_row_permutation_leaves_reference_unchanged():
    # permuting the K axis of x, of the codes and of g_idx together is a reordering of the sum only
    case = workloads.make_case(2, 128, 16, 32, seed=9, act_order=True)
    q = oracle.unpack_qweight(case["qweight"])
    perm = np.random.default_rng(3).permutation(128)
    qp = oracle.pack_qweight(q[perm])
    xp = np.ascontiguousarray(case["x"][:, perm])
    gp = np.ascontiguousarray(case["g_idx"][perm])
    a = oracle.gemm_ref(case["x"], case["qweight"], case["qzeros"], case["scales"], case["g_idx"], 32)
    b = oracle.gemm_ref(xp, qp, case["qzeros"], case["scales"], gp, 32)
    assert np.allclose(a, b, rtol=0, atol=1e-12)


# --------------------------------------------------------------------------------------
# O6: the fp64 reference
# --------------------------------------------------------------------------------------

def test_gemm_hand_case_closed_form():
    # weights of test_dequant_hand_case_closed_form, x = [1, 2, ..., 8]:
    # ref[n] = sum_k (k+1)(k-8-n)/2 = (168 - 36(8+n))/2 = -60 - 18n
    qweight = u32([[0x76543210] * 8])
    qzeros = u32([[0xFEDCBA98]])
    scales = np.full((1, 8), 0.5, F16)
    x = np.arange(1, 9, dtype=F16)[None, :]
    ref = oracle.gemm_ref(x, qweight, qzeros, scales, None, 8)
    assert ref.tolist() == [[-60.0, -78.0, -96.0, -114.0, -132.0, -150.0, -168.0, -186.0]]


def test_gemm_one_hot_selects_weight_rows_exactly():
    case = workloads.make_weights(256, 40, 64, seed=21, act_order=True)
    hot = [0, 7, 8, 129, 255]
    x = workloads.one_hot_activations(len(hot), 256, hot)
    w = oracle.dequant(case["qweight"], case["qzeros"], case["scales"], case["g_idx"], 64)
    ref = oracle.gemm_ref(x, case["qweight"], case["qzeros"], case["scales"], case["g_idx"], 64)
    for m, j in enumerate(hot):
        assert np.array_equal(ref[m], w[j].astype(np.float64))


def test_gemm_constant_codes_closed_form():
    # every code c, every zero point zc, scale 2^-7: ref[m, n] = 2^-7 (c - zc) * sum_k x[m, k], exact for ternary x
    K, N, M = 512, 24, 3
    c, zc = 11, 4
    qweight = u32([[0x11111111 * c] * N for _ in range(K // 8)])
    qzeros = u32([[0x11111111 * zc] * (N // 8) for _ in range(K // 128)])
    scales = np.full((K // 128, N), 2.0 ** -7, F16)
    x = workloads.ternary_activations(M, K, seed=2)
    ref = oracle.gemm_ref(x, qweight, qzeros, scales, None, 128)
    row_sums = x.astype(np.int64).sum(axis=1)
    for m in range(M):
        assert np.all(ref[m] == 2.0 ** -7 * (c - zc) * row_sums[m])


def test_gemm_zero_when_codes_equal_zero_points():
    K, N = 256, 16
    z = np.random.default_rng(4).integers(0, 16, size=(2, N), dtype=np.uint8)
    q = np.repeat(z, 128, axis=0)
    x = workloads.make_activations(4, K, seed=4)
    scales = np.full((2, N), 0.01, F16)
    ref = oracle.gemm_ref(x, oracle.pack_qweight(q), oracle.pack_qzeros(z), scales, None, 128)
    assert np.all(ref == 0.0)


def test_gemm_against_library_fp64_matmul():
    # distinct M, K, N so that a transposed operand or a swapped dimension cannot pass
    case = workloads.make_case(5, 384, 72, 128, seed=31, act_order=True)
    w = oracle.dequant(case["qweight"], case["qzeros"], case["scales"], case["g_idx"], 128)
    ref = oracle.gemm_ref(case["x"], case["qweight"], case["qzeros"], case["scales"], case["g_idx"], 128)
    lib = case["x"].astype(np.float64) @ w.astype(np.float64)
    assert ref.shape == (5, 72)
    assert np.allclose(ref, lib, rtol=0, atol=1e-11)
    m_idx, n_idx = workloads.sample_positions(5, 72, 50, seed=1)
    sampled = oracle.gemm_ref_sampled(case["x"], case["qweight"], case["qzeros"], case["scales"], case["g_idx"],
                                      128, m_idx, n_idx)
    assert np.array_equal(sampled, ref[m_idx, n_idx])


def _brute_force(x, qweight, qzeros, scales, g_idx, group):
    """Exact rational arithmetic with Python integers, element by element (tiny inputs only)."""
    M, K = x.shape
    N = qweight.shape[1]
    w16 = np.zeros((K, N), F16)
    ref = [[Fraction(0) for _ in range(N)] for _ in range(M)]
    for k in range(K):
        r = int(g_idx[k]) if g_idx is not None else k // group
        for n in range(N):
            word = int(qweight[k // 8, n]) & 0xFFFFFFFF
            zword = int(qzeros[r, n // 8]) & 0xFFFFFFFF
            code = (word >> (4 * (k % 8))) % 16
            zero = (zword >> (4 * (n % 8))) % 16
            exact = Fraction(float(scales[r, n])) * (code - zero)
            # the exact product has at most 15 significant bits: float() is exact, float16() rounds once
            w16[k, n] = F16(float(exact))
            for m in range(M):
                ref[m][n] += Fraction(float(x[m, k])) * Fraction(float(w16[k, n]))
    return w16, np.array([[float(v) for v in row] for row in ref])


@pytest.mark.parametrize("act_order", [False, True])
def test_brute_force_on_tiny_inputs(act_order):
    case = workloads.make_case(2, 32, 16, 8, seed=41, act_order=act_order)
    w_bf, ref_bf = _brute_force(case["x"], case["qweight"], case["qzeros"], case["scales"], case["g_idx"], 8)
    w = oracle.dequant(case["qweight"], case["qzeros"], case["scales"], case["g_idx"], 8)
    assert np.array_equal(w.view(np.uint16), w_bf.view(np.uint16))
    ref = oracle.gemm_ref(case["x"], case["qweight"], case["qzeros"], case["scales"], case["g_idx"], 8)
    assert np.allclose(ref, ref_bf, rtol=0, atol=1e-13)


def test_half_conversions_against_library():
    bits = np.arange(65536, dtype=np.uint16)
    lib = bits.view(F16).astype(np.float64)
    mine = oracle.half_bits_to_double(bits)
    finite = ~np.isnan(lib)
    assert np.array_equal(mine[finite], lib[finite]) and np.all(np.isnan(mine[~finite]))
    rng = np.random.default_rng(0)
    v = rng.standard_normal(100000) * 10.0 ** rng.uniform(-9, 5, 100000)
    ties = np.array([65519.999, 65520.0, 65504.0, 2.0 ** -25, 2.0 ** -25 * 1.0000001, 3 * 2.0 ** -25, 1.00048828125])
    v = np.concatenate([v, ties, -ties])
    with np.errstate(over="ignore"):
        assert np.array_equal(oracle.double_to_half_bits(v), v.astype(F16).view(np.uint16))

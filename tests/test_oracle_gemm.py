"""Pins for the oracle's de-quantisation and contraction.  The contraction is
the paper's problem statement C[M,N] = A[M,K] x B[K,N] (Section "An Example of
Tilus Program"); the affine group de-quantisation is this build's reading of the
"casting and de-quantizing" step.  Nothing here calls the HIP path."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import qgemm_oracle as O

U, I, F = O.KIND_UINT, O.KIND_INT, O.KIND_FLOAT


def _half(x):
    return np.asarray(x, dtype=np.float16).astype(np.float64)


def test_identity_scale_gives_code_values_exactly():
    rng = np.random.default_rng(0)
    for kind, bits, e, m in [(U, 5, 0, 0), (I, 7, 0, 0), (I, 1, 0, 0), (F, 6, 3, 2), (F, 4, 2, 1)]:
        codes = rng.integers(0, 1 << bits, size=(12, 9), dtype=np.uint8)
        wr, wb = O.dequant_rounded(codes, kind, bits, e, m, np.ones((3, 9)), None, 4, "f16")
        assert np.array_equal(wr, O.code_values(kind, bits, e, m)[codes])
        assert np.array_equal(O.from_bits(wb, "f16"), wr)


@pytest.mark.parametrize("bits", range(1, 9))
def test_uint_with_midpoint_zero_equals_int_with_flipped_sign_bit(bits):
    rng = np.random.default_rng(bits)
    K, N, g = 16, 10, 4
    codes = rng.integers(0, 1 << bits, size=(K, N), dtype=np.uint8)
    s = _half(rng.uniform(0.005, 0.02, size=(K // g, N)))
    z = np.full((K // g, N), 1 << (bits - 1), dtype=np.uint8)
    a, _ = O.dequant_rounded(codes, U, bits, 0, 0, s, z, g, "f16")
    b, _ = O.dequant_rounded(codes ^ (1 << (bits - 1)), I, bits, 0, 0, s, None, g, "f16")
    assert np.array_equal(a, b)


def test_dequant_against_exact_rationals_and_indexing():
    """Every element re-derived with Fractions: catches a wrong group index, a
    transposed scale table, a zero-point added instead of subtracted."""
    rng = np.random.default_rng(7)
    K, N, g, bits = 12, 5, 3, 6
    codes = rng.integers(0, 64, size=(K, N), dtype=np.uint8)
    s = _half(rng.uniform(0.005, 0.02, size=(K // g, N)))
    z = rng.integers(0, 64, size=(K // g, N)).astype(np.uint8)
    w = O.dequant_exact(codes, U, bits, 0, 0, s, z, g)
    for k in range(K):
        for n in range(N):
            want = (Fraction(int(codes[k, n])) - int(z[k // g, n])) * Fraction(float(s[k // g, n]))
            assert Fraction(float(w[k, n])) == want
    wr, _ = O.dequant_rounded(codes, U, bits, 0, 0, s, z, g, "f16")
    assert np.array_equal(wr, w.astype(np.float16).astype(np.float64))


def test_uint8_unit_scale_is_a_plain_integer_matmul():
    rng = np.random.default_rng(8)
    M, K, N = 5, 64, 7
    A = rng.integers(-4, 5, size=(M, K))
    codes = rng.integers(0, 256, size=(K, N), dtype=np.uint8)
    stream = O.pack_canonical(codes, 8)
    C = O.qgemm_from_stream(A, stream, U, 8, 0, 0, np.ones((1, N)), None, K, K, N, "f16")
    assert np.array_equal(C, (A.astype(np.int64) @ codes.astype(np.int64)).astype(np.float64))


@pytest.mark.parametrize("act", ["f16", "bf16"])
def test_one_hot_rows_return_rounded_weight_rows(act):
    rng = np.random.default_rng(9)
    K, N, g, bits = 32, 11, 8, 3
    codes = rng.integers(0, 8, size=(K, N), dtype=np.uint8)
    s = _half(rng.uniform(0.005, 0.02, size=(K // g, N)))
    z = np.full((K // g, N), 4, dtype=np.uint8)
    wr, _ = O.dequant_rounded(codes, U, bits, 0, 0, s, z, g, act)
    rows = [0, 5, 31]
    A = np.zeros((len(rows), K))
    A[np.arange(len(rows)), rows] = 1.0
    C = O.qgemm_from_stream(A, O.pack_canonical(codes, bits), U, bits, 0, 0, s, z, g, K, N, act)
    assert np.array_equal(C, wr[rows])


def test_all_equal_codes_factor_out():
    rng = np.random.default_rng(10)
    M, K, N = 3, 40, 6
    A = _half(rng.standard_normal((M, K)))
    codes = np.full((K, N), 5, dtype=np.uint8)
    s = np.full((1, N), float(np.float16(0.0137)))
    z = np.full((1, N), 2, dtype=np.uint8)
    C = O.qgemm_from_stream(A, O.pack_canonical(codes, 4), U, 4, 0, 0, s, z, K, K, N, "f16")
    w = float(np.float16(3 * float(np.float16(0.0137))))
    assert np.allclose(C, (A.sum(axis=1) * w)[:, None], rtol=1e-13, atol=1e-15)


@pytest.mark.parametrize("bits", range(1, 9))
@pytest.mark.parametrize("gsel", ["one", "two", "K"])
def test_brute_force_triple_loop_on_tiny_shapes(bits, gsel):
    rng = np.random.default_rng(1000 + bits)
    M, K, N = 3, 8, 5                                 # non-square: a transposed operand cannot pass
    g = {"one": 1, "two": 2, "K": K}[gsel]
    kind = I if bits % 2 else U
    A = _half(rng.standard_normal((M, K)))
    codes = rng.integers(0, 1 << bits, size=(K, N), dtype=np.uint8)
    s = _half(rng.uniform(0.005, 0.02, size=(K // g, N)))
    z = rng.integers(0, 1 << bits, size=(K // g, N)).astype(np.uint8) if kind == U else None
    stream = O.pack_canonical(codes, bits)
    C = O.qgemm_from_stream(A, stream, kind, bits, 0, 0, s, z, g, K, N, "f16")
    tab = O.code_values(kind, bits)
    for mm in range(M):
        for n in range(N):
            acc = Fraction(0)
            for k in range(K):
                c = int(O.unpack_elements(stream, bits, np.array([k * N + n]))[0])
                zz = 0 if z is None else int(z[k // g, n])
                w = (Fraction(float(tab[c])) - zz) * Fraction(float(s[k // g, n]))
                w16 = Fraction(float(np.float16(float(w))))        # correctly rounded half
                acc += Fraction(float(A[mm, k])) * w16
            assert abs(float(acc) - C[mm, n]) <= 1e-12 * (1 + abs(float(acc)))


def test_linearity_in_A_and_column_subset():
    rng = np.random.default_rng(11)
    M, K, N, g, bits = 4, 64, 24, 16, 5
    A1, A2 = rng.standard_normal((M, K)), rng.standard_normal((M, K))
    codes = rng.integers(0, 32, size=(K, N), dtype=np.uint8)
    s = _half(rng.uniform(0.005, 0.02, size=(K // g, N)))
    z = np.full((K // g, N), 16, dtype=np.uint8)
    st = O.pack_canonical(codes, bits)
    f = lambda A, cols=None: O.qgemm_from_stream(A, st, U, bits, 0, 0, s, z, g, K, N, "bf16", cols=cols, col_block=7)
    assert np.allclose(f(A1 + 2 * A2), f(A1) + 2 * f(A2), rtol=1e-12, atol=1e-12)
    cols = np.array([23, 0, 7, 7, 12])
    assert np.allclose(f(A1, cols), f(A1)[:, cols], rtol=1e-13, atol=1e-14)   # BLAS blocking may differ


def test_rounded_and_unrounded_contractions_differ_beyond_rounding_noise():
    """The contraction runs over the ROUNDED weights; make sure the oracle is
    on that side (a contraction over unrounded w gives a measurably different C)."""
    rng = np.random.default_rng(12)
    M, K, N = 2, 4096, 8
    A = _half(rng.standard_normal((M, K)))
    codes = rng.integers(0, 256, size=(K, N), dtype=np.uint8)
    s = _half(rng.uniform(0.01, 0.1, size=(1, N)))
    C = O.qgemm_from_stream(A, O.pack_canonical(codes, 8), I, 8, 0, 0, s, None, K, K, N, "bf16")
    w = O.dequant_exact(codes, I, 8, 0, 0, s, None, K)
    C_unrounded = A @ w
    C_rounded = A @ O.round_rne(w, "bf16")
    assert np.array_equal(C, C_rounded)
    assert np.max(np.abs(C - C_unrounded)) > 1e-3


def test_tolerance_predicate():
    ref = np.array([0.0, 1.0, -100.0])
    assert O.within_tolerance(ref + np.array([0.0099, 0.0149, 0.5]), ref).tolist() == [True, True, True]
    assert O.within_tolerance(ref + np.array([0.0101, 0.0151, 0.52]), ref).tolist() == [False, False, False]

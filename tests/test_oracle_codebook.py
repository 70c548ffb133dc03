"""Pins of the oracle's codebook leg (no GPU): each checks codebook_exact / codebook_rounded /
qgemm_codebook_from_stream against something other than itself -- tables that must reproduce
the already pinned integer and float types, exact rationals, numpy's and torch's half and
bfloat16 casts, one-hot rows -- chosen so that a dropped scale, a wrong group index, a
transposed operand, a table indexed by value instead of by code or a second rounding fails."""
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import qgemm_oracle as O

U, I, F = O.KIND_UINT, O.KIND_INT, O.KIND_FLOAT


def _levels(seed, bits):
    """2^bits distinct half-precision levels in (-1.5, 1.5), unsorted on purpose."""
    rng = np.random.default_rng(seed)
    lv = rng.uniform(-1.5, 1.5, size=1 << bits).astype(np.float16)
    return lv.astype(np.float64)


def _draw(seed, K, N, bits, group):
    rng = np.random.default_rng(seed)
    codes = rng.integers(0, 1 << bits, size=(K, N), dtype=np.uint8)
    scales = rng.uniform(0.005, 0.02, size=(K // group, N)).astype(np.float16).astype(np.float64)
    return codes, scales


@pytest.mark.parametrize("bits", range(1, 9))
@pytest.mark.parametrize("act", ["f16", "bf16"])
def test_table_of_uint_values_minus_a_zero_point_is_the_affine_integer_type(bits, act):
    # table[q] = q - z for one z: the codebook form must give the affine form's bits
    K, N, group = 64, 12, 16
    codes, scales = _draw(bits, K, N, bits, group)
    z = (1 << bits) // 2
    table = np.arange(1 << bits, dtype=np.float64) - z
    zeros = np.full((K // group, N), z, dtype=np.uint8)
    want, want_bits = O.dequant_rounded(codes, U, bits, 0, 0, scales, zeros, group, act)
    got, got_bits = O.codebook_rounded(codes, table, scales, group, act)
    assert np.array_equal(got_bits, want_bits) and np.array_equal(got, want)


@pytest.mark.parametrize("bits,e,m", [(3, 1, 1), (4, 2, 1), (5, 2, 2), (6, 3, 2), (7, 3, 3)])
def test_table_of_float_code_values_is_the_float_type(bits, e, m):
    K, N, group = 32, 10, 8
    codes, scales = _draw(20 + bits, K, N, bits, group)
    table = O.code_values(F, bits, e, m)
    want, want_bits = O.dequant_rounded(codes, F, bits, e, m, scales, None, group, "f16")
    got, got_bits = O.codebook_rounded(codes, table, scales, group, "f16")
    assert np.array_equal(got_bits, want_bits)


def test_table_is_indexed_by_code_not_by_rank_or_value():
    # a permuted table with the inverse permutation applied to the codes gives the same weights
    bits, K, N, group = 4, 32, 6, 8
    codes, scales = _draw(5, K, N, bits, group)
    table = _levels(6, bits)
    perm = np.random.default_rng(7).permutation(1 << bits)
    inv = np.argsort(perm)
    a = O.codebook_exact(codes, table, scales, group)
    b = O.codebook_exact(inv[codes].astype(np.uint8), table[perm], scales, group)
    assert np.array_equal(a, b)
    # and a table entry is what a one-code matrix returns
    for q in (0, 3, 15):
        w = O.codebook_exact(np.full((8, 2), q, dtype=np.uint8), table, np.ones((1, 2)), 8)
        assert np.all(w == table[q])


@pytest.mark.parametrize("bits,group", [(2, 2), (3, 4), (5, 1), (8, 8)])
def test_exact_rational_evaluation_and_single_rounding(bits, group):
    K, N = 8, 5
    codes, scales = _draw(40 + bits, K, N, bits, group)
    table = _levels(41 + bits, bits)
    w = O.codebook_exact(codes, table, scales, group)
    _, bits16 = O.codebook_rounded(codes, table, scales, group, "f16")
    _, bitsb = O.codebook_rounded(codes, table, scales, group, "bf16")
    for k in range(K):
        for n in range(N):
            exact = Fraction(float(table[codes[k, n]])) * Fraction(float(scales[k // group, n]))
            assert Fraction(float(w[k, n])) == exact          # the fp64 product of two halves is exact
            # one rounding: numpy's / torch's own casts of the exact product
            h = np.float64(float(exact)).astype(np.float16)
            assert int(bits16[k, n]) == int(h.view(np.uint16))
            b = torch.tensor(float(exact), dtype=torch.float64).to(torch.bfloat16)
            assert int(bitsb[k, n]) == int(b.view(torch.int16).item()) & 0xffff


def test_group_index_runs_along_k_and_scales_are_per_column():
    bits, K, N, group = 3, 16, 4, 4
    codes = np.full((K, N), 5, dtype=np.uint8)
    table = np.zeros(8); table[5] = 1.0
    scales = (np.arange((K // group) * N, dtype=np.float64).reshape(K // group, N) + 1.0) / 64.0
    w = O.codebook_exact(codes, table, scales, group)
    for k in range(K):
        for n in range(N):
            assert w[k, n] == scales[k // group, n]


@pytest.mark.parametrize("bits", [1, 3, 4, 6, 8])
def test_matmul_from_stream_brute_force_and_one_hot(bits):
    M, K, N, group = 3, 16, 7, 8
    rng = np.random.default_rng(60 + bits)
    codes, scales = _draw(61 + bits, K, N, bits, group)
    table = _levels(62 + bits, bits)
    stream = O.pack_canonical(codes.reshape(-1), bits)
    A = rng.standard_normal((M, K)).astype(np.float16).astype(np.float64)
    got = O.qgemm_codebook_from_stream(A, stream, bits, table, scales, group, K, N, "f16")
    for m in range(M):
        for n in range(N):
            total = Fraction(0)
            for k in range(K):
                w = np.float64(table[codes[k, n]] * scales[k // group, n]).astype(np.float16)
                total += Fraction(float(A[m, k])) * Fraction(float(w))
            assert abs(Fraction(float(got[m, n])) - total) <= Fraction(1, 10 ** 12) * (1 + abs(total))
    # one-hot rows pick rows of the rounded weight, so C is not W transposed or shifted
    E = np.zeros((K, K)); E[np.arange(K), np.arange(K)] = 1.0
    wr, _ = O.codebook_rounded(codes, table, scales, group, "f16")
    got = O.qgemm_codebook_from_stream(E, stream, bits, table, scales, group, K, N, "f16")
    assert np.array_equal(got, wr)
    # a subset of columns equals the same columns of the full result
    cols = np.array([6, 0, 3])
    sub = O.qgemm_codebook_from_stream(A, stream, bits, table, scales, group, K, N, "f16", cols=cols)
    full = O.qgemm_codebook_from_stream(A, stream, bits, table, scales, group, K, N, "f16")
    assert np.array_equal(sub, full[:, cols])


def test_out_of_range_code_is_refused():
    with pytest.raises(AssertionError):
        O.codebook_exact(np.full((4, 4), 9, dtype=np.uint8), np.zeros(8), np.ones((1, 4)), 4)

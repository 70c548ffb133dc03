"""Pins of the oracle's int8-activation leg (no GPU): each checks qgemm_int8 against
something other than itself -- numpy's integer matmul, exact rationals, the already pinned
16-bit-activation contraction where that one is exact, and algebraic identities that a
dropped term, a wrong sign, a transposed operand or a wrong group index would break."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import qgemm_oracle as O

U, I = O.KIND_UINT, O.KIND_INT


def _draw(seed, M, K, N, kind, bits, group, zeros=True):
    rng = np.random.default_rng(seed)
    A8 = rng.integers(-128, 128, size=(M, K), dtype=np.int8)
    codes = rng.integers(0, 1 << bits, size=(K, N), dtype=np.uint8)
    G = K // group
    scales = rng.uniform(0.005, 0.02, size=(G, N)).astype(np.float16).astype(np.float64)
    z = rng.integers(0, 1 << bits, size=(G, N), dtype=np.uint8) if zeros else None
    a_scale = rng.uniform(0.01, 0.1, size=M).astype(np.float32)
    return A8, a_scale, codes, scales, z


@pytest.mark.parametrize("kind,bits", [(U, 1), (U, 3), (U, 4), (U, 8), (I, 2), (I, 5), (I, 8)])
def test_unit_scales_give_numpy_integer_matmul(kind, bits):
    # scales 1, no zero-points, no activation scale: C is the plain integer product
    A8, _, codes, scales, _ = _draw(10 + bits, 9, 96, 20, kind, bits, 32, zeros=False)
    values = O.code_values(kind, bits).astype(np.int64)[codes]
    want = A8.astype(np.int64) @ values
    got = O.qgemm_int8(A8, None, codes, kind, bits, np.ones_like(scales), None, 32)
    assert np.array_equal(got, want.astype(np.float64))


def test_inner_sums_are_exact_against_int64_on_a_long_k():
    # worst case magnitudes over K = 4096 in one group: float64 products and sums stay exact
    rng = np.random.default_rng(3)
    K, N, M = 4096, 24, 5
    A8 = np.where(rng.integers(0, 2, size=(M, K)) == 1, 127, -128).astype(np.int8)
    codes = np.where(rng.integers(0, 2, size=(K, N)) == 1, 255, 0).astype(np.uint8)
    z = np.full((1, N), 3, dtype=np.uint8)
    want = A8.astype(np.int64) @ (codes.astype(np.int64) - 3)
    got = O.qgemm_int8(A8, None, codes, U, 8, np.ones((1, N)), z, K)
    assert np.array_equal(got, want.astype(np.float64)) and np.abs(want).max() > 1e6


@pytest.mark.parametrize("kind,bits,group", [(U, 3, 2), (I, 4, 4), (U, 6, 8), (I, 7, 1)])
def test_exact_rational_triple_loop_on_tiny_non_square_shapes(kind, bits, group):
    M, K, N = 3, 8, 5
    A8, a_scale, codes, scales, z = _draw(100 + bits, M, K, N, kind, bits, group)
    got = O.qgemm_int8(A8, a_scale, codes, kind, bits, scales, z, group)
    half = 1 << (bits - 1)
    for m in range(M):
        for n in range(N):
            total = Fraction(0)
            for g in range(K // group):
                inner = 0
                for k in range(g * group, (g + 1) * group):
                    c = int(codes[k, n])
                    v = c if kind == U else (c - (1 << bits) if c >= half else c)
                    inner += int(A8[m, k]) * (v - int(z[g, n]))
                total += Fraction(float(scales[g, n])) * inner
            total *= Fraction(float(a_scale[m]))
            assert abs(Fraction(float(got[m, n])) - total) <= abs(total) * Fraction(1, 1 << 48) + Fraction(1, 1 << 60)


def test_agrees_with_the_16_bit_activation_contraction_where_that_one_is_exact():
    # power-of-two scales make (q - z) * s exactly representable in fp16, and int8 values are
    # fp16 numbers: the rounded-weight contraction of the other leg is then this same sum
    rng = np.random.default_rng(7)
    M, K, N, group, bits = 6, 256, 40, 64, 5
    A8 = rng.integers(-128, 128, size=(M, K), dtype=np.int8)
    codes = rng.integers(0, 1 << bits, size=(K, N), dtype=np.uint8)
    scales = np.ldexp(1.0, rng.integers(-8, -2, size=(K // group, N)))
    z = rng.integers(0, 1 << bits, size=(K // group, N), dtype=np.uint8)
    wr, _ = O.dequant_rounded(codes, U, bits, 0, 0, scales, z, group, "f16")
    assert np.array_equal(wr, O.dequant_exact(codes, U, bits, 0, 0, scales, z, group))
    want = O.gemm_fp64(A8.astype(np.float64), wr)
    got = O.qgemm_int8(A8, None, codes, U, bits, scales, z, group)
    assert np.allclose(got, want, rtol=1e-13, atol=1e-9)
    stream = O.pack_canonical(codes, bits)
    via = O.qgemm_int8_from_stream(A8, None, stream, U, bits, scales, z, group, K, N)
    assert np.array_equal(via, got)
    sub = np.array([0, 39, 7, 7, 20])
    assert np.array_equal(O.qgemm_int8_from_stream(A8, None, stream, U, bits, scales, z, group, K, N, cols=sub), got[:, sub])


def test_zero_point_equals_the_row_sum_form():
    # sum a (q - z) = sum a q - z * sum a, per group
    A8, a_scale, codes, scales, z = _draw(21, 7, 128, 16, U, 4, 32)
    full = O.qgemm_int8(A8, a_scale, codes, U, 4, scales, z, 32)
    noz = O.qgemm_int8(A8, a_scale, codes, U, 4, scales, None, 32)
    rowsum = A8.astype(np.int64).reshape(7, 4, 32).sum(axis=2)                  # [M, groups]
    corr = (rowsum[:, :, None] * (z.astype(np.float64) * scales)[None]).sum(axis=1) * a_scale.astype(np.float64)[:, None]
    assert np.allclose(full, noz - corr, rtol=1e-12, atol=1e-12)
    assert not np.allclose(full, noz)


def test_uint_with_mid_zero_point_is_the_signed_type_with_its_sign_bit_flipped():
    A8, a_scale, codes, scales, _ = _draw(22, 4, 64, 12, U, 6, 64, zeros=False)
    z = np.full((1, 12), 32, dtype=np.uint8)
    as_uint = O.qgemm_int8(A8, a_scale, codes, U, 6, scales, z, 64)
    as_int = O.qgemm_int8(A8, a_scale, codes ^ 32, I, 6, scales, None, 64)
    assert np.array_equal(as_uint, as_int)


def test_one_hot_rows_return_the_scaled_integer_weights_and_groups_do_not_mix():
    A8, _, codes, scales, z = _draw(23, 8, 64, 10, I, 5, 16)
    rows = np.array([0, 15, 16, 17, 31, 32, 48, 63])
    A8[:] = 0
    A8[np.arange(8), rows] = 1
    got = O.qgemm_int8(A8, None, codes, I, 5, scales, z, 16)
    want = O.dequant_exact(codes, I, 5, 0, 0, scales, z, 16)[rows]
    assert np.array_equal(got, want)
    a_scale = np.arange(1, 9, dtype=np.float32)
    assert np.array_equal(O.qgemm_int8(A8, a_scale, codes, I, 5, scales, z, 16), want * a_scale[:, None].astype(np.float64))


def test_float_weights_are_refused():
    with pytest.raises(ValueError):
        O.qgemm_int8(np.zeros((1, 8), np.int8), None, np.zeros((8, 1), np.uint8), O.KIND_FLOAT, 4, np.ones((1, 1)), None, 8)

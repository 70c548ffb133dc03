"""Pins for the oracle's code->value tables and its single RNE rounding.
Type families: paper, Section "Key Ideas" (uint1-8, int2-8, float3-8 with any
exponent/mantissa split).  Nothing here calls the HIP path."""
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import qgemm_oracle as O
from conftest import read_golden


# ---------------------------------------------------------------- integers
@pytest.mark.parametrize("bits", range(1, 9))
def test_uint_and_int_closed_forms(bits):
    n = 1 << bits
    u = O.code_values(O.KIND_UINT, bits)
    assert u.tolist() == list(range(n))
    i = O.code_values(O.KIND_INT, bits)
    assert i.sum() == -(n // 2)                       # one more negative than positive
    assert i.min() == -(n // 2) and i.max() == n // 2 - 1
    # two's complement: value == code (mod 2^bits), and signed order == code ^ signbit order
    assert all((int(v) - c) % n == 0 for c, v in enumerate(i))
    order = np.argsort(np.arange(n) ^ (n // 2), kind="stable")
    assert np.all(np.diff(i[order]) == 1)
    if bits == 1:
        assert i.tolist() == [0.0, -1.0]


# ------------------------------------------------------------------ floats
def _exact_float(code, bits, e, m):
    bias = (1 << (e - 1)) - 1
    s = (code >> (bits - 1)) & 1
    E = (code >> m) & ((1 << e) - 1)
    M = code & ((1 << m) - 1)
    if E == 0:
        mag = Fraction(M, 1 << m) * Fraction(2) ** (1 - bias)
    else:
        mag = (1 + Fraction(M, 1 << m)) * Fraction(2) ** (E - bias)
    return -mag if s else mag, s


ALL_SPLITS = [(b, e, b - 1 - e) for b in range(3, 9) for e in range(1, b)]


@pytest.mark.parametrize("bits,e,m", ALL_SPLITS)
def test_float_formats_against_exact_rationals(bits, e, m):
    v = O.code_values(O.KIND_FLOAT, bits, e, m)
    bias = (1 << (e - 1)) - 1
    for code in range(1 << bits):
        want, s = _exact_float(code, bits, e, m)
        if (e, m) == (4, 3) and (code & 0x7F) == 0x7F:
            assert np.isnan(v[code])
            continue
        assert Fraction(float(v[code])) == want
        assert np.signbit(v[code]) == bool(s)         # -0 keeps its sign
    half = 1 << (bits - 1)
    fin = np.isfinite(v[:half])
    assert np.all(np.diff(v[:half][fin]) > 0)         # monotone within a sign
    assert np.array_equal(v[half:][fin], -v[:half][fin])
    if m > 0:
        assert v[1] == 2.0 ** (1 - bias - m)          # smallest subnormal
    assert v[0] == 0 and not np.signbit(v[0]) and v[half] == 0 and np.signbit(v[half])


def test_named_formats_extremes_and_counts():
    e2m1 = O.code_values(O.KIND_FLOAT, 4, 2, 1)
    assert sorted(set(np.abs(e2m1).tolist())) == [0, 0.5, 1, 1.5, 2, 3, 4, 6]
    e3m2 = O.code_values(O.KIND_FLOAT, 6, 3, 2)
    assert np.nanmax(e3m2) == 28 and np.isfinite(e3m2).all()
    e4m3 = O.code_values(O.KIND_FLOAT, 8, 4, 3)
    assert np.nanmax(e4m3) == 448
    assert O.finite_codes(O.KIND_FLOAT, 4, 2, 1).size == 16
    assert O.finite_codes(O.KIND_FLOAT, 6, 3, 2).size == 64
    f8 = O.finite_codes(O.KIND_FLOAT, 8, 4, 3)
    assert f8.size == 254 and 0x7F not in f8 and 0xFF not in f8


def test_e4m3_table_equals_torch_float8_e4m3fn():
    codes = torch.arange(256, dtype=torch.uint8)
    lib = codes.view(torch.float8_e4m3fn).to(torch.float64).numpy()
    mine = O.code_values(O.KIND_FLOAT, 8, 4, 3)
    fin = np.isfinite(mine)
    assert fin.sum() == 254 and np.isnan(lib[~fin]).all()
    assert np.array_equal(mine[fin], lib[fin])
    assert np.array_equal(np.signbit(mine[fin]), np.signbit(lib[fin]))


def test_e5m2_formula_equals_torch_where_torch_is_finite():
    # torch's e5m2 reserves E=31 for inf/nan; below that the bias/subnormal rule is the same
    codes = torch.arange(256, dtype=torch.uint8)
    lib = codes.view(torch.float8_e5m2).to(torch.float64).numpy()
    mine = O.code_values(O.KIND_FLOAT, 8, 5, 2)
    ok = ((np.arange(256) >> 2) & 31) != 31
    assert np.array_equal(mine[ok], lib[ok])
    assert np.isfinite(mine).all()                    # our reading: no inf, no nan here


def test_formula_reproduces_ieee_half_for_all_finite_patterns():
    # the same sign|exponent|mantissa rule with e=5, m=10 must give IEEE binary16
    c = np.arange(1 << 16, dtype=np.int64)
    bias, m = 15, 10
    E = (c >> m) & 31
    frac = (c & 1023) / 1024.0
    v = np.where(E == 0, np.ldexp(frac, 1 - bias), np.ldexp(1 + frac, E - bias))
    v = np.where(c >> 15 == 1, -v, v)
    lib = c.astype(np.uint16).view(np.float16).astype(np.float64)
    ok = E != 31
    assert np.array_equal(v[ok], lib[ok])
    # and the oracle's from_bits/to_bits are inverse on every finite pattern
    u = c.astype(np.uint16)[ok]
    assert np.array_equal(O.to_bits(O.from_bits(u, "f16"), "f16"), u)


# ---------------------------------------------------------------- rounding
def _all_finite(fmt):
    u = np.arange(1 << 16, dtype=np.uint16)
    v = O.from_bits(u, fmt)
    ok = np.isfinite(v)
    return u[ok], v[ok]


def _nearest_even_by_search(x: Fraction, grid_vals, grid_bits):
    """Correct rounding by brute-force search in the sorted table of all values."""
    import bisect
    fr = [Fraction(float(g)) for g in grid_vals]
    i = bisect.bisect_left(fr, x)
    cands = [j for j in (i - 1, i) if 0 <= j < len(fr)]
    best = min(cands, key=lambda j: (abs(fr[j] - x), grid_bits[j] & 1))
    return grid_bits[best]


@pytest.mark.parametrize("fmt", ["f16", "bf16"])
def test_rounding_matches_brute_force_nearest_even(fmt):
    u, v = _all_finite(fmt)
    pos = ~np.signbit(v)
    order = np.argsort(v[pos], kind="stable")
    gv, gb = v[pos][order], u[pos][order]
    small = gv < 1e4 if fmt == "f16" else gv < 1e6
    gv, gb = gv[small], gb[small]
    rng = np.random.default_rng(3)
    xs = []
    # products (q - z) * s as they occur, plus midpoints and subnormal-range values
    s_bits = rng.integers(0x0400, 0x3000, size=150).astype(np.uint16)
    for sb in s_bits:
        s = float(np.array([sb], dtype=np.uint16).view(np.float16)[0])
        xs.append(Fraction(s) * int(rng.integers(1, 256)))
    for k in rng.integers(1, len(gv) - 1, size=100):
        xs.append((Fraction(float(gv[k])) + Fraction(float(gv[k + 1]))) / 2)   # exact ties
    xs += [Fraction(float(gv[1])) / 2, Fraction(float(gv[1])) * 3 / 2, Fraction(float(gv[1])) / 4]
    for x in xs:
        want = _nearest_even_by_search(x, gv.tolist(), gb.tolist())
        xf = float(x)
        assert Fraction(xf) == x                      # exactly representable in fp64
        got = int(O.to_bits(O.round_rne(np.array([xf]), fmt), fmt)[0])
        assert got == want, (fmt, xf, hex(got), hex(want))
        gotn = int(O.to_bits(O.round_rne(np.array([-xf]), fmt), fmt)[0])
        assert gotn == want | 0x8000


def test_f16_rounding_equals_numpy_half_cast():
    rng = np.random.default_rng(4)
    x = np.concatenate([
        rng.standard_normal(200000) * 10.0 ** rng.integers(-9, 5, size=200000),
        np.array([0.0, -0.0, 65504.0, 65519.99, 65520.0, 1e6, -1e6, 2.0 ** -24, 2.0 ** -25,
                  3 * 2.0 ** -26, 2.0 ** -14, 2.0 ** -14 - 2.0 ** -26]),
    ])
    lib = x.astype(np.float16)
    mine = O.round_rne(x, "f16")
    assert np.array_equal(mine, lib.astype(np.float64))
    assert np.array_equal(np.signbit(mine), np.signbit(lib))
    # every midpoint between neighbouring halves goes to the even one
    u, v = _all_finite("f16")
    p = np.sort(v[v >= 0])
    mid = (p[:-1] + p[1:]) / 2
    assert np.array_equal(O.round_rne(mid, "f16"), mid.astype(np.float16).astype(np.float64))


def test_bf16_rounding_equals_torch_cast_on_float32_inputs():
    rng = np.random.default_rng(5)
    x32 = (rng.standard_normal(200000) * 10.0 ** rng.integers(-20, 20, size=200000)).astype(np.float32)
    u, v = _all_finite("bf16")
    p = np.sort(v[(v >= 0) & (v < 1e30)])
    mid = ((p[:-1] + p[1:]) / 2).astype(np.float32)          # midpoints are exact in fp32
    x32 = np.concatenate([x32, mid, -mid])
    lib = torch.from_numpy(x32).to(torch.bfloat16)
    lib_bits = lib.view(torch.int16).numpy().view(np.uint16)
    mine = O.round_rne(x32.astype(np.float64), "bf16")
    assert np.array_equal(O.to_bits(mine, "bf16"), lib_bits)


def test_hand_derived_ties():
    g = read_golden("rounding.txt")
    s = O.from_bits(np.array([int(g["f16_tie_scale_bits"][0], 16)], dtype=np.uint16), "f16")[0]
    k = int(g["f16_tie_multiplier"][0])
    assert Fraction(float(s)) == Fraction(1, 128) * (1 + Fraction(287, 1024))
    got = int(O.to_bits(O.round_rne(np.array([k * s]), "f16"), "f16")[0])
    assert got == int(g["f16_tie_rne_bits"][0], 16) != int(g["f16_tie_half_away_bits"][0], 16)
    for tag in ("a", "b"):
        num, den = (int(t) for t in g[f"bf16_tie_{tag}_num_den"])
        got = int(O.to_bits(O.round_rne(np.array([num / den]), "bf16"), "bf16")[0])
        assert got == int(g[f"bf16_tie_{tag}_bits"][0], 16)


def test_every_pattern_round_trips():
    for fmt in ("f16", "bf16"):
        u, v = _all_finite(fmt)
        assert np.array_equal(O.round_rne(v, fmt), v)
        assert np.array_equal(O.to_bits(v, fmt), u)


def test_e8m0_block_scales_are_powers_of_two_and_match_torch():
    import torch
    e = np.arange(256, dtype=np.uint8)
    v = O.e8m0_values(e)
    assert v[127] == 1.0 and v[128] == 2.0 and v[126] == 0.5 and v[0] == 2.0 ** -127 and v[254] == 2.0 ** 127
    assert np.isnan(v[255]) and np.all(v[1:255] == 2.0 * v[0:254])
    if hasattr(torch, "float8_e8m0fnu"):                       # the library's table of the same format
        t = torch.from_numpy(e.copy()).view(torch.float8_e8m0fnu).to(torch.float32).numpy().astype(np.float64)
        assert np.array_equal(t[:255], v[:255]) and np.isnan(t[255])
    # with such scales the rounded weight is the exact product while it stays in range
    codes = np.arange(16, dtype=np.uint8).reshape(16, 1)
    s = O.e8m0_values(np.array([[120]], dtype=np.uint8))
    wr, bits = O.dequant_rounded(codes, O.KIND_FLOAT, 4, 2, 1, s, None, 16, "f16")
    assert np.array_equal(wr, O.code_values(O.KIND_FLOAT, 4, 2, 1)[codes] * 2.0 ** -7)

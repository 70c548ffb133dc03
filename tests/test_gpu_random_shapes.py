"""GPU parity, part 4: seeded random shapes, types, group sizes and layouts with
the library's automatic choices (no knobs), so that every dispatch rule -- row
tiles, strips per workgroup, split-K, row blocks, tile heights, split launches --
is crossed with ragged sizes; two integer cases in three carry a different zero-point per
(group, column).  A second family has long K (1024 .. 8192), where
the tiled kernel splits K into slabs of various lengths.  Each case is compared
in full with the oracle, |C_gpu - C_ref| <= 1e-2 + 5e-3 |C_ref| elementwise."""
import numpy as np
import pytest

from paper_2504_12984_amd import workloads as WL
from gpu_util import Prepared, assert_c_close

pytestmark = pytest.mark.gpu

FLOATS = {3: (1, 1), 4: (2, 1), 5: (2, 2), 6: (3, 2), 7: (3, 3), 8: (4, 3)}


def _random_case(seed: int) -> tuple[WL.Case, int]:
    rng = np.random.default_rng(90000 + seed)
    kind = int(rng.integers(0, 3))
    bits = int(rng.integers(3, 9)) if kind == WL.KIND_FLOAT else int(rng.integers(1, 9))
    e, m = FLOATS[bits] if kind == WL.KIND_FLOAT else (0, 0)
    K = 128 * int(rng.integers(1, 9))
    N = 64 * int(rng.integers(1, 21))
    # M across every regime: one row tile, several, row blocks, 64 / 128 / 256-row tiles
    M = int(rng.choice([rng.integers(1, 17), rng.integers(17, 65), rng.integers(65, 257), rng.integers(257, 641)]))
    groups = [g for g in (64, 128, 256, 512, K) if K % g == 0]
    group = int(rng.choice(groups))
    act = str(rng.choice(["f16", "bf16"]))
    sdt = "f16" if act == "f16" else str(rng.choice(["f16", "bf16"]))
    if kind == WL.KIND_UINT:
        zero = int(rng.integers(0, 1 << bits))
    elif kind == WL.KIND_INT:
        zero = None if rng.integers(0, 2) else int(rng.integers(0, 4))
    else:
        zero = None
    lo, hi = (0.01, 0.1) if kind == WL.KIND_FLOAT else (0.005, 0.02)
    layout = int(rng.integers(0, 2))
    if layout == 0 and rng.integers(0, 4) == 0:        # group size 32 exists on the first layout only
        group = 32
    zero_hi = None
    if kind != WL.KIND_FLOAT and rng.integers(0, 3) > 0:      # two integer cases in three: a zero-point per (group, column)
        zero, zero_hi = "random", int(rng.choice([(1 << bits) - 1, 255]))
    case = WL.Case(f"rand{seed}_k{kind}b{bits}_M{M}_K{K}_N{N}_g{group}_{act}_L{layout}", M, K, N, kind, bits, e, m,
                   group=group, act=act, scale_dtype=sdt, zero=zero, zero_hi=zero_hi, scale_lo=lo, scale_hi=hi,
                   seed=91000 + seed)
    return case, layout


@pytest.mark.parametrize("seed", range(48))
def test_random_case_matches_oracle(seed):
    case, layout = _random_case(seed)
    P = Prepared(case)
    assert_c_close(P.gpu_c(layout=layout), P.oracle_c(), case.name)


def _random_long_k_case(seed: int) -> WL.Case:
    rng = np.random.default_rng(770000 + seed)
    kind = int(rng.integers(0, 3))
    bits = int(rng.integers(3, 9)) if kind == WL.KIND_FLOAT else int(rng.integers(1, 9))
    e, m = FLOATS[bits] if kind == WL.KIND_FLOAT else (0, 0)
    K = 128 * int(rng.integers(8, 65))
    N = 64 * int(rng.integers(1, 33))
    M = int(rng.choice([rng.integers(1, 65), rng.integers(65, 257), rng.integers(257, 641)]))
    groups = [g for g in (32, 64, 128, 256, 512, K)
              if K % g == 0 and (g == K or g <= 64 or (g // 128) & (g // 128 - 1) == 0)]
    group = int(rng.choice(groups))
    act = str(rng.choice(["f16", "bf16"]))
    sdt = "f16" if act == "f16" else str(rng.choice(["f16", "bf16"]))
    if kind == WL.KIND_UINT:
        zero = int(rng.integers(0, 1 << bits))
    elif kind == WL.KIND_INT:
        zero = None if rng.integers(0, 2) else int(rng.integers(0, 4))
    else:
        zero = None
    lo, hi = (0.01, 0.1) if kind == WL.KIND_FLOAT else (0.005, 0.02)
    zero_hi = None
    if kind != WL.KIND_FLOAT and rng.integers(0, 3) > 0:      # two integer cases in three: a zero-point per (group, column)
        zero, zero_hi = "random", int(rng.choice([(1 << bits) - 1, 255]))
    return WL.Case(f"big{seed}_k{kind}b{bits}_M{M}_K{K}_N{N}_g{group}_{act}", M, K, N, kind, bits, e, m, group=group,
                   act=act, scale_dtype=sdt, zero=zero, zero_hi=zero_hi, scale_lo=lo, scale_hi=hi, seed=771000 + seed)


@pytest.mark.parametrize("seed", range(16))
def test_random_long_k_case_matches_oracle(seed):
    case = _random_long_k_case(seed)
    P = Prepared(case)
    assert_c_close(P.gpu_c(), P.oracle_c(), case.name)

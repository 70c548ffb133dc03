"""GPU parity, part 2b: the matmul on the second device layout (32x32x16 matrix
instruction, one tiled kernel for every M) against the oracle, to the same bar
as the first layout: |C_gpu - C_ref| <= 1e-2 + 5e-3 |C_ref| elementwise, exact
where the arithmetic admits one answer."""
import numpy as np
import pytest
import torch

from paper_2504_12984_amd import workloads as WL
from gpu_util import Prepared, assert_c_close, bits_of, to_f64

pytestmark = pytest.mark.gpu

U, I, F = WL.KIND_UINT, WL.KIND_INT, WL.KIND_FLOAT
FLOATS = [(3, 1, 1), (4, 2, 1), (5, 2, 2), (6, 3, 2), (7, 3, 3), (8, 4, 3)]
R32 = 1


@pytest.fixture(autouse=True)
def _reset_knobs():
    from paper_2504_12984_amd import binding as B
    yield
    for k in range(4):
        B.qg_set_knob(k, 0)


@pytest.mark.parametrize("bm", [128, 256])
@pytest.mark.parametrize("M,K,N", [(1, 128, 64), (16, 256, 128), (65, 128, 64), (200, 512, 256),
                                   (257, 384, 320), (300, 1408, 192), (512, 1024, 512)])
def test_ragged_shapes(M, K, N, bm):
    # rows past M inside a tile, idle wavefronts (N not a multiple of 256), one
    # chunk only, odd and even chunk counts
    from paper_2504_12984_amd import binding as B
    case = WL.Case(f"r32_{M}_{K}_{N}_{bm}", M, K, N, U, 5, group=64, act="bf16", scale_dtype="bf16",
                   zero=16, seed=9700 + M)
    P = Prepared(case)
    B.qg_set_knob(2, bm)
    assert_c_close(P.gpu_c(layout=R32), P.oracle_c(), case.name)


@pytest.mark.parametrize("act", ["f16", "bf16"])
@pytest.mark.parametrize("bits", range(1, 9))
@pytest.mark.parametrize("kind", [U, I])
def test_integer_types(kind, bits, act):
    sdt = "f16" if act == "f16" else "bf16"
    case = WL.Case(f"r32_{kind}_{bits}_{act}", 130, 640, 192, kind, bits, group=64 if bits % 2 else 128,
                   act=act, scale_dtype=sdt, zero=(1 << (bits - 1)) if kind == U else None, seed=9800 + bits)
    P = Prepared(case)
    assert_c_close(P.gpu_c(layout=R32), P.oracle_c(), case.name)


@pytest.mark.parametrize("act", ["f16", "bf16"])
@pytest.mark.parametrize("bits,e,m", FLOATS)
def test_float_types(bits, e, m, act):
    case = WL.Case(f"r32_f{bits}_{act}", 140, 1024, 128, F, bits, e, m, group=1024, act=act, scale_dtype="f16",
                   zero=None, scale_lo=0.01, scale_hi=0.1, seed=9900 + bits)
    P = Prepared(case)
    assert_c_close(P.gpu_c(layout=R32), P.oracle_c(), case.name)


@pytest.mark.parametrize("group", [64, 128, 256, 768])
def test_group_sizes(group):
    case = WL.Case(f"r32_g{group}", 96, 768, 128, U, 4, group=group, act="f16", zero=8, seed=9950 + group)
    P = Prepared(case)
    assert_c_close(P.gpu_c(layout=R32), P.oracle_c(), case.name)


def test_one_hot_rows_return_weight_rows_bit_exactly():
    # ties the matmul to the bit-exact de-quantisation, element by element: every
    # (k, n) of the weight is routed through its own accumulator slot
    for act, kind, bits in (("bf16", I, 6), ("f16", U, 3)):
        case = WL.Case(f"r32_onehot_{act}", 256, 256, 128, kind, bits, group=128, act=act, scale_dtype="f16",
                       zero=None if kind == I else 3, seed=9960)
        inp = WL.make_inputs(case)
        A = torch.zeros((256, 256), dtype=inp["A"].dtype)
        A[torch.arange(256), torch.arange(256)] = 1.0
        inp["A"] = A
        P = Prepared(case, inp)
        _, wbits = P.oracle_w()
        assert np.array_equal(bits_of(P.gpu_c(layout=R32)), wbits), act


def test_uint8_unit_scale_small_integers_is_exact():
    case = WL.Case("r32_int_exact", 150, 256, 128, U, 8, group=256, zero=None, seed=9970)
    inp = WL.make_inputs(case)
    rng = np.random.default_rng(2)
    inp["A"] = torch.from_numpy(rng.integers(-1, 2, size=(150, 256)).astype(np.float32)).to(torch.float16)
    inp["codes"] = rng.integers(0, 8, size=(256, 128), dtype=np.uint8)
    inp["scales"] = torch.ones((1, 128), dtype=torch.float16)
    P = Prepared(case, inp)
    want = to_f64(inp["A"]).astype(np.int64) @ inp["codes"].astype(np.int64)
    assert np.array_equal(to_f64(P.gpu_c(layout=R32)), want.astype(np.float64))


def test_both_layouts_give_the_same_bits_for_one_k_chunk():
    # one chunk of K: both kernels add the same 128 products per element; the
    # orders differ, so only the oracle's tolerance is asserted for each, plus
    # exact equality of the de-quantised weights
    case = WL.Case("r32_vs_r16", 64, 128, 128, U, 4, group=128, act="bf16", scale_dtype="bf16", zero=8, seed=9980)
    P = Prepared(case)
    ref = P.oracle_c()
    assert_c_close(P.gpu_c(layout=0), ref, "layout 0")
    assert_c_close(P.gpu_c(layout=R32), ref, "layout 1")
    assert np.array_equal(bits_of(P.gpu_w(0)), bits_of(P.gpu_w(R32)))


def test_empty_m():
    case = WL.Case("r32_edge", 1, 128, 64, U, 4, group=128, zero=8, seed=9990)
    P = Prepared(case)
    A0 = torch.empty((0, 128), dtype=torch.float16, device="cuda")
    assert P.gpu_c(A0, layout=R32).shape == (0, 64)

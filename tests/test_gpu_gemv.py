"""GPU parity, part 10: the matrix-vector kernel (forced path 5, M <= 4) -- the decode-sized product
on the vector ALU with two-element dot products and an in-wavefront lane-permute reduction, the
measured alternative to the matrix-core streaming kernel.  Same contract: the products are formed
from the bit-exact rounded weights, |C_gpu - C_ref| <= 1e-2 + 5e-3 |C_ref| elementwise, one-hot
rows bit for bit."""
import numpy as np
import pytest
import torch

from oracle import qgemm_oracle as O
from paper_2504_12984_amd import workloads as WL
from gpu_util import Prepared, assert_c_close, bits_of

pytestmark = pytest.mark.gpu

U, I, F = WL.KIND_UINT, WL.KIND_INT, WL.KIND_FLOAT
FLOATS = [(3, 1, 1), (4, 2, 1), (5, 2, 2), (6, 3, 2), (7, 3, 3), (8, 4, 3)]


@pytest.fixture(autouse=True)
def _gemv_path():
    from paper_2504_12984_amd import binding as B
    B.qg_set_knob(0, 5)
    yield
    for k in range(4):
        B.qg_set_knob(k, 0)


@pytest.mark.parametrize("waves", [0, 4, 8, 16])
@pytest.mark.parametrize("M", [1, 2, 3, 4])
def test_gemv_every_row_count_and_wavefront_count(M, waves):
    from paper_2504_12984_amd import binding as B
    # 3 strips, 11 chunks of K: ragged shares per wavefront, idle wavefronts with 16 per strip
    case = WL.Case(f"gemv_M{M}_w{waves}", M, 1408, 192, U, 4, group=128, zero=8, seed=61000 + M)
    P = Prepared(case)
    B.qg_set_knob(3, waves)
    plan = B.qg_plan(P.wtype, case.group, M, case.N, case.K)
    assert plan["path"] == 5 and (waves == 0 or plan["variant"] == (waves if (waves < 16 or M == 1) else 4)), plan
    assert_c_close(P.gpu_c(), P.oracle_c(), case.name)


@pytest.mark.parametrize("act", ["f16", "bf16"])
@pytest.mark.parametrize("bits", range(1, 9))
@pytest.mark.parametrize("kind", [U, I])
def test_gemv_integer_types(kind, bits, act):
    case = WL.Case(f"gemv_{kind}_{bits}_{act}", 1 + bits % 4, 640, 128, kind, bits, group=64 if bits % 2 else 128, act=act,
                   scale_dtype="bf16" if (act == "bf16" and bits > 4) else "f16",
                   zero=("random" if kind == U else None), seed=61100 + 10 * bits + kind)
    P = Prepared(case)
    assert_c_close(P.gpu_c(), P.oracle_c(), case.name)


@pytest.mark.parametrize("act", ["f16", "bf16"])
@pytest.mark.parametrize("bits,e,m", FLOATS)
def test_gemv_float_types(bits, e, m, act):
    case = WL.Case(f"gemv_f{bits}_{act}", 1, 768, 128, F, bits, e, m, group=768, act=act, zero=None,
                   scale_lo=0.01, scale_hi=0.1, seed=61300 + bits)
    P = Prepared(case)
    assert_c_close(P.gpu_c(), P.oracle_c(), case.name)


@pytest.mark.parametrize("group", [32, 64, 256])
def test_gemv_group_sizes(group):
    case = WL.Case(f"gemv_g{group}", 3, 1024, 192, U, 5, group=group, zero="random", seed=61400 + group)
    P = Prepared(case)
    assert_c_close(P.gpu_c(), P.oracle_c(), case.name)


@pytest.mark.parametrize("splitk", [2, 3, 11])
@pytest.mark.parametrize("M", [1, 4])
def test_gemv_split_k_and_counters_left_clean(M, splitk):
    from paper_2504_12984_amd import binding as B
    case = WL.Case(f"gemv_sk{splitk}_M{M}", M, 1408, 320, I, 3, group=128, zero=None, seed=61500 + splitk)
    P = Prepared(case)
    ref = P.oracle_c()
    B.qg_set_knob(1, splitk)
    first = P.gpu_c()
    assert_c_close(first, ref, case.name)
    assert np.array_equal(bits_of(first), bits_of(P.gpu_c()))
    # the streaming kernel shares the counters: it must find them at zero
    B.qg_set_knob(0, 1)
    assert_c_close(P.gpu_c(), ref, case.name + " streaming after")


@pytest.mark.parametrize("act", ["f16", "bf16"])
def test_gemv_one_hot_rows_bit_exact(act):
    K, N = 512, 128
    case = WL.Case(f"gemv_onehot_{act}", 4, K, N, U, 6, group=64, act=act, zero=32, seed=61600)
    inp = WL.make_inputs(case)
    rows = np.array([0, 129, 300, 511])
    A = torch.zeros((4, K), dtype=inp["A"].dtype)
    A[torch.arange(4), torch.from_numpy(rows)] = 1.0
    inp["A"] = A
    P = Prepared(case, inp)
    _, wbits = P.oracle_w()
    want = wbits[rows].copy()
    want[want == 0x8000] = 0
    assert np.array_equal(bits_of(P.gpu_c()), want)


def test_gemv_decode_configuration_full_size():
    # the W3A16 decode configuration at M = 1 and 4, every column
    for M in (1, 4):
        P = Prepared(WL.cfg2(M))
        assert_c_close(P.gpu_c(), P.oracle_c(), f"cfg2 M={M} gemv")


def test_gemv_refuses_more_than_four_rows_and_block_scales():
    from paper_2504_12984_amd import binding as B
    case = WL.Case("gemv_m5", 5, 256, 128, U, 4, group=128, zero=8, seed=61700)
    P = Prepared(case)
    with pytest.raises(B.QgError) as e:
        P.gpu_c()
    assert e.value.status == B.QG_EINVAL

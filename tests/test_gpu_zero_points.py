"""GPU parity, part 5: the matmul with a DIFFERENT zero-point for every (group, column).

The interface takes zero-points as an array [K/group, N]; each matmul kernel has its own
code that fetches them (pointer arithmetic in the streaming kernel, buffer resources with
scalar group offsets in the two tiled kernels), so every kernel, every number of groups per
128-row chunk (group 32 / 64 / 128 and groups that span several chunks), both rounding
routes and split-K are run here with zero-points drawn per (group, column) and compared
with the oracle -- in full, |C_gpu - C_ref| <= 1e-2 + 5e-3 |C_ref| elementwise, and bit for
bit through one-hot rows (a row of C is then a row of the de-quantised weight).
A zero-point read from the wrong group row or column moves a whole group of weights by a
multiple of the scale, far outside the tolerance.
"""
import numpy as np
import pytest
import torch

from paper_2504_12984_amd import workloads as WL
from gpu_util import Prepared, assert_c_close, bits_of

pytestmark = pytest.mark.gpu

U, I = WL.KIND_UINT, WL.KIND_INT


@pytest.fixture(autouse=True)
def _reset_knobs():
    from paper_2504_12984_amd import binding as B
    yield
    for k in range(4):
        B.qg_set_knob(k, 0)


def _case(name, M, K, N, kind, bits, group, act, seed, zero_hi=None):
    sdt = "f16" if act == "f16" else "bf16"
    return WL.Case(name, M, K, N, kind, bits, group=group, act=act, scale_dtype=sdt, zero="random",
                   zero_hi=zero_hi, seed=seed)


def test_random_zero_points_are_really_different_per_group_and_column():
    inp = WL.make_inputs(_case("zp_probe", 1, 1024, 128, U, 4, 128, "f16", 31000))
    z = inp["zeros"]
    assert z.shape == (8, 128) and z.min() == 0 and z.max() == 15
    assert len(np.unique(z[:, 0])) > 2 and len(np.unique(z[0])) > 8


# ---------------------------------------------------------------- streaming kernel (M <= 64)
@pytest.mark.parametrize("act", ["f16", "bf16"])
@pytest.mark.parametrize("group", [32, 64, 128, 256, 1280])
@pytest.mark.parametrize("M", [1, 16, 24, 64])
def test_streaming_kernel_random_zero_points(M, group, act):
    # 10 chunks of K on 5 strips: a ragged share per wavefront; group 256 spans two chunks
    # (the shift form of the group index), group 1280 = K is one scale per column
    from paper_2504_12984_amd import binding as B
    case = _case(f"zp_stream_{M}_{group}_{act}", M, 1280, 320, U, 4, group, act, 31100 + M + group)
    P = Prepared(case)
    ref = P.oracle_c()
    B.qg_set_knob(0, 1)
    assert_c_close(P.gpu_c(), ref, case.name)
    B.qg_set_knob(1, 3)                              # K over three workgroups (slabs of 4, 4, 2 chunks)
    assert_c_close(P.gpu_c(), ref, case.name + " split-K 3")


@pytest.mark.parametrize("variant", [10, 11, 12, 14, 15, 16])
@pytest.mark.parametrize("kind,bits,zero_hi", [(U, 3, None), (I, 5, 3), (U, 8, 255), (U, 2, 255)])
def test_streaming_kernel_arrangements_random_zero_points(kind, bits, zero_hi, variant):
    # every wavefront arrangement (several strips per workgroup changes the column offset of
    # the fetch); zero-points beyond the code range are legal (any uint8)
    from paper_2504_12984_amd import binding as B
    case = _case(f"zp_arr_{kind}_{bits}_{variant}", 9, 1408, 512, kind, bits, 128, "f16", 31300 + bits, zero_hi)
    P = Prepared(case)
    B.qg_set_knob(3, variant)
    assert_c_close(P.gpu_c(), P.oracle_c(), case.name)


# ---------------------------------------------------------------- tiled kernel, first layout
@pytest.mark.parametrize("act", ["f16", "bf16"])
@pytest.mark.parametrize("bm", [64, 128, 256])
@pytest.mark.parametrize("group", [32, 64, 128, 256, 896])
def test_tiled_kernel_random_zero_points(group, bm, act):
    # 7 chunks (odd: the zero-padded chunk), 3 strips (one idle wavefront per workgroup), rows past M
    from paper_2504_12984_amd import binding as B
    K = 896 if group != 256 else 1024
    case = _case(f"zp_tiled_{group}_{bm}_{act}", 150, K, 192, U, 5, group, act, 31500 + group + bm)
    P = Prepared(case)
    ref = P.oracle_c()
    B.qg_set_knob(0, 2)
    B.qg_set_knob(2, bm)
    assert_c_close(P.gpu_c(), ref, case.name)
    if bm <= 128:
        B.qg_set_knob(1, 2)
        assert_c_close(P.gpu_c(), ref, case.name + " split-K 2")


@pytest.mark.parametrize("kind,bits,zero_hi", [(U, 1, 255), (I, 3, 7), (U, 6, None), (U, 8, 255)])
def test_tiled_kernel_types_random_zero_points(kind, bits, zero_hi):
    from paper_2504_12984_amd import binding as B
    case = _case(f"zp_tiled_t{kind}_{bits}", 300, 640, 320, kind, bits, 64, "bf16", 31700 + bits, zero_hi)
    P = Prepared(case)
    B.qg_set_knob(0, 2)
    assert_c_close(P.gpu_c(), P.oracle_c(), case.name)


# ---------------------------------------------------------------- tiled kernel, second layout
@pytest.mark.parametrize("act", ["f16", "bf16"])
@pytest.mark.parametrize("bm", [0, 128, 256])
@pytest.mark.parametrize("group", [64, 128, 256, 896])
def test_second_layout_random_zero_points(group, bm, act):
    from paper_2504_12984_amd import binding as B
    K = 896 if group != 256 else 1024
    case = _case(f"zp_r32_{group}_{bm}_{act}", 150, K, 192, U, 5, group, act, 31800 + group + bm)
    P = Prepared(case)
    B.qg_set_knob(2, bm)
    assert_c_close(P.gpu_c(layout=1), P.oracle_c(), case.name)


@pytest.mark.parametrize("M", [1, 40])
def test_second_layout_small_m_random_zero_points(M):
    case = _case(f"zp_r32_small_{M}", M, 1408, 320, I, 4, 128, "f16", 31900 + M, 15)
    P = Prepared(case)
    assert_c_close(P.gpu_c(layout=1), P.oracle_c(), case.name)


# ---------------------------------------------------------------- bit for bit through one-hot rows
@pytest.mark.parametrize("act", ["f16", "bf16"])
@pytest.mark.parametrize("path,layout,group", [(1, 0, 32), (1, 0, 64), (1, 0, 128), (2, 0, 32), (2, 0, 64),
                                               (2, 0, 128), (2, 1, 64), (2, 1, 128)])
def test_one_hot_rows_with_random_zero_points_are_bit_exact(path, layout, group, act):
    # A = rows of the identity: C[m, :] is row rows[m] of the rounded weight, so a wrong
    # zero-point in ANY (group, column) touched shows as a wrong bit pattern
    from paper_2504_12984_amd import binding as B
    K, N = 512, 192
    rows = np.array([0, 1, 31, 32, 33, 63, 64, 65, 95, 96, 127, 128, 129, 255, 256, 257, 300, 319, 320, 383, 384,
                     385, 415, 416, 447, 448, 479, 480, 481, 509, 510, 511])
    if path == 2:                                    # 80 rows: a 64-row tile and a ragged second one
        rows = np.concatenate([rows, np.random.default_rng(7).integers(0, K, size=48)])
    M = rows.size
    case = _case(f"zp_onehot_{path}_{layout}_{group}_{act}", M, K, N, U, 6, group, act, 32000 + group)
    inp = WL.make_inputs(case)
    A = torch.zeros((M, K), dtype=inp["A"].dtype)
    A[torch.arange(M), torch.from_numpy(rows)] = 1.0
    inp["A"] = A
    P = Prepared(case, inp)
    _, wbits = P.oracle_w()
    if layout == 0:
        B.qg_set_knob(0, path)
    assert np.array_equal(bits_of(P.gpu_c(layout=layout)), wbits[rows]), case.name

"""GPU parity, part 6: the paper's prefill variant as a path of qgemm -- the whole weight is
de-quantised to 16 bits first (into the operand order of the matrix instruction), then a plain
16-bit matmul runs on it (the tiled kernel with its unpack stage replaced by a pass-through).
Selected with the path override 4.  Compared with the oracle like every other path: within
|C_gpu - C_ref| <= 1e-2 + 5e-3 |C_ref| elementwise, bit for bit through one-hot rows; the
weights this path multiplies are the same rounded weights, so its results should also agree
with the fused tiled kernel's bit for bit whenever both use the same tile height and split.
"""
import numpy as np
import pytest
import torch

from paper_2504_12984_amd import workloads as WL
from gpu_util import Prepared, assert_c_close, bits_of

pytestmark = pytest.mark.gpu

U, I, F = WL.KIND_UINT, WL.KIND_INT, WL.KIND_FLOAT


@pytest.fixture(autouse=True)
def _reset_knobs():
    from paper_2504_12984_amd import binding as B
    yield
    for k in range(4):
        B.qg_set_knob(k, 0)


@pytest.mark.parametrize("act", ["f16", "bf16"])
@pytest.mark.parametrize("kind,bits,e,m", [(U, 1, 0, 0), (I, 2, 0, 0), (U, 3, 0, 0), (U, 4, 0, 0), (I, 5, 0, 0), (U, 6, 0, 0),
                                           (I, 7, 0, 0), (U, 8, 0, 0), (F, 3, 1, 1), (F, 4, 2, 1), (F, 5, 2, 2),
                                           (F, 6, 3, 2), (F, 7, 3, 3), (F, 8, 4, 3)])
def test_dense_path_every_weight_type(kind, bits, e, m, act):
    from paper_2504_12984_amd import binding as B
    case = WL.Case(f"dense_t{kind}_{bits}_{act}", 130, 640, 192, kind, bits, e, m, group=128, act=act,
                   scale_dtype="f16", zero="random" if kind != F else None,
                   scale_lo=0.01 if kind == F else 0.005, scale_hi=0.1 if kind == F else 0.02, seed=33000 + bits)
    P = Prepared(case)
    ref = P.oracle_c()
    B.qg_set_knob(0, 2)
    fused = P.gpu_c()
    B.qg_set_knob(0, 4)
    dense = P.gpu_c()
    assert_c_close(dense, ref, case.name)
    assert np.array_equal(bits_of(dense), bits_of(fused)), "the two paths multiply the same rounded weights"


@pytest.mark.parametrize("bm", [0, 64, 128, 256])
@pytest.mark.parametrize("M,K,N,group", [(1, 512, 128, 128), (40, 1408, 320, 32), (200, 512, 256, 64), (257, 384, 320, 128),
                                         (512, 1024, 512, 1024), (700, 896, 192, 128)])
def test_dense_path_ragged_shapes_group_sizes_and_tile_heights(M, K, N, group, bm):
    from paper_2504_12984_amd import binding as B
    case = WL.Case(f"dense_{M}_{K}_{N}_{group}_{bm}", M, K, N, U, 5, group=group, act="bf16", scale_dtype="bf16",
                   zero="random", seed=33100 + M)
    P = Prepared(case)
    B.qg_set_knob(0, 4)
    B.qg_set_knob(2, bm)
    assert_c_close(P.gpu_c(), P.oracle_c(), case.name)


@pytest.mark.parametrize("bm", [64, 128])
@pytest.mark.parametrize("splitk", [2, 3, 11])
def test_dense_path_split_k(splitk, bm):
    from paper_2504_12984_amd import binding as B
    case = WL.Case(f"dense_splitk_{splitk}_{bm}", 150, 1408, 320, I, 4, group=128, act="f16", zero="random", zero_hi=5,
                   seed=33200 + splitk)
    P = Prepared(case)
    ref = P.oracle_c()
    B.qg_set_knob(0, 4); B.qg_set_knob(1, splitk); B.qg_set_knob(2, bm)
    first = P.gpu_c()
    assert_c_close(first, ref, case.name)
    assert np.array_equal(bits_of(first), bits_of(P.gpu_c()))


@pytest.mark.parametrize("act", ["f16", "bf16"])
def test_dense_path_one_hot_rows_bit_exact(act):
    from paper_2504_12984_amd import binding as B
    K, N = 512, 192
    case = WL.Case(f"dense_onehot_{act}", K, K, N, U, 6, group=64, act=act, scale_dtype="f16", zero="random", seed=33300)
    inp = WL.make_inputs(case)
    A = torch.zeros((K, K), dtype=inp["A"].dtype)
    A[torch.arange(K), torch.arange(K)] = 1.0           # C = the rounded weight itself, every element of it
    inp["A"] = A
    P = Prepared(case, inp)
    _, wbits = P.oracle_w()
    B.qg_set_knob(0, 4)
    assert np.array_equal(bits_of(P.gpu_c()), wbits)


def test_dense_path_prefill_configuration_full_size():
    # cfg5 u6 at M = 1024 (whole rounds of 256-row tiles + the second launch): sampled columns for all rows
    import torch as _t
    from oracle import qgemm_oracle as O
    from paper_2504_12984_amd import binding as B
    from gpu_util import to_f64
    case = WL.cfg5(6, 1024)
    P = Prepared(case)
    cols = np.unique(np.concatenate([np.arange(4), np.arange(case.N - 4, case.N),
                                     np.random.default_rng(3).integers(0, case.N, size=64)]))
    B.qg_set_knob(0, 4)
    C = P.gpu_c()
    assert_c_close(C[:, _t.from_numpy(cols).cuda()], P.oracle_c(cols=cols), case.name + " de-quantise first")
    B.qg_set_knob(0, 0)
    assert np.array_equal(bits_of(C), bits_of(P.gpu_c())), "same tiles, same rounded weights: same bits as the fused kernel"


def test_dense_path_buffer_grows_and_is_reused_across_weights_of_different_size():
    # small weight, larger weight (the buffer is replaced), small again; different inputs each time
    from paper_2504_12984_amd import binding as B
    small = Prepared(WL.Case("dense_small", 70, 256, 128, U, 4, group=128, zero=8, seed=33400))
    big = Prepared(WL.Case("dense_big", 300, 1024, 1024, U, 3, group=128, act="bf16", scale_dtype="bf16", zero=4, seed=33401))
    B.qg_set_knob(0, 4)
    outs = [small.gpu_c(), big.gpu_c(), small.gpu_c(), big.gpu_c()]
    torch.cuda.synchronize()
    for P, C in zip([small, big, small, big], outs):
        assert_c_close(C, P.oracle_c(), P.case.name)


def test_dense_path_is_refused_by_the_entry_point_that_allocates_nothing():
    from paper_2504_12984_amd import binding as B
    P = Prepared(WL.Case("dense_noalloc", 70, 256, 128, U, 4, group=128, zero=8, seed=33500))
    out = torch.empty((70, 128), dtype=torch.float16, device="cuda")
    B.qg_set_knob(0, 4)
    with pytest.raises(B.QgError) as err:
        B.qgemm_noalloc(P.d_A, P.d_packed, P.d_scales, P.d_zeros, P.wtype, 128, 128, out)
    assert err.value.status == B.QG_EUNSUPPORTED

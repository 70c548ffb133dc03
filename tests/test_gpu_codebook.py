"""GPU parity, part 9: codebook quantisation (a k-bit code is an index into one table of 2^k
half-precision levels per weight matrix; the group scale multiplies the level; one rounding).

qdequant_codebook is compared bit for bit with the oracle over every code in every lane
position; qgemm_codebook within |C_gpu - C_ref| <= 1e-2 + 5e-3 |C_ref| elementwise, and bit
for bit through one-hot rows.
"""
import numpy as np
import pytest
import torch

from oracle import qgemm_oracle as O
from paper_2504_12984_amd import workloads as WL
from gpu_util import ACT, assert_c_close, bits_of, to_f64

pytestmark = pytest.mark.gpu

CB = WL.KIND_CODEBOOK


@pytest.fixture(autouse=True)
def _reset_knobs():
    from paper_2504_12984_amd import binding as B
    yield
    for k in range(4):
        B.qg_set_knob(k, 0)


class CbCase:
    def __init__(self, case: WL.Case, inputs=None):
        from paper_2504_12984_amd import binding as B
        self.B, self.case = B, case
        c = case
        self.inp = inputs if inputs is not None else WL.make_inputs(c)
        self.wtype = B.WType(B.QG_CODEBOOK, c.bits)
        self.stream = O.pack_canonical(self.inp["codes"], c.bits)
        self.S64 = to_f64(self.inp["scales"])
        self.T64 = to_f64(self.inp["codebook"])
        self.d_scales = self.inp["scales"].cuda()
        self.d_table = self.inp["codebook"].cuda()
        self.d_A = self.inp["A"].cuda()
        self.d_packed = B.repack(torch.from_numpy(self.stream).cuda(), self.wtype, c.K, c.N)

    def oracle_w(self):
        c = self.case
        return O.codebook_rounded(self.inp["codes"], self.T64, self.S64, c.group, c.act)

    def oracle_c(self, cols=None):
        c = self.case
        return O.qgemm_codebook_from_stream(to_f64(self.inp["A"]), self.stream, c.bits, self.T64, self.S64, c.group,
                                            c.K, c.N, c.act, cols=cols)

    def gpu_w(self):
        c = self.case
        return self.B.qdequant_codebook(self.d_packed, self.d_table, self.d_scales, c.bits, ACT[c.act], c.group, c.K, c.N)

    def gpu_c(self):
        c = self.case
        return self.B.qgemm_codebook(self.d_A, self.d_packed, self.d_table, self.d_scales, c.bits, c.group, c.N)


def _case(name, M, K, N, bits, act, seed, group=128, scale_dtype="f16"):
    return WL.Case(name, M, K, N, CB, bits, group=group, act=act, scale_dtype=scale_dtype, zero=None, seed=seed)


@pytest.mark.parametrize("act,scale_dtype", [("f16", "f16"), ("bf16", "f16"), ("bf16", "bf16")])
@pytest.mark.parametrize("bits", range(1, 9))
def test_codebook_weights_dequantise_bit_exactly(bits, act, scale_dtype):
    # every code in every position of a lane's bit stream: codes cycled over a 512 x 256 weight,
    # a table with both signs, zero, the largest and the smallest normal half among its levels
    case = _case(f"cb_w_{bits}_{act}", 1, 512, 256, bits, act, 60000 + bits, group=64, scale_dtype=scale_dtype)
    inp = WL.make_inputs(case)
    inp["codes"] = ((np.arange(512)[:, None] * 7 + np.arange(256)[None, :] * 3) % (1 << bits)).astype(np.uint8)
    lv = inp["codebook"].clone()
    special = torch.tensor([0.0, -0.0, 65504.0, -6.103515625e-05, 1.0, -2.5], dtype=torch.float16)
    n = min(lv.numel(), special.numel())
    lv[:n] = special[:n]
    inp["codebook"] = lv
    P = CbCase(case, inp)
    _, wbits = P.oracle_w()
    got = bits_of(P.gpu_w())
    assert np.array_equal(got, wbits), f"{(got != wbits).sum()} weights differ"


@pytest.mark.parametrize("group", [32, 64, 128, 256, 1408])
@pytest.mark.parametrize("bits", [2, 4, 5, 8])
def test_codebook_weights_every_group_size(bits, group):
    K = 1408 if group == 1408 else 1024
    case = _case(f"cb_g_{bits}_{group}", 1, K, 192, bits, "f16", 60050 + bits + group, group=group)
    P = CbCase(case)
    _, wbits = P.oracle_w()
    assert np.array_equal(bits_of(P.gpu_w()), wbits)


@pytest.mark.parametrize("M", [1, 5, 16, 17, 40, 64, 65, 150])
@pytest.mark.parametrize("bits", [1, 3, 4, 6, 8])
def test_codebook_matmul_every_row_count(bits, M):
    # 11 chunks of K on 5 strips (ragged shares per wavefront); beyond 64 rows: blocks of 64
    case = _case(f"cb_c_{bits}_{M}", M, 1408, 320, bits, "bf16" if M % 2 else "f16", 60100 + bits + M)
    P = CbCase(case)
    plan = P.B.qg_plan(P.wtype, case.group, M, case.N, case.K)
    assert plan["path"] == (1 if M <= 64 else 2), plan
    ref = P.oracle_c()
    assert_c_close(P.gpu_c(), ref, case.name)
    P.B.qg_set_knob(0, 2)                          # the tiled kernel at every tile height, also below its usual range
    for bm in (64, 128, 256):
        P.B.qg_set_knob(2, bm)
        assert_c_close(P.gpu_c(), ref, f"{case.name} tiled {bm}")
    P.B.qg_set_knob(2, 0)
    P.B.qg_set_knob(0, 3)                          # and the streaming kernel over blocks of 64 rows
    assert_c_close(P.gpu_c(), ref, case.name + " row blocks")


@pytest.mark.parametrize("variant", [10, 11, 12, 14, 15, 16])
@pytest.mark.parametrize("bits", [2, 4, 7])
def test_codebook_matmul_every_wavefront_arrangement(bits, variant):
    case = _case(f"cb_arr_{bits}_{variant}", 9, 1408, 512, bits, "bf16", 60150 + bits)
    P = CbCase(case)
    P.B.qg_set_knob(3, variant)
    assert_c_close(P.gpu_c(), P.oracle_c(), case.name)


@pytest.mark.parametrize("M,variant", [(20, 21), (30, 26), (40, 41), (64, 46)])
@pytest.mark.parametrize("bits", [3, 8])
def test_codebook_matmul_several_row_tiles(bits, M, variant):
    case = _case(f"cb_rows_{bits}_{M}_{variant}", M, 1152, 256, bits, "f16", 60170 + M + bits)
    P = CbCase(case)
    P.B.qg_set_knob(3, variant)
    assert_c_close(P.gpu_c(), P.oracle_c(), case.name)


@pytest.mark.parametrize("group", [32, 64, 256])
@pytest.mark.parametrize("bits", [4, 5])
def test_codebook_matmul_group_sizes(bits, group):
    case = _case(f"cb_grp_{bits}_{group}", 24, 1024, 256, bits, "f16", 60190 + bits + group, group=group)
    P = CbCase(case)
    assert_c_close(P.gpu_c(), P.oracle_c(), case.name)


@pytest.mark.parametrize("splitk", [2, 3])
@pytest.mark.parametrize("bits", [4, 6])
def test_codebook_matmul_split_k(bits, splitk):
    case = _case(f"cb_sk_{bits}_{splitk}", 9, 1408, 320, bits, "f16", 60200 + bits)
    P = CbCase(case)
    ref = P.oracle_c()
    P.B.qg_set_knob(1, splitk)
    first = P.gpu_c()
    assert_c_close(first, ref, case.name)
    assert np.array_equal(bits_of(first), bits_of(P.gpu_c()))


@pytest.mark.parametrize("act", ["f16", "bf16"])
@pytest.mark.parametrize("bits", [1, 2, 3, 4, 5, 6, 7, 8])
def test_codebook_one_hot_rows_bit_exact(bits, act):
    K, N = 256, 128
    case = _case(f"cb_onehot_{bits}_{act}", 64, K, N, bits, act, 60300 + bits)
    inp = WL.make_inputs(case)
    rows = np.concatenate([np.arange(0, 40), np.arange(120, 136), np.arange(248, 256)])
    A = torch.zeros((64, K), dtype=inp["A"].dtype)
    A[torch.arange(64), torch.from_numpy(rows)] = 1.0
    inp["A"] = A
    P = CbCase(case, inp)
    _, wbits = P.oracle_w()
    want = wbits[rows].copy()
    want[want == 0x8000] = 0            # a sum of one -0 and zeros is +0
    assert np.array_equal(bits_of(P.gpu_c()), want)


@pytest.mark.parametrize("bits", [3, 4, 8])
def test_codebook_decode_shape_full_size(bits):
    # K = N = 8192, M = 16: sampled columns, then every column
    case = _case(f"cb_full_{bits}", 16, 8192, 8192, bits, "f16", 60400 + bits)
    P = CbCase(case)
    C = P.gpu_c()
    cols = np.unique(np.concatenate([np.arange(4), np.arange(8188, 8192), np.random.default_rng(bits).integers(0, 8192, 64)]))
    assert_c_close(C[:, torch.from_numpy(cols).cuda()], P.oracle_c(cols=cols), case.name + " sampled")
    assert_c_close(C, P.oracle_c(), case.name + " all columns")


def test_codebook_sweep_shape_full_size():
    # the type sweep's shape, K = 8192, N = 57344, M = 16, 4-bit codes: sampled columns
    case = WL.codebook(4)
    P = CbCase(case)
    C = P.gpu_c()
    cols = np.unique(np.concatenate([np.arange(4), np.arange(57340, 57344), np.random.default_rng(4).integers(0, 57344, 96)]))
    assert_c_close(C[:, torch.from_numpy(cols).cuda()], P.oracle_c(cols=cols), case.name)


@pytest.mark.parametrize("M,K,N", [(1, 128, 64), (64, 128, 64), (7, 256, 128)])
def test_codebook_smallest_shapes(M, K, N):
    case = _case(f"cb_tiny_{M}_{K}_{N}", M, K, N, 4, "f16", 60600 + K + N)
    P = CbCase(case)
    _, wbits = P.oracle_w()
    assert np.array_equal(bits_of(P.gpu_w()), wbits)
    assert_c_close(P.gpu_c(), P.oracle_c(), case.name)


@pytest.mark.parametrize("act", ["f16", "bf16"])
@pytest.mark.parametrize("bits", [2, 4, 6, 8])
def test_codebook_tiled_kernel_ragged_shapes_split_k_and_one_hot(bits, act):
    from paper_2504_12984_amd import binding as B
    # 7 chunks (odd: the padding chunk), 3 strips (an idle wavefront), rows past M; then K in two slabs;
    # then the de-quantise-first path
    case = _case(f"cb_tiled_{bits}_{act}", 300, 896, 192, bits, act, 60700 + bits, group=64 if bits == 4 else 128)
    P = CbCase(case)
    ref = P.oracle_c()
    assert_c_close(P.gpu_c(), ref, case.name)
    B.qg_set_knob(0, 2); B.qg_set_knob(2, 64); B.qg_set_knob(1, 2)
    assert_c_close(P.gpu_c(), ref, case.name + " split")
    B.qg_set_knob(1, 0); B.qg_set_knob(2, 0)
    B.qg_set_knob(0, 4)
    assert_c_close(P.gpu_c(), ref, case.name + " de-quantise first")
    B.qg_set_knob(0, 0)
    # one-hot rows through the tiled kernel: the de-quantised weight itself (a lone -0 sums to +0)
    K, N = 256, 128
    c2 = _case(f"cb_tiled_onehot_{bits}_{act}", K, K, N, bits, act, 60710 + bits)
    inp = WL.make_inputs(c2)
    A = torch.zeros((K, K), dtype=inp["A"].dtype)
    A[torch.arange(K), torch.arange(K)] = 1.0
    inp["A"] = A
    P2 = CbCase(c2, inp)
    _, wbits = P2.oracle_w()
    want = wbits.copy()
    want[want == 0x8000] = 0
    assert np.array_equal(bits_of(P2.gpu_c()), want)


@pytest.mark.parametrize("group", [32, 64])
def test_codebook_tiled_kernel_small_groups(group):
    case = _case(f"cb_tiled_g{group}", 200, 1024, 256, 3, "bf16", 60750 + group, group=group, scale_dtype="bf16")
    P = CbCase(case)
    assert_c_close(P.gpu_c(), P.oracle_c(), case.name)


@pytest.mark.parametrize("bits", [5, 8])
def test_codebook_wide_codes_on_many_rows_take_the_dequantise_first_path(bits):
    # chosen by the library from 1024 rows on; the same rounded weights, so the same tolerance (and one-hot rows bit for bit)
    case = _case(f"cb_auto4_{bits}", 1024, 384, 192, bits, "bf16", 60800 + bits, group=128)
    inp = WL.make_inputs(case)
    A = inp["A"].clone()
    A[:384] = 0
    A[torch.arange(384), torch.arange(384)] = 1.0
    inp["A"] = A
    P = CbCase(case, inp)
    assert P.B.qg_plan(P.wtype, case.group, case.M, case.N, case.K, act=P.B.QG_BF16)["path"] == 4
    C = P.gpu_c()
    assert_c_close(C, P.oracle_c(), case.name)
    _, wbits = P.oracle_w()
    want = wbits.copy()
    want[want == 0x8000] = 0
    assert np.array_equal(bits_of(C[:384]), want)
    P.B.qg_set_knob(0, 2)                          # the fused kernel gives the same bits on the one-hot rows
    assert np.array_equal(bits_of(P.gpu_c()[:384]), want)


def test_codebook_prefill_shape_full_size():
    # K = 8192, N = 57344 (the prefill shape), 4-bit codes, M = 1024: sampled columns for all rows
    case = WL.codebook(4, 1024)
    P = CbCase(case)
    plan = P.B.qg_plan(P.wtype, case.group, case.M, case.N, case.K)
    assert plan["path"] == 2, plan
    C = P.gpu_c()
    cols = np.unique(np.concatenate([np.arange(4), np.arange(57340, 57344), np.random.default_rng(4).integers(0, 57344, 64)]))
    assert_c_close(C[:, torch.from_numpy(cols).cuda()], P.oracle_c(cols=cols), case.name)


def test_codebook_argument_checks():
    from paper_2504_12984_amd import binding as B
    case = _case("cb_args", 4, 256, 128, 4, "f16", 60700)
    P = CbCase(case)
    # the plain calls have no table: a codebook weight type is an invalid argument there
    with pytest.raises(B.QgError) as e:
        B.qgemm(P.d_A, P.d_packed, P.d_scales, None, P.wtype, case.group, case.N)
    assert e.value.status == B.QG_EINVAL
    with pytest.raises(B.QgError) as e:
        B.qdequant(P.d_packed, P.d_scales, None, P.wtype, torch.float16, case.group, case.K, case.N)
    assert e.value.status == B.QG_EINVAL
    # the other layouts have no lookup kernels
    assert B.qgemm_packed_bytes(P.wtype, case.K, case.N, layout=B.QG_LAYOUT_TILE128x64_R32) == 0
    assert B.qgemm_packed_bytes(P.wtype, case.K, case.N, layout=B.QG_LAYOUT_TILE128x64_I8) == 0
    # bits out of range, fp16 activations with bf16 scales
    with pytest.raises(ValueError):
        B.qgemm_codebook(P.d_A, P.d_packed, P.d_table, P.d_scales, 9, case.group, case.N)
    with pytest.raises(B.QgError) as e:
        B.qgemm_codebook(P.d_A, P.d_packed, P.d_table, P.d_scales.to(torch.bfloat16), 4, case.group, case.N)
    assert e.value.status == B.QG_EUNSUPPORTED


def _random_codebook_case(seed: int) -> WL.Case:
    rng = np.random.default_rng(660000 + seed)
    bits = int(rng.integers(1, 9))
    long_k = seed % 2 == 1
    K = 128 * int(rng.integers(8, 49) if long_k else rng.integers(1, 9))
    N = 64 * int(rng.integers(1, 25))
    M = int(rng.choice([rng.integers(1, 17), rng.integers(17, 65), rng.integers(65, 257), rng.integers(257, 641),
                        rng.integers(1024, 1100)]))
    groups = [g for g in (32, 64, 128, 256, 512, K)
              if K % g == 0 and (g == K or g <= 64 or (g // 128) & (g // 128 - 1) == 0)]
    group = int(rng.choice(groups))
    act = str(rng.choice(["f16", "bf16"]))
    sdt = "f16" if act == "f16" else str(rng.choice(["f16", "bf16"]))
    return WL.Case(f"cbrand{seed}_b{bits}_M{M}_K{K}_N{N}_g{group}_{act}_{sdt}", M, K, N, CB, bits, group=group, act=act,
                   scale_dtype=sdt, zero=None, seed=661000 + seed)


@pytest.mark.parametrize("seed", range(32))
def test_codebook_random_shapes_through_the_automatic_dispatch(seed):
    # streaming kernel (every arrangement the planner picks), tiled kernel (tile heights, split-K, split launches) and,
    # for wide codes on 1024 or more rows, the de-quantise-first path -- whatever the library chooses for the shape
    case = _random_codebook_case(seed)
    P = CbCase(case)
    assert_c_close(P.gpu_c(), P.oracle_c(), case.name)

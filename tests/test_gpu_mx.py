"""GPU parity, part 8: power-of-two block scales (one 8-bit exponent per 32 rows and column --
the shared scale of the microscaling types) with e2m1 and e4m3 codes, the two element types
the hardware's scaled converts handle pair by pair.

qdequant is compared bit for bit with the oracle (value(code) * 2^(e - 127), which is exact
inside the target type's range, so any mistake in the scale's row, column or exponent shows);
qgemm within |C_gpu - C_ref| <= 1e-2 + 5e-3 |C_ref| elementwise, and bit for bit through
one-hot rows.
"""
import numpy as np
import pytest
import torch

from oracle import qgemm_oracle as O
from paper_2504_12984_amd import workloads as WL
from gpu_util import ACT, assert_c_close, bits_of, to_f64

pytestmark = pytest.mark.gpu

F = WL.KIND_FLOAT
TYPES = [(4, 2, 1), (8, 4, 3)]


@pytest.fixture(autouse=True)
def _reset_knobs():
    from paper_2504_12984_amd import binding as B
    yield
    for k in range(4):
        B.qg_set_knob(k, 0)


class MxCase:
    def __init__(self, case: WL.Case, inputs=None):
        from paper_2504_12984_amd import binding as B
        self.B, self.case = B, case
        c = case
        self.inp = inputs if inputs is not None else WL.make_inputs(c)
        assert self.inp["scales"].dtype == torch.uint8 and self.inp["zeros"] is None
        self.wtype = B.WType(c.kind, c.bits, c.ebits, c.mbits)
        self.stream = O.pack_canonical(self.inp["codes"], c.bits)
        self.S64 = O.e8m0_values(self.inp["scales"].numpy())
        self.d_scales = self.inp["scales"].cuda()
        self.d_A = self.inp["A"].cuda()
        self.d_packed = B.repack(torch.from_numpy(self.stream).cuda(), self.wtype, c.K, c.N)

    def oracle_w(self):
        c = self.case
        return O.dequant_rounded(self.inp["codes"], c.kind, c.bits, c.ebits, c.mbits, self.S64, None, 32, c.act)

    def oracle_c(self, cols=None):
        c = self.case
        return O.qgemm_from_stream(to_f64(self.inp["A"]), self.stream, c.kind, c.bits, c.ebits, c.mbits, self.S64, None,
                                   32, c.K, c.N, c.act, cols=cols)

    def gpu_w(self):
        c = self.case
        return self.B.qdequant(self.d_packed, self.d_scales, None, self.wtype, ACT[c.act], 32, c.K, c.N)

    def gpu_c(self):
        c = self.case
        return self.B.qgemm(self.d_A, self.d_packed, self.d_scales, None, self.wtype, 32, c.N)


def _case(name, M, K, N, bits, e, m, act, seed):
    return WL.Case(name, M, K, N, F, bits, e, m, group=32, act=act, scale_dtype="e8m0", zero=None, seed=seed)


@pytest.mark.parametrize("act", ["f16", "bf16"])
@pytest.mark.parametrize("bits,e,m", TYPES)
def test_block_scaled_weights_dequantise_bit_exactly(bits, e, m, act):
    # every code in every lane position: all 2^bits finite codes cycled over a 512 x 256 weight
    case = _case(f"mx_w_{bits}_{act}", 1, 512, 256, bits, e, m, act, 50000 + bits)
    inp = WL.make_inputs(case)
    fin = O.finite_codes(F, bits, e, m)
    inp["codes"] = fin[(np.arange(512)[:, None] * 7 + np.arange(256)[None, :] * 3) % fin.size].astype(np.uint8)
    P = MxCase(case, inp)
    wr, wbits = P.oracle_w()
    assert np.array_equal(wr, O.dequant_exact(inp["codes"], F, bits, e, m, P.S64, None, 32)), "exact: nothing to round"
    got = bits_of(P.gpu_w())
    assert np.array_equal(got, wbits), f"{(got != wbits).sum()} weights differ"


@pytest.mark.parametrize("M", [1, 5, 16, 17, 40, 64, 65, 150])
@pytest.mark.parametrize("bits,e,m", TYPES)
def test_block_scaled_matmul_every_row_count(bits, e, m, M):
    # 11 chunks of K on 5 strips (ragged shares per wavefront); beyond 64 rows: blocks of 64
    case = _case(f"mx_c_{bits}_{M}", M, 1408, 320, bits, e, m, "bf16" if M % 2 else "f16", 50100 + bits + M)
    P = MxCase(case)
    plan = P.B.qg_plan(P.wtype, 32, M, case.N, case.K, act=P.B.QG_F16, scale_dtype=P.B.QG_E8M0)
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
@pytest.mark.parametrize("bits,e,m", TYPES)
def test_block_scaled_matmul_every_wavefront_arrangement(bits, e, m, variant):
    case = _case(f"mx_arr_{bits}_{variant}", 9, 1408, 512, bits, e, m, "bf16", 50150 + bits)
    P = MxCase(case)
    P.B.qg_set_knob(3, variant)
    assert_c_close(P.gpu_c(), P.oracle_c(), case.name)


@pytest.mark.parametrize("M,variant", [(20, 21), (30, 26), (40, 41), (64, 46)])
def test_block_scaled_matmul_several_row_tiles(M, variant):
    case = _case(f"mx_rows_{M}_{variant}", M, 1152, 256, 8, 4, 3, "f16", 50170 + M)
    P = MxCase(case)
    P.B.qg_set_knob(3, variant)
    assert_c_close(P.gpu_c(), P.oracle_c(), case.name)


@pytest.mark.parametrize("splitk", [2, 3])
@pytest.mark.parametrize("bits,e,m", TYPES)
def test_block_scaled_matmul_split_k(bits, e, m, splitk):
    case = _case(f"mx_sk_{bits}_{splitk}", 9, 1408, 320, bits, e, m, "f16", 50200 + bits)
    P = MxCase(case)
    ref = P.oracle_c()
    P.B.qg_set_knob(1, splitk)
    first = P.gpu_c()
    assert_c_close(first, ref, case.name)
    assert np.array_equal(bits_of(first), bits_of(P.gpu_c()))


@pytest.mark.parametrize("act", ["f16", "bf16"])
@pytest.mark.parametrize("bits,e,m", TYPES)
def test_block_scaled_one_hot_rows_bit_exact(bits, e, m, act):
    K, N = 256, 128
    case = _case(f"mx_onehot_{bits}_{act}", 64, K, N, bits, e, m, act, 50300 + bits)
    inp = WL.make_inputs(case)
    rows = np.concatenate([np.arange(0, 40), np.arange(120, 136), np.arange(248, 256)])
    A = torch.zeros((64, K), dtype=inp["A"].dtype)
    A[torch.arange(64), torch.from_numpy(rows)] = 1.0
    inp["A"] = A
    P = MxCase(case, inp)
    _, wbits = P.oracle_w()
    want = wbits[rows].copy()
    want[want == 0x8000] = 0            # a sum of one -0 and zeros is +0
    assert np.array_equal(bits_of(P.gpu_c()), want)


@pytest.mark.parametrize("bits,e,m", TYPES)
def test_block_scaled_decode_shape_full_size(bits, e, m):
    # K = N = 8192 (the low-bit float configuration's shape), M = 16: sampled columns, then every column
    case = _case(f"mx_full_{bits}", 16, 8192, 8192, bits, e, m, "bf16", 50400 + bits)
    P = MxCase(case)
    C = P.gpu_c()
    cols = np.unique(np.concatenate([np.arange(4), np.arange(8188, 8192), np.random.default_rng(bits).integers(0, 8192, 64)]))
    assert_c_close(C[:, torch.from_numpy(cols).cuda()], P.oracle_c(cols=cols), case.name + " sampled")
    assert_c_close(C, P.oracle_c(), case.name + " all columns")


@pytest.mark.parametrize("M,K,N", [(1, 128, 64), (64, 128, 64), (7, 256, 128)])
def test_block_scaled_smallest_shapes(M, K, N):
    case = _case(f"mx_tiny_{M}_{K}_{N}", M, K, N, 4, 2, 1, "f16", 50600 + K + N)
    P = MxCase(case)
    _, wbits = P.oracle_w()
    assert np.array_equal(bits_of(P.gpu_w()), wbits)
    assert_c_close(P.gpu_c(), P.oracle_c(), case.name)


@pytest.mark.parametrize("act", ["f16", "bf16"])
@pytest.mark.parametrize("bits,e,m", TYPES)
def test_block_scaled_tiled_kernel_ragged_shapes_split_k_and_one_hot(bits, e, m, act):
    from paper_2504_12984_amd import binding as B
    # 7 chunks (odd: the padding chunk), 3 strips (an idle wavefront), rows past M; then K in two slabs
    case = _case(f"mx_tiled_{bits}_{act}", 300, 896, 192, bits, e, m, act, 50700 + bits)
    P = MxCase(case)
    ref = P.oracle_c()
    assert_c_close(P.gpu_c(), ref, case.name)
    B.qg_set_knob(0, 2); B.qg_set_knob(2, 64); B.qg_set_knob(1, 2)
    assert_c_close(P.gpu_c(), ref, case.name + " split")
    B.qg_set_knob(1, 0); B.qg_set_knob(2, 0)
    # one-hot rows through the tiled kernel: the de-quantised weight itself (a lone -0 sums to +0)
    K, N = 256, 128
    c2 = _case(f"mx_tiled_onehot_{bits}_{act}", K, K, N, bits, e, m, act, 50710 + bits)
    inp = WL.make_inputs(c2)
    A = torch.zeros((K, K), dtype=inp["A"].dtype)
    A[torch.arange(K), torch.arange(K)] = 1.0
    inp["A"] = A
    P2 = MxCase(c2, inp)
    _, wbits = P2.oracle_w()
    want = wbits.copy()
    want[want == 0x8000] = 0
    assert np.array_equal(bits_of(P2.gpu_c()), want)


def test_block_scaled_prefill_shape_full_size():
    # K = 8192, N = 57344 (the prefill shape), e2m1 with block scales, M = 1024: sampled columns for all rows
    case = _case("mx_prefill_f4", 1024, 8192, 57344, 4, 2, 1, "bf16", 50800)
    P = MxCase(case)
    C = P.gpu_c()
    cols = np.unique(np.concatenate([np.arange(4), np.arange(57340, 57344), np.random.default_rng(4).integers(0, 57344, 64)]))
    assert_c_close(C[:, torch.from_numpy(cols).cuda()], P.oracle_c(cols=cols), case.name)


def test_block_scales_argument_errors():
    from paper_2504_12984_amd import binding as B
    P = MxCase(_case("mx_err", 4, 128, 64, 4, 2, 1, "f16", 50500))
    s = P.d_scales
    with pytest.raises(B.QgError) as err:          # 6-bit floats: no per-pair scaled convert
        B.qgemm(P.d_A, P.d_packed, s, None, B.WType(B.QG_FLOAT, 6, 3, 2), 32, 64)
    assert err.value.status == B.QG_EUNSUPPORTED
    with pytest.raises(B.QgError) as err:          # integer codes
        B.qgemm(P.d_A, P.d_packed, s, None, B.WType(B.QG_UINT, 4), 32, 64)
    assert err.value.status == B.QG_EUNSUPPORTED
    with pytest.raises(B.QgError) as err:          # block scales mean 32 rows per scale
        B.qgemm(P.d_A, P.d_packed, s[:1].contiguous(), None, P.wtype, 128, 64)
    assert err.value.status == B.QG_EUNSUPPORTED
    with pytest.raises(B.QgError) as err:          # no zero-points with block scales
        B.qgemm(P.d_A, P.d_packed, s, torch.zeros((4, 64), dtype=torch.uint8, device="cuda"), P.wtype, 32, 64)
    assert err.value.status == B.QG_EINVAL
    B.qg_set_knob(0, 4)                            # the de-quantise-first path has no block-scaled variant
    with pytest.raises(B.QgError) as err:
        P.gpu_c()
    assert err.value.status == B.QG_EUNSUPPORTED

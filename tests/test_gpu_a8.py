"""GPU parity, part 7: int8 activations (qgemm_a8) against the oracle's int8 leg.

    C[m,n] = a_scale[m] * sum_g s[g,n] * sum_{k in g} A8[m,k] * (value(code[k,n]) - z[g,n])

Compared in full within |C_gpu - C_ref| <= 1e-2 + 5e-3 |C_ref| (the integer part is exact on
both sides; what differs is fp32 against fp64 scaling and the output rounding), and bit for
bit through one-hot rows: with a single 1 in a row of A8 and no activation scale, C[m, :] is
(q - z) * s rounded once to the output type, which is the oracle's rounded de-quantised
weight -- a bit-exact check of the third device layout and of its unpack for every code.
"""
import numpy as np
import pytest
import torch

from oracle import qgemm_oracle as O
from paper_2504_12984_amd import workloads as WL
from gpu_util import assert_c_close, bits_of, to_f64

pytestmark = pytest.mark.gpu

U, I = WL.KIND_UINT, WL.KIND_INT
ACT = {"f16": torch.float16, "bf16": torch.bfloat16}


@pytest.fixture(autouse=True)
def _reset_knobs():
    from paper_2504_12984_amd import binding as B
    yield
    for k in range(4):
        B.qg_set_knob(k, 0)


class A8Case:
    def __init__(self, case: WL.Case, inputs=None):
        from paper_2504_12984_amd import binding as B
        self.B, self.case = B, case
        c = case
        self.inp = inputs if inputs is not None else WL.make_inputs(c)
        self.wtype = B.WType(c.kind, c.bits)
        self.stream = O.pack_canonical(self.inp["codes"], c.bits)
        self.S64 = to_f64(self.inp["scales"])
        self.d_A = self.inp["A"].cuda()
        self.d_as = None if self.inp.get("a_scale") is None else self.inp["a_scale"].cuda()
        self.d_scales = self.inp["scales"].cuda()
        self.d_zeros = None if self.inp["zeros"] is None else torch.from_numpy(self.inp["zeros"]).cuda()
        self.d_packed = B.repack(torch.from_numpy(self.stream).cuda(), self.wtype, c.K, c.N,
                                 layout=B.QG_LAYOUT_TILE128x64_I8)

    def gpu(self):
        c = self.case
        return self.B.qgemm_a8(self.d_A, self.d_as, self.d_packed, self.d_scales, self.d_zeros, self.wtype, c.group, c.N,
                               out_dtype=ACT[c.act])

    def ref(self, cols=None, rows=None):
        c = self.case
        A8 = self.inp["A"].numpy()
        a_s = None if self.inp.get("a_scale") is None else self.inp["a_scale"].numpy()
        if rows is not None:
            A8, a_s = A8[rows], (None if a_s is None else a_s[rows])
        return O.qgemm_int8_from_stream(A8, a_s, self.stream, c.kind, c.bits, self.S64, self.inp["zeros"], c.group,
                                        c.K, c.N, cols=cols)


def _case(name, M, K, N, kind, bits, group, act="f16", sdt=None, zero="random", zero_hi=None, seed=0):
    return WL.Case(name, M, K, N, kind, bits, group=group, act=act, scale_dtype=sdt or ("f16" if act == "f16" else "bf16"),
                   zero=zero, zero_hi=zero_hi, a8=True, seed=seed)


@pytest.mark.parametrize("act", ["f16", "bf16"])
@pytest.mark.parametrize("bits", range(1, 9))
@pytest.mark.parametrize("kind", [U, I])
def test_one_hot_rows_give_the_rounded_weight_bit_for_bit(kind, bits, act):
    # M = K rows of the identity (four blocks of 64 rows, two chunks of K, three strips)
    K, N = 256, 192
    case = _case(f"a8_onehot_{kind}_{bits}_{act}", K, K, N, kind, bits, 64 if bits % 2 else 128, act=act, sdt="f16",
                 zero="random", zero_hi=255 if bits in (2, 8) else None, seed=40000 + bits)
    inp = WL.make_inputs(case)
    A = torch.zeros((K, K), dtype=torch.int8)
    A[torch.arange(K), torch.arange(K)] = 1
    inp["A"], inp["a_scale"] = A, None
    P = A8Case(case, inp)
    _, wbits = O.dequant_rounded(inp["codes"], kind, bits, 0, 0, P.S64, inp["zeros"], case.group, act)
    assert np.array_equal(bits_of(P.gpu()), wbits)


@pytest.mark.parametrize("M", [1, 7, 16, 17, 32, 33, 64, 65, 200])
@pytest.mark.parametrize("kind,bits,group", [(U, 4, 128), (I, 3, 64), (U, 8, 256), (I, 8, 1408), (U, 1, 128), (U, 6, 64)])
def test_every_row_count_against_the_oracle(M, kind, bits, group):
    K = 1408 if group != 256 else 1536                 # 11 (12) chunks: ragged shares per wavefront
    case = _case(f"a8_{M}_{kind}_{bits}_{group}", M, K, 320, kind, bits, group, act="f16" if M % 2 else "bf16",
                 zero="random" if kind == U else None, seed=40100 + M + bits)
    P = A8Case(case)
    assert_c_close(P.gpu(), P.ref(), case.name)


@pytest.mark.parametrize("splitk", [2, 3, 11])
@pytest.mark.parametrize("M", [5, 30, 64, 100])
def test_split_k_and_repeat_calls(M, splitk):
    from paper_2504_12984_amd import binding as B
    case = _case(f"a8_splitk_{M}_{splitk}", M, 1408, 320, I, 5, 128, zero="random", zero_hi=7, seed=40300 + M)
    P = A8Case(case)
    ref = P.ref()
    B.qg_set_knob(1, splitk)
    first = P.gpu()
    assert_c_close(first, ref, case.name)
    assert np.array_equal(bits_of(first), bits_of(P.gpu()))


def test_long_k_splits_by_itself_and_different_inputs_follow_each_other():
    X = A8Case(_case("a8_X", 16, 8192, 2048, U, 4, 128, seed=40400))
    Y = A8Case(_case("a8_Y", 16, 8192, 2048, U, 4, 128, seed=40401))
    rx, ry = X.ref(), Y.ref()
    outs = [X.gpu(), Y.gpu(), X.gpu()]
    torch.cuda.synchronize()
    assert_c_close(outs[0], rx, "X"); assert_c_close(outs[1], ry, "Y"); assert_c_close(outs[2], rx, "X again")
    assert np.array_equal(bits_of(outs[0]), bits_of(outs[2]))


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_signed_sweep_shape_full_size(bits):
    # K = 8192, N = 28672, M = 16 (the signed bit-width sweep's shape) with int8 activations:
    # sampled columns for a first check, then every column
    case = WL.shrink(WL.cfg3(bits), a8=True, name=f"a8_cfg3_i{bits}")
    P = A8Case(case)
    C = P.gpu()
    cols = np.unique(np.concatenate([np.arange(4), np.arange(case.N - 4, case.N),
                                     np.random.default_rng(bits).integers(0, case.N, size=64)]))
    assert_c_close(C[:, torch.from_numpy(cols).cuda()], P.ref(cols=cols), case.name + " sampled")
    assert_c_close(C, P.ref(), case.name + " all columns")


@pytest.mark.parametrize("act,sdt", [("f16", "bf16"), ("bf16", "f16"), ("f16", "f16"), ("bf16", "bf16")])
@pytest.mark.parametrize("M,K,N", [(1, 128, 64), (64, 128, 64), (3, 256, 128), (0, 128, 64)])
def test_smallest_shapes_and_every_output_scale_type_pair(M, K, N, act, sdt):
    # one chunk, one strip; the output type and the scale type are independent of each other
    case = _case(f"a8_tiny_{M}_{K}_{N}_{act}_{sdt}", max(M, 1), K, N, U, 4, 64, act=act, sdt=sdt, seed=40600 + K + N)
    P = A8Case(case)
    if M == 0:
        A0 = torch.empty((0, K), dtype=torch.int8, device="cuda")
        out = P.B.qgemm_a8(A0, None, P.d_packed, P.d_scales, P.d_zeros, P.wtype, 64, N, out_dtype=ACT[act])
        assert out.shape == (0, N)
        return
    assert_c_close(P.gpu(), P.ref(), case.name)


def test_argument_errors():
    from paper_2504_12984_amd import binding as B
    P = A8Case(_case("a8_err", 4, 128, 64, U, 4, 128, seed=40500))
    with pytest.raises(B.QgError) as e:                  # float weights have no integer instruction
        B.qgemm_a8(P.d_A, None, P.d_packed, P.d_scales, None, B.WType(B.QG_FLOAT, 4, 2, 1), 128, 64)
    assert e.value.status == B.QG_EUNSUPPORTED
    with pytest.raises(B.QgError) as e:                  # group 32: the instruction sums 64 values of k
        s = torch.ones((4, 64), dtype=torch.float16, device="cuda")
        B.qgemm_a8(P.d_A, None, P.d_packed, s, None, P.wtype, 32, 64)
    assert e.value.status == B.QG_EUNSUPPORTED
    assert B.qgemm_packed_bytes(B.WType(B.QG_FLOAT, 4, 2, 1), 128, 64, layout=B.QG_LAYOUT_TILE128x64_I8) == 0
    assert B.qgemm_packed_bytes(P.wtype, 128, 64, layout=B.QG_LAYOUT_TILE128x64_I8) == 128 * 64 // 2

"""GPU parity, part 3: the five named configurations at their FULL sizes, in the
launch configuration bench.py times (library defaults, no knobs).

The oracle cannot produce 10^8..10^9 outputs in seconds, so each case checks
  * the de-quantised weights bit for bit on a seeded sample of columns (all K
    rows of each sampled column), and
  * the matmul within |C_gpu - C_ref| <= 1e-2 + 5e-3 |C_ref| on the same sampled
    columns, for ALL M rows (each output column depends on one weight column
    only, so a sampled column is checked exactly as in a full comparison).
Weights of one (config, type) are drawn once and shared by its M values; A is
drawn per M from that case's own seed.

The other cut -- ALL N columns on a subset of rows (rows of C are independent, so
a row is checked exactly as in a full comparison) -- covers every workgroup, every
64-column strip, every L2 panel and both launches of a split tiled call: all rows
for the decode-sized configurations, 64 seeded rows of each M for the prefill one.
"""
import numpy as np
import pytest
import torch

from oracle import qgemm_oracle as O
from paper_2504_12984_amd import workloads as WL
from gpu_util import ACT, bits_of, to_f64

pytestmark = pytest.mark.gpu
NSAMPLE = 96


class FullCase:
    def __init__(self, case: WL.Case, layout: int = 0):
        from paper_2504_12984_amd import binding as B
        self.B = B
        self.layout = layout
        self.case = c = case
        self.inp = WL.make_inputs(c)
        self.wtype = B.WType(c.kind, c.bits, c.ebits, c.mbits)
        self.stream = O.pack_canonical(self.inp["codes"], c.bits)
        rng = np.random.default_rng(c.seed + 12345)
        # sampled columns: the first and last strips plus random ones
        self.cols = np.unique(np.concatenate([np.arange(4), np.arange(c.N - 4, c.N),
                                              rng.integers(0, c.N, size=NSAMPLE)]))
        self.S64 = to_f64(self.inp["scales"])
        self.d_scales = self.inp["scales"].cuda()
        self.d_zeros = None if self.inp["zeros"] is None else torch.from_numpy(self.inp["zeros"]).cuda()
        d_stream = torch.from_numpy(self.stream).cuda()
        self.d_packed = B.repack(d_stream, self.wtype, c.K, c.N, layout=layout)
        del d_stream
        self.d_cols = torch.from_numpy(self.cols).cuda()

    def oracle_w_cols(self):
        c = self.case
        rows = np.arange(c.K, dtype=np.int64)[:, None] * c.N
        codes = O.unpack_elements(self.stream, c.bits, rows + self.cols[None, :])
        assert np.array_equal(codes, self.inp["codes"][:, self.cols])          # canonical stream round trip
        z = None if self.inp["zeros"] is None else self.inp["zeros"][:, self.cols]
        return O.dequant_rounded(codes, c.kind, c.bits, c.ebits, c.mbits, self.S64[:, self.cols], z, c.group, c.act)

    def check_weights(self):
        c = self.case
        W = self.B.qdequant(self.d_packed, self.d_scales, self.d_zeros, self.wtype, ACT[c.act], c.group, c.K, c.N,
                            layout=self.layout)
        got = bits_of(W[:, self.d_cols])
        del W
        wr, want = self.oracle_w_cols()
        assert np.array_equal(got, want), f"{c.name}: {(got != want).sum()} sampled weights differ"
        return wr

    def check_gemm(self, A: torch.Tensor, wr: np.ndarray, tag: str):
        c = self.case
        C = self.B.qgemm(A.cuda(), self.d_packed, self.d_scales, self.d_zeros, self.wtype, c.group, c.N,
                         layout=self.layout)
        got = to_f64(C[:, self.d_cols])
        ref = O.gemm_fp64(to_f64(A), wr)
        ok = O.within_tolerance(got, ref)
        assert ok.all(), f"{tag}: {(~ok).sum()} of {ok.size} sampled outputs outside tolerance"


    def check_gemm_all_columns(self, runs, tag: str, layouts=(0,)):
        """runs: list of (A [M, K] torch, rows to compare); one oracle pass over all N columns
        serves every run (their compared rows are stacked), each layout is then compared with it."""
        c = self.case
        stacked = np.concatenate([to_f64(A)[rows] for A, rows in runs], axis=0)
        ref = O.qgemm_from_stream(stacked, self.stream, c.kind, c.bits, c.ebits, c.mbits, self.S64, self.inp["zeros"],
                                  c.group, c.K, c.N, c.act)
        for layout in layouts:
            packed = self.d_packed if layout == self.layout else \
                self.B.repack(torch.from_numpy(self.stream).cuda(), self.wtype, c.K, c.N, layout=layout)
            at = 0
            for A, rows in runs:
                C = self.B.qgemm(A.cuda(), packed, self.d_scales, self.d_zeros, self.wtype, c.group, c.N, layout=layout)
                got = to_f64(C[torch.from_numpy(rows).cuda()])
                del C
                ok = O.within_tolerance(got, ref[at:at + rows.size])
                assert ok.all(), (f"{tag} M={A.shape[0]} layout {layout}: {(~ok).sum()} of {ok.size} outputs outside "
                                  f"tolerance, first at row {rows[np.argwhere(~ok)[0][0]]} column {np.argwhere(~ok)[0][1]}")
                at += rows.size
            del packed


def _seeded_rows(M: int, count: int, seed: int) -> np.ndarray:
    """`count` distinct rows of 0..M-1: the first and last, the two sides of the 256-row tile
    boundaries nearest the middle, and seeded random ones."""
    if M <= count:
        return np.arange(M)
    fixed = np.array([0, 1, M - 1, M - 2, 255, 256, (M // 512) * 256 - 1, (M // 512) * 256])
    rng = np.random.default_rng(seed)
    rows = np.unique(np.concatenate([fixed, rng.choice(M, size=count, replace=False)]))
    keep = np.concatenate([fixed, np.setdiff1d(rows, fixed)])[:count]
    return np.sort(np.unique(keep))


def test_config2_w3a16_decode_all_columns():
    f = FullCase(WL.cfg2(1))
    f.check_gemm_all_columns([(_A_of(WL.cfg2(M)), np.arange(M)) for M in (1, 4, 16)], "cfg2 all columns")


@pytest.mark.parametrize("bits", [1, 3, 4, 8])
def test_config3_signed_all_columns(bits):
    f = FullCase(WL.cfg3(bits))
    f.check_gemm_all_columns([(f.inp["A"], np.arange(16))], f"cfg3 int{bits} all columns")


def test_config4_e3m2_all_columns():
    f = FullCase(WL.cfg4(6, 1))
    f.check_gemm_all_columns([(_A_of(WL.cfg4(6, M)), np.arange(M)) for M in (1, 16, 64)], "cfg4 e3m2 all columns")


def test_config5_prefill_u6_all_columns_on_64_rows_both_layouts():
    f = FullCase(WL.cfg5(6, 1024))
    runs = [(_A_of(WL.cfg5(6, M)), _seeded_rows(M, 64, 5600 + M)) for M in (1024, 4096)]
    assert all(r.size == 64 for _, r in runs)
    f.check_gemm_all_columns(runs, "cfg5 u6 all columns", layouts=(0, 1))


def test_config5_prefill_u5_all_columns_on_64_rows():
    f = FullCase(WL.cfg5(5, 1024))
    runs = [(_A_of(WL.cfg5(5, M)), _seeded_rows(M, 64, 5500 + M)) for M in (1024, 4096)]
    f.check_gemm_all_columns(runs, "cfg5 u5 all columns")


def test_config2_w3a16_decode_full():
    f = FullCase(WL.cfg2(1))
    wr = f.check_weights()
    for M in (1, 4, 16):
        f.check_gemm(_A_of(WL.cfg2(M)), wr, f"cfg2 M={M}")


def _A_of(case: WL.Case) -> torch.Tensor:
    """A of a case without drawing its weights: A is the first draw of the seed."""
    rng = np.random.Generator(np.random.PCG64(case.seed))
    A = torch.from_numpy(rng.standard_normal((case.M, case.K), dtype=np.float32))
    return A.to(ACT[case.act])


@pytest.mark.parametrize("bits", range(1, 9))
def test_config3_signed_sweep_full(bits):
    f = FullCase(WL.cfg3(bits))
    wr = f.check_weights()
    f.check_gemm(f.inp["A"], wr, f"cfg3 int{bits}")


@pytest.mark.parametrize("bits", [4, 6, 8])
def test_config4_low_bit_floats_full(bits):
    f = FullCase(WL.cfg4(bits, 1))
    wr = f.check_weights()
    for M in (1, 16, 64):
        f.check_gemm(_A_of(WL.cfg4(bits, M)), wr, f"cfg4 f{bits} M={M}")


@pytest.mark.parametrize("bits", [3, 8])
def test_config3_shape_at_33_to_64_rows_full(bits):
    # K = 8192, N = 28672 with 40 and 64 rows: the tiled kernel on 64-row tiles with K split in
    # two, which the library prefers to the streaming kernel there
    f = FullCase(WL.cfg3(bits))
    wr = f.check_weights()
    for M in (40, 64):
        plan = f.B.qg_plan(f.wtype, f.case.group, M, f.case.N, f.case.K)
        assert (plan["path"], plan["row_tile"]) == (2, 64), plan
        f.check_gemm(_A_of(WL.shrink(WL.cfg3(bits), M=M, name=f"cfg3_i{bits}_M{M}")), wr, f"cfg3 int{bits} M={M}")


@pytest.mark.parametrize("bits", [4, 6])
def test_config4_shape_at_moderate_m_full(bits):
    # K = N = 8192 with 128 / 256 / 512 rows: the shapes on which the tiled kernel splits K
    # (64- and 128-row tiles, 2 and 4 slabs), as the library chooses them
    f = FullCase(WL.cfg4(bits, 1))
    wr = f.check_weights()
    for M in (128, 256, 512):
        plan = f.B.qg_plan(f.wtype, f.case.group, M, f.case.N, f.case.K, act=f.B.QG_BF16, scale_dtype=f.B.QG_F16)
        assert plan["path"] == 2 and plan["splitk"] > 1, plan
        f.check_gemm(_A_of(WL.cfg4(bits, M)), wr, f"cfg4 f{bits} M={M}")


@pytest.mark.parametrize("bits", [5, 6])
def test_config5_prefill_full(bits):
    f = FullCase(WL.cfg5(bits, 1024))
    wr = f.check_weights()
    for M in (1024, 4096):
        f.check_gemm(_A_of(WL.cfg5(bits, M)), wr, f"cfg5 u{bits} M={M}")


def test_config5_prefill_full_on_the_second_layout():
    f = FullCase(WL.cfg5(6, 1024), layout=1)
    wr = f.check_weights()
    for M in (1024, 4096):
        f.check_gemm(_A_of(WL.cfg5(6, M)), wr, f"cfg5 u6 M={M} layout 1")


SWEEP = ([(WL.KIND_UINT, b) for b in range(1, 9)] + [(WL.KIND_INT, b) for b in range(2, 9)] +
         [(WL.KIND_FLOAT, b) for b in range(3, 9)])


@pytest.mark.parametrize("kind,bits", SWEEP)
def test_type_sweep_shapes_full(kind, bits):
    # the paper's full type sweep at its shape (M = 16, K = 8192, N = 57344): uint1..8, int2..8 and
    # the representative float of every width from 3 to 8 bits
    f = FullCase(WL.sweep(kind, bits))
    wr = f.check_weights()
    f.check_gemm(f.inp["A"], wr, f.case.name)


@pytest.mark.parametrize("kind,bits", [(WL.KIND_UINT, 4), (WL.KIND_FLOAT, 6)])
def test_batch_size_axis_full(kind, bits):
    # the paper's batch-size sweep (its figure of speedup over batch sizes: decode 1, 4, 8, 16 and
    # prefill 4096, 8192, 12288 on K = 8192, N = 57344 with u4 and f6 weights): the sizes the five
    # configurations do not have -- 8, 8192 and 12288 rows -- each on sampled columns for all rows
    # and on all columns for 64 seeded rows
    f = FullCase(WL.sweep(kind, bits))
    wr = f.check_weights()
    runs = []
    for M in (8, 8192, 12288):
        case = WL.shrink(WL.sweep(kind, bits, M), seed=WL.sweep(kind, bits).seed + M)
        A = _A_of(case)
        f.check_gemm(A, wr, case.name)
        runs.append((A, _seeded_rows(M, 64, 7000 + M)))
    f.check_gemm_all_columns(runs, f"batch sizes {f.case.wname}")


def test_generator_draw_order_gives_A_first():
    c = WL.cfg2(4)
    assert torch.equal(_A_of(c), WL.make_inputs(WL.shrink(c, N=64))["A"])
